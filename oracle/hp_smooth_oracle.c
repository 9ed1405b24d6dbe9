/*
 * CPU oracle for the optional smoothing of the upsampled confidence maps.
 *
 * TEST INFRASTRUCTURE ONLY.  It shares no code with the HIP library and must
 * never be called from the product path.
 *
 * The paper's post-processing operator (Section 2.2.1, operator 4) is given
 * without its arithmetic; implementations of the PAF family it names (Section
 * 2.3) commonly smooth the upsampled confidence maps with a small Gaussian
 * before the peak search.  This build offers that as a separate, optional
 * step, read as follows:
 *   G1 each map is correlated with an odd-length vector of taps along x and
 *      then along y (a separable filter); the caller supplies the taps (the
 *      tests use a sampled Gaussian normalised to sum 1);
 *   G2 beyond the borders the edge pixel is repeated;
 *   G3 fp32 arithmetic, horizontal pass first:
 *        t[y][x]   = sum_i taps[i] * src[y][clamp(x + i - r)]
 *        dst[y][x] = sum_j taps[j] * t[clamp(y + j - r)][x],   r = (n_taps - 1) / 2,
 *      each sum accumulated from 0 in ascending tap order, one fused
 *      multiply-add per tap.
 *
 * Parity pins (tests/test_oracle_smooth.py): a library separable correlation
 * with edge replication (scipy.ndimage.correlate1d, mode "nearest") in
 * float64, the impulse response (outer product of the taps), constants kept
 * when the taps sum to 1, a single tap of 1 as the identity, shifted impulses
 * at the borders, and separability against a direct 2-D sum.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>

static int hps_clamp(int v, int n) { return v < 0 ? 0 : (v >= n ? n - 1 : v); }

/* src, dst: [planes][H][W]; taps: n_taps (odd) values.  Returns 0, or -1 when out of memory. */
int hps_smooth(const float *src, float *dst, int planes, int H, int W, const float *taps, int n_taps)
{
    const int r = (n_taps - 1) / 2;
    float *t = (float *)malloc(sizeof(float) * (size_t)H * W);
    if (!t) return -1;
    for (int p = 0; p < planes; ++p) {
        const float *s = src + (size_t)p * H * W;
        float *d = dst + (size_t)p * H * W;
        for (int y = 0; y < H; ++y)
            for (int x = 0; x < W; ++x) {
                float acc = 0.0f;
                for (int i = 0; i < n_taps; ++i) acc = fmaf(taps[i], s[(size_t)y * W + hps_clamp(x + i - r, W)], acc);
                t[(size_t)y * W + x] = acc;
            }
        for (int y = 0; y < H; ++y)
            for (int x = 0; x < W; ++x) {
                float acc = 0.0f;
                for (int j = 0; j < n_taps; ++j) acc = fmaf(taps[j], t[(size_t)hps_clamp(y + j - r, H) * W + x], acc);
                d[(size_t)y * W + x] = acc;
            }
    }
    free(t);
    return 0;
}
