/*
 * CPU oracle for the optional sub-pixel refinement of peak positions.
 *
 * TEST INFRASTRUCTURE ONLY.  It shares no code with the HIP library and must
 * never be called from the product path.
 *
 * The paper's operator is given without arithmetic (Section 2.2.1, operator
 * 4); its peaks are whole pixels here (reading P4).  As an optional step after
 * the peak search, a peak can be moved to the vertex of the parabola through
 * its value and its two neighbours' values, per axis:
 *   F1 along x, with a = u(x-1, y), b = u(x, y), c = u(x+1, y):
 *        den = (a + c) - (b + b),  off = (0.5f * (a - c)) / den   (fp32, IEEE divide),
 *      taken only when den < 0 (a strict maximum of the parabola) and clamped
 *      to [-0.5, 0.5]; otherwise, and on the first and last column, off = 0;
 *      xf = (float)x + off.  The same along y with the neighbours above and below.
 *   F2 the map is the one the peaks were found on (smoothed or not).
 *
 * Parity pins (tests/test_oracle_refine.py): samples of a parabola give its
 * vertex, symmetric neighbourhoods give no offset, plateaus and borders give
 * none, a sampled Gaussian gives its centre within the interpolation's known
 * error, and offsets stay within half a pixel.
 */
#include <stddef.h>
#include <stdint.h>

static float hpf_axis(float a, float b, float c)
{
    const float den = (a + c) - (b + b);
    if (!(den < 0.0f)) return 0.0f;
    float off = (0.5f * (a - c)) / den;
    if (off < -0.5f) off = -0.5f;
    if (off > 0.5f) off = 0.5f;
    return off;
}

/* u: one plane [H][W]; n peaks at (px, py); writes xf, yf. */
void hpf_refine(const float *u, int H, int W, int n, const int32_t *px, const int32_t *py, float *xf, float *yf)
{
    for (int k = 0; k < n; ++k) {
        const int x = px[k], y = py[k];
        const float b = u[(size_t)y * W + x];
        float ox = 0.0f, oy = 0.0f;
        if (x > 0 && x < W - 1) ox = hpf_axis(u[(size_t)y * W + x - 1], b, u[(size_t)y * W + x + 1]);
        if (y > 0 && y < H - 1) oy = hpf_axis(u[(size_t)(y - 1) * W + x], b, u[(size_t)(y + 1) * W + x]);
        xf[k] = (float)x + ox;
        yf[k] = (float)y + oy;
    }
}
