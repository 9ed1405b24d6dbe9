/*
 * CPU oracle for the pre-processing operator.
 *
 * TEST INFRASTRUCTURE ONLY.  The slow, plain statement of what operator 2 of
 * the paper's inference dataflow computes (Section 2.2.1: decoded images are
 * resized and switched to the channel-first layout the network expects;
 * Section 2.2 lists "resizing and data layout switching" as the
 * pre-processing).  It shares no code with the HIP library and must never be
 * called from the product path.
 *
 * The paper names the two steps but none of their arithmetic (its imaging
 * operations are delegated to an imaging library, Section 2.3), so the rules
 * are this build's reading, written out step by step:
 *   Q1 decoded images are 8-bit, interleaved (height, width, channel);
 *   Q2 resizing is bilinear with half-pixel centres: output index X samples
 *      the source at (X + 1/2) * Ws / Wd - 1/2, clamped at the borders.  The
 *      cell and the weight come from integers: num = (2X + 1) Ws - Wd,
 *      den = 2 Wd, x0 = floor(num / den) (0 with weight 0 when num < 0),
 *      f = (float)(num mod den) / (float)den (one rounded division),
 *      x1 = min(x0 + 1, Ws - 1);
 *   Q3 fp32 arithmetic on the 0..255 values, horizontal pass first:
 *      r = fma(f, v[x1], (1 - f) * v[x0]) on the two source rows, then the same
 *      form vertically (1 - f is a rounded subtraction);
 *   Q4 output channel c reads input channel c, or C - 1 - c when the colour
 *      order is reversed, and is written channel-first as
 *      fma(alpha[c], u, beta[c]) (scaling / mean-std normalisation folded into
 *      two constants per output channel).
 *
 * Parity pins (tests/test_oracle_preprocess.py): a library bilinear resize
 * (torch, align_corners=False) on the same values, identity size = exact copy,
 * constants, affine ramps in closed form, hand-derived values for 2x
 * enlargement and 2x reduction, layout and channel order on per-channel
 * constants.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

static void hpq_axis(int X, int ns, int nd, int *i0, int *i1, float *f)
{
    long long num = (long long)(2 * X + 1) * ns - nd;
    long long den = 2LL * nd;
    if (num < 0) {
        *i0 = 0;
        *f = 0.0f;
    } else {
        *i0 = (int)(num / den);
        *f = (float)(num % den) / (float)den;
    }
    *i1 = (*i0 + 1 < ns) ? *i0 + 1 : ns - 1;
}

/* src uint8 [N][Hs][Ws][C] -> dst fp32 [N][C][Hd][Wd]. */
void hpq_preprocess(const uint8_t *src, int N, int Hs, int Ws, int C, int Hd, int Wd,
                    int reverse_channels, const float *alpha, const float *beta, float *dst)
{
    for (int n = 0; n < N; ++n) {
        const uint8_t *im = src + (size_t)n * Hs * Ws * C;
        for (int c = 0; c < C; ++c) {
            int cs = reverse_channels ? C - 1 - c : c;
            float *out = dst + ((size_t)n * C + c) * Hd * Wd;
            for (int Y = 0; Y < Hd; ++Y) {
                int y0, y1;
                float g;
                hpq_axis(Y, Hs, Hd, &y0, &y1, &g);
                for (int X = 0; X < Wd; ++X) {
                    int x0, x1;
                    float f;
                    hpq_axis(X, Ws, Wd, &x0, &x1, &f);
                    float v00 = (float)im[((size_t)y0 * Ws + x0) * C + cs];
                    float v01 = (float)im[((size_t)y0 * Ws + x1) * C + cs];
                    float v10 = (float)im[((size_t)y1 * Ws + x0) * C + cs];
                    float v11 = (float)im[((size_t)y1 * Ws + x1) * C + cs];
                    float r0 = fmaf(f, v01, (1.0f - f) * v00);
                    float r1 = fmaf(f, v11, (1.0f - f) * v10);
                    float u = fmaf(g, r1, (1.0f - g) * r0);
                    out[(size_t)Y * Wd + X] = fmaf(alpha[c], u, beta[c]);
                }
            }
        }
    }
}
