// Pre-processing operator of the paper's inference dataflow (Section 2.2.1, operator 2:
// decoded images are resized and switched to the channel-first layout the network expects).
// Arithmetic as stated at hp_preprocess in hp.h.
//
// The kernel is written from the output: a thread produces 4 consecutive pixels of kPreRows
// consecutive rows for all channels, so every store is one 16-byte (fp32) or 8-byte (fp16)
// piece of a row that the wavefront completes to a contiguous kilobyte, and the interleaved
// source pixel is read once for all its channels, as one 32-bit word where the layout allows.
// The column cells and weights are computed once per thread and serve all its rows (measured
// for 64 frames 640x360 -> 656x368: 1 row per thread 44.7 us, 2 rows 45.8, 4 rows 49.8, 8 rows 56.3).
#include <type_traits>

#include "hp_dev.h"

namespace hp {

constexpr int kPreRows = 1;       // rows per thread
constexpr int kPreThreads = 512;   // most threads of a workgroup: (column groups of a row) x (row groups)

struct PreParams {
    float alpha[4], beta[4];
    int Hs, Ws, Hd, Wd, N;
    float rden_x, rden_y;         // 1 / (2 Wd), 1 / (2 Hd)
    int step_qx, step_rx;         // 2 Ws = step_qx * (2 Wd) + step_rx: what one output column adds to num
    int step_qy, step_ry;
};

// Position of output index X along an axis of ns source nodes resized to nd, as the floored
// quotient q and remainder r of num = (2X + 1) ns - nd over den = 2 nd (num >= -den, so q >= -1).
// The quotient is estimated through the reciprocal and made exact: num < 2^31 and q < 2^15 keep
// the estimate within one of the truth.
__device__ __forceinline__ void pre_axis_first(int X, int ns, int nd, float rden, int &q, int &r)
{
    const int num = (2 * X + 1) * ns - nd, den = 2 * nd;
    q = (int)floorf((float)num * rden);
    r = num - q * den;
    if (r < 0) { --q; r += den; }
    if (r < 0) { --q; r += den; }
    if (r >= den) { ++q; r -= den; }
    if (r >= den) { ++q; r -= den; }
}

// The next output index: num grows by 2 ns = step_q * den + step_r.
__device__ __forceinline__ void pre_axis_next(int den, int step_q, int step_r, int &q, int &r)
{
    q += step_q;
    r += step_r;
    if (r >= den) { ++q; r -= den; }
}

// Lower node, upper node and weight from (q, r): left of node 0 the sample is clamped onto it
// (the upper clamp of i0 only matters for the padding positions past the last output index).
__device__ __forceinline__ void pre_cell(int q, int r, int den, int ns, int &i0, int &i1, float &f)
{
    i0 = min(max(q, 0), ns - 1);
    f = q < 0 ? 0.0f : (float)r / (float)den;
    i1 = min(i0 + 1, ns - 1);
}

// The C bytes of the source pixel at byte offset `at` of an image as the low bytes of a word.
// TAIL: the image is the tensor's last one, whose last pixel (at == last_at) has only three
// bytes left to read: it is read one byte early.
template <int C, bool TAIL>
__device__ __forceinline__ uint32_t load_px(const uint8_t *__restrict__ img, unsigned at, unsigned last_at)
{
    if (C == 4) return *reinterpret_cast<const uint32_t *>(img + at);
    if (C == 1) return img[at];
    if (C == 2) {
        struct __attribute__((packed)) U16 { uint16_t v; };
        return reinterpret_cast<const U16 *>(img + at)->v;
    }
    struct __attribute__((packed)) U32 { uint32_t v; };
    if (TAIL) {
        if (last_at == 0) return (uint32_t)img[0] | ((uint32_t)img[1] << 8) | ((uint32_t)img[2] << 16);   // one-pixel tensor
        const unsigned from = at == last_at ? at - 1 : at;
        const uint32_t v = reinterpret_cast<const U32 *>(img + from)->v;
        return from == at ? v : v >> 8;
    }
    return reinterpret_cast<const U32 *>(img + at)->v;
}

template <int K>
__device__ __forceinline__ float byte_of(uint32_t v)
{
    return (float)((v >> (8 * K)) & 0xffu);
}

template <int C, typename OUT, bool VEC, bool REVERSE, bool TAIL>
__device__ __forceinline__ void pre_rows(const uint8_t *__restrict__ img, OUT *__restrict__ out, const PreParams &p, int X0,
                                         int Yb)
{
    const int nx = min(4, p.Wd - X0);
    const int denx = 2 * p.Wd, deny = 2 * p.Hd;
    unsigned ox0[4], ox1[4];          // byte offsets of the two nodes within a source row
    float f[4];
    {
        int q, r;
        pre_axis_first(X0, p.Ws, p.Wd, p.rden_x, q, r);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            int i0, i1;
            pre_cell(q, r, denx, p.Ws, i0, i1, f[k]);
            ox0[k] = (unsigned)(C * i0);
            ox1[k] = (unsigned)(C * i1);
            pre_axis_next(denx, p.step_qx, p.step_rx, q, r);
        }
    }
    const unsigned last_at = (unsigned)(C * (p.Hs * p.Ws - 1));
    const size_t plane = (size_t)p.Hd * p.Wd;
    int qy, ry;
    pre_axis_first(Yb, p.Hs, p.Hd, p.rden_y, qy, ry);
#pragma unroll
    for (int r = 0; r < kPreRows; ++r) {
        const int Y = Yb + r;
        int y0, y1;
        float g;
        pre_cell(qy, ry, deny, p.Hs, y0, y1, g);
        pre_axis_next(deny, p.step_qy, p.step_ry, qy, ry);
        if (Y < p.Hd) {
            const unsigned row0 = (unsigned)(C * p.Ws) * (unsigned)y0, row1 = (unsigned)(C * p.Ws) * (unsigned)y1;
            uint32_t v00[4], v01[4], v10[4], v11[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                v00[k] = load_px<C, TAIL>(img, row0 + ox0[k], last_at);
                v01[k] = load_px<C, TAIL>(img, row0 + ox1[k], last_at);
                v10[k] = load_px<C, TAIL>(img, row1 + ox0[k], last_at);
                v11[k] = load_px<C, TAIL>(img, row1 + ox1[k], last_at);
            }
            const float g1 = 1.0f - g;
            auto channel = [&](auto cs_tag, int c) {
                constexpr int CS = decltype(cs_tag)::value;
                float o[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float f1 = 1.0f - f[k];
                    const float r0 = __fmaf_rn(f[k], byte_of<CS>(v01[k]), f1 * byte_of<CS>(v00[k]));
                    const float r1 = __fmaf_rn(f[k], byte_of<CS>(v11[k]), f1 * byte_of<CS>(v10[k]));
                    const float u = __fmaf_rn(g, r1, g1 * r0);
                    o[k] = __fmaf_rn(p.alpha[c], u, p.beta[c]);
                }
                OUT *q = out + (size_t)c * plane + ((unsigned)Y * (unsigned)p.Wd + (unsigned)X0);
                if (VEC) {
                    if (sizeof(OUT) == 4) {
                        typedef float v4f __attribute__((ext_vector_type(4)));
                        const v4f w = {o[0], o[1], o[2], o[3]};
                        __builtin_nontemporal_store(w, reinterpret_cast<v4f *>(q));
                    } else {
                        typedef _Float16 v4h __attribute__((ext_vector_type(4)));
                        const v4h w = {(_Float16)o[0], (_Float16)o[1], (_Float16)o[2], (_Float16)o[3]};
                        __builtin_nontemporal_store(w, reinterpret_cast<v4h *>(q));
                    }
                } else {
                    for (int k = 0; k < nx; ++k) q[k] = (OUT)o[k];
                }
            };
            // output channel c reads source channel c, or C - 1 - c
            channel(std::integral_constant<int, REVERSE ? C - 1 : 0>{}, 0);
            if (C > 1) channel(std::integral_constant<int, REVERSE ? (C > 1 ? C - 2 : 0) : (C > 1 ? 1 : 0)>{}, 1);
            if (C > 2) channel(std::integral_constant<int, REVERSE ? (C > 2 ? C - 3 : 0) : (C > 2 ? 2 : 0)>{}, 2);
            if (C > 3) channel(std::integral_constant<int, REVERSE ? 0 : (C > 3 ? 3 : 0)>{}, 3);
        }
    }
}

template <int C, typename OUT, bool VEC, bool REVERSE>
__global__ __launch_bounds__(kPreThreads) void k_preprocess(const uint8_t *__restrict__ src, OUT *__restrict__ dst,
                                                               PreParams p)
{
    const int X0 = 4 * (blockIdx.x * blockDim.x + threadIdx.x);
    const int Yb = kPreRows * (blockIdx.y * blockDim.y + threadIdx.y);
    const int n = blockIdx.z;
    if (X0 >= p.Wd || Yb >= p.Hd) return;
    const uint8_t *img = src + (size_t)n * p.Hs * p.Ws * C;
    OUT *out = dst + (size_t)n * C * p.Hd * p.Wd;
    // only the last image holds the tensor's last pixel
    if (C == 3 && n == p.N - 1)
        pre_rows<C, OUT, VEC, REVERSE, true>(img, out, p, X0, Yb);
    else
        pre_rows<C, OUT, VEC, REVERSE, false>(img, out, p, X0, Yb);
}

template <int C, typename OUT, bool VEC>
static void launch_pre_r(dim3 grid, dim3 block, hipStream_t s, const uint8_t *src, OUT *dst, const PreParams &p, bool reverse)
{
    if (reverse)
        HP_KERNEL((k_preprocess<C, OUT, VEC, true>), grid, block, 0, s, src, dst, p);
    else
        HP_KERNEL((k_preprocess<C, OUT, VEC, false>), grid, block, 0, s, src, dst, p);
}

template <int C>
static hipError_t launch_pre_c(const uint8_t *src, void *dst, hp_dtype out_dt, int N, const PreParams &p, bool reverse,
                               hipStream_t s)
{
    // a workgroup spans a whole row of 4-pixel groups when that fits, so that few lanes idle at
    // the right edge, and as many row groups as its thread budget allows
    const int W4 = (p.Wd + 3) / 4;
    const int bx = W4 < kPreThreads ? W4 : kPreThreads;
    int by = kPreThreads / bx;
    if (by > 8) by = 8;
    dim3 block(bx, by), grid((W4 + bx - 1) / bx, (p.Hd + kPreRows * by - 1) / (kPreRows * by), N);
    if (grid.y > 65535 || grid.z > 65535) return hipErrorInvalidValue;
    const bool vec = p.Wd % 4 == 0 && ((uintptr_t)dst % 16) == 0;
    if (out_dt == HP_F32) {
        if (vec)
            launch_pre_r<C, float, true>(grid, block, s, src, (float *)dst, p, reverse);
        else
            launch_pre_r<C, float, false>(grid, block, s, src, (float *)dst, p, reverse);
    } else {
        if (vec)
            launch_pre_r<C, _Float16, true>(grid, block, s, src, (_Float16 *)dst, p, reverse);
        else
            launch_pre_r<C, _Float16, false>(grid, block, s, src, (_Float16 *)dst, p, reverse);
    }
    return hipGetLastError();
}

hipError_t launch_preprocess(const uint8_t *src, int N, int Hs, int Ws, int C, hp_dtype out_dt, void *dst, int Hd, int Wd,
                             int reverse_channels, const float *alpha, const float *beta, hipStream_t s)
{
    PreParams p;
    for (int c = 0; c < 4; ++c) {
        p.alpha[c] = c < C ? alpha[c] : 0.0f;
        p.beta[c] = c < C ? beta[c] : 0.0f;
    }
    p.Hs = Hs; p.Ws = Ws; p.Hd = Hd; p.Wd = Wd; p.N = N;
    p.rden_x = 1.0f / (float)(2 * Wd);
    p.rden_y = 1.0f / (float)(2 * Hd);
    p.step_qx = (2 * Ws) / (2 * Wd); p.step_rx = (2 * Ws) % (2 * Wd);
    p.step_qy = (2 * Hs) / (2 * Hd); p.step_ry = (2 * Hs) % (2 * Hd);
    const bool reverse = reverse_channels != 0;
    switch (C) {
    case 1: return launch_pre_c<1>(src, dst, out_dt, N, p, reverse, s);
    case 2: return launch_pre_c<2>(src, dst, out_dt, N, p, reverse, s);
    case 3: return launch_pre_c<3>(src, dst, out_dt, N, p, reverse, s);
    case 4: return launch_pre_c<4>(src, dst, out_dt, N, p, reverse, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace hp
