// Pre-processing operator of the paper's inference dataflow (Section 2.2.1, operator 2:
// decoded images are resized and switched to the channel-first layout the network expects).
// Arithmetic as stated at hp_preprocess in hp.h.
//
// The kernel is written from the output: a thread produces 4 consecutive pixels of kRows
// consecutive rows for all channels, so every store is one 16-byte (fp32) or 8-byte (fp16)
// piece of a row that the wavefront completes to a contiguous kilobyte, and the interleaved
// source pixel is read once for all its channels, as one 32-bit word where the layout allows.
// The column cells and weights are computed once per thread and serve all its rows.
#include "hp_dev.h"

namespace hp {

constexpr int kPreRows = 4;       // rows per thread
constexpr int kPreBx = 64, kPreBy = 4;

struct PreParams {
    float alpha[4], beta[4];
    int Hs, Ws, Hd, Wd;
    int reverse;
    float rden_x, rden_y;         // 1 / (2 Wd), 1 / (2 Hd)
    unsigned long long total_bytes;
};

// Cell and weight of output index X along an axis of ns source nodes resized to nd:
// num = (2X + 1) ns - nd over den = 2 nd; the quotient is taken through the reciprocal and made
// exact (num < 2^31 and the quotient < 2^15 keep the estimate within one of the truth).
__device__ __forceinline__ void pre_axis(int X, int ns, int nd, float rden, int &i0, int &i1, float &f)
{
    const int num = (2 * X + 1) * ns - nd, den = 2 * nd;
    if (num < 0) {
        i0 = 0;
        f = 0.0f;
    } else {
        int q = (int)((float)num * rden);
        int r = num - q * den;
        if (r < 0) { --q; r += den; }
        if (r < 0) { --q; r += den; }
        if (r >= den) { ++q; r -= den; }
        if (r >= den) { ++q; r -= den; }
        i0 = q;
        f = (float)r / (float)den;
    }
    i1 = min(i0 + 1, ns - 1);
}

// The C bytes of source pixel `px` (index over the whole tensor) as the low bytes of a word.
template <int C>
__device__ __forceinline__ uint32_t load_px(const uint8_t *__restrict__ src, size_t px, unsigned long long total_bytes)
{
    if (C == 4) return *reinterpret_cast<const uint32_t *>(src + 4 * px);
    if (C == 1) return src[px];
    if (C == 2) {
        struct __attribute__((packed)) U16 { uint16_t v; };
        return reinterpret_cast<const U16 *>(src + 2 * px)->v;
    }
    // three bytes: read four where four exist; the tensor's last pixel is read one byte early
    struct __attribute__((packed)) U32 { uint32_t v; };
    const size_t at = 3 * px;
    if (total_bytes < 4) return (uint32_t)src[at] | ((uint32_t)src[at + 1] << 8) | ((uint32_t)src[at + 2] << 16);
    const size_t from = at + 4 <= total_bytes ? at : at - 1;
    const uint32_t v = reinterpret_cast<const U32 *>(src + from)->v;
    return from == at ? v : v >> 8;
}

__device__ __forceinline__ float byte_of(uint32_t v, int c) { return (float)((v >> (8 * c)) & 0xffu); }

template <int C, typename OUT, bool VEC>
__global__ __launch_bounds__(kPreBx *kPreBy) void k_preprocess(const uint8_t *__restrict__ src, OUT *__restrict__ dst,
                                                               PreParams p)
{
    const int X0 = 4 * (blockIdx.x * kPreBx + threadIdx.x);
    const int Yb = kPreRows * (blockIdx.y * kPreBy + threadIdx.y);
    const int n = blockIdx.z;
    if (X0 >= p.Wd || Yb >= p.Hd) return;
    const int nx = min(4, p.Wd - X0);

    int x0[4], x1[4];
    float f[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) pre_axis(min(X0 + k, p.Wd - 1), p.Ws, p.Wd, p.rden_x, x0[k], x1[k], f[k]);

    const size_t img_px = (size_t)n * p.Hs * p.Ws;
    const size_t plane = (size_t)p.Hd * p.Wd;
    OUT *out = dst + (size_t)n * C * plane;
    for (int r = 0; r < kPreRows; ++r) {
        const int Y = Yb + r;
        if (Y >= p.Hd) break;
        int y0, y1;
        float g;
        pre_axis(Y, p.Hs, p.Hd, p.rden_y, y0, y1, g);
        const size_t row0 = img_px + (size_t)y0 * p.Ws, row1 = img_px + (size_t)y1 * p.Ws;
        uint32_t v00[4], v01[4], v10[4], v11[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v00[k] = load_px<C>(src, row0 + x0[k], p.total_bytes);
            v01[k] = load_px<C>(src, row0 + x1[k], p.total_bytes);
            v10[k] = load_px<C>(src, row1 + x0[k], p.total_bytes);
            v11[k] = load_px<C>(src, row1 + x1[k], p.total_bytes);
        }
        const float g1 = 1.0f - g;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const int cs = p.reverse ? C - 1 - c : c;
            float o[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float f1 = 1.0f - f[k];
                const float r0 = __fmaf_rn(f[k], byte_of(v01[k], cs), f1 * byte_of(v00[k], cs));
                const float r1 = __fmaf_rn(f[k], byte_of(v11[k], cs), f1 * byte_of(v10[k], cs));
                const float u = __fmaf_rn(g, r1, g1 * r0);
                o[k] = __fmaf_rn(p.alpha[c], u, p.beta[c]);
            }
            OUT *q = out + (size_t)c * plane + (size_t)Y * p.Wd + X0;
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
        }
    }
}

template <int C>
static hipError_t launch_pre_c(const uint8_t *src, void *dst, hp_dtype out_dt, int N, const PreParams &p, hipStream_t s)
{
    const int W4 = (p.Wd + 3) / 4;
    dim3 block(kPreBx, kPreBy), grid((W4 + kPreBx - 1) / kPreBx, (p.Hd + kPreRows * kPreBy - 1) / (kPreRows * kPreBy), N);
    if (grid.y > 65535 || grid.z > 65535) return hipErrorInvalidValue;
    const bool vec = p.Wd % 4 == 0 && ((uintptr_t)dst % 16) == 0;
    if (out_dt == HP_F32) {
        if (vec)
            hipLaunchKernelGGL((k_preprocess<C, float, true>), grid, block, 0, s, src, (float *)dst, p);
        else
            hipLaunchKernelGGL((k_preprocess<C, float, false>), grid, block, 0, s, src, (float *)dst, p);
    } else {
        if (vec)
            hipLaunchKernelGGL((k_preprocess<C, _Float16, true>), grid, block, 0, s, src, (_Float16 *)dst, p);
        else
            hipLaunchKernelGGL((k_preprocess<C, _Float16, false>), grid, block, 0, s, src, (_Float16 *)dst, p);
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
    p.Hs = Hs; p.Ws = Ws; p.Hd = Hd; p.Wd = Wd;
    p.reverse = reverse_channels ? 1 : 0;
    p.rden_x = 1.0f / (float)(2 * Wd);
    p.rden_y = 1.0f / (float)(2 * Hd);
    p.total_bytes = (unsigned long long)N * Hs * Ws * C;
    switch (C) {
    case 1: return launch_pre_c<1>(src, dst, out_dt, N, p, s);
    case 2: return launch_pre_c<2>(src, dst, out_dt, N, p, s);
    case 3: return launch_pre_c<3>(src, dst, out_dt, N, p, s);
    case 4: return launch_pre_c<4>(src, dst, out_dt, N, p, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace hp
