// Optional smoothing of the upsampled confidence maps before the peak search: a separable
// correlation with a caller-supplied odd-length tap vector, edge pixels repeated beyond the
// borders, fp32, horizontal pass first, every sum accumulated from 0 in ascending tap order with
// one fused multiply-add per tap (so the result is defined bit for bit).
//
// One workgroup produces a tile of 64 x 64 outputs in one launch, the horizontally filtered rows
// living only in LDS.  Horizontal pass: the tile's source rows (64 + 2r of them, 64 + 2r wide) are
// staged 16 at a time, one coalesced row per wavefront load; a thread filters four neighbouring
// outputs of a row from a sliding window held in registers (two 16-byte LDS reads per four taps,
// sixteen multiply-adds).  Vertical pass: a thread walks down one column of the filtered rows,
// four outputs at a time, with the same window scheme, and stores rows 256 bytes wide.  With 17
// taps that is 38 multiply-adds and 8 bytes of memory traffic per output pixel: the kernel sits
// near the balance of the vector ALUs and HBM.
#include "hp_dev.h"

namespace hp {

constexpr int kSmoothTile = 64;      // outputs per tile side
constexpr int kSmoothStage = 16;     // source rows staged at a time: 16 rows x 16 threads x 4 outputs
constexpr int kSmoothMaxR = 32;      // largest radius: 65 taps
constexpr int kSmoothSrcW = kSmoothTile + 2 * kSmoothMaxR + 8;   // floats per staged row: a multiple of 4, with room
                                                                 // for the last window's unused tail

__global__ __launch_bounds__(kBlock) void k_smooth(const float *__restrict__ src, float *__restrict__ dst, int C,
                                                   int C_mem, int H, int W, const float *__restrict__ taps, int T)
{
    __shared__ float s_taps[2 * kSmoothMaxR + 4];
    __shared__ __attribute__((aligned(16))) float s_src[kSmoothStage][kSmoothSrcW];
    extern __shared__ __attribute__((aligned(16))) float s_t[];   // [64 + 2r][64] horizontally filtered rows

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
    const int r = (T - 1) >> 1;
    const int plane = blockIdx.z;
    const size_t plane_off = ((size_t)(plane / C) * C_mem + plane % C) * H * W;
    const float *s = src + plane_off;
    float *d = dst + plane_off;
    const int x0 = blockIdx.x * kSmoothTile, y0 = blockIdx.y * kSmoothTile;
    const int rows = kSmoothTile + 2 * r, cols = kSmoothTile + 2 * r;

    if (tid < T) s_taps[tid] = taps[tid];

    // ---- horizontal pass into s_t -------------------------------------------------------------
    const int hr = tid >> 4, hx = 4 * (tid & 15);   // this thread's row of the stage and its four outputs
    for (int rs = 0; rs < rows; rs += kSmoothStage) {
        __syncthreads();   // the previous stage has been consumed (and s_taps is in place)
        for (int rr = wv; rr < kSmoothStage; rr += kBlock / kWave) {
            const int y = min(max(y0 - r + rs + rr, 0), H - 1);
            for (int c = lane; c < cols; c += kWave) s_src[rr][c] = s[(size_t)y * W + min(max(x0 - r + c, 0), W - 1)];
        }
        __syncthreads();
        if (rs + hr < rows) {
            float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            float4 lo = *(const float4 *)&s_src[hr][hx];
            for (int i = 0; i < T; i += 4) {
                const float4 hi = *(const float4 *)&s_src[hr][hx + i + 4];
                const float w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    if (i + m < T) {   // the same for every thread
                        const float tap = s_taps[i + m];
#pragma unroll
                        for (int o = 0; o < 4; ++o) acc[o] = __fmaf_rn(tap, w[o + m], acc[o]);
                    }
                }
                lo = hi;
            }
            *(float4 *)&s_t[(rs + hr) * kSmoothTile + hx] = make_float4(acc[0], acc[1], acc[2], acc[3]);
        }
    }
    __syncthreads();

    // ---- vertical pass out of s_t ----------------------------------------------------------------
    const int vx = tid & (kSmoothTile - 1), vg = tid >> 6;   // this thread's column and its 16 rows
    if (x0 + vx >= W) return;
#pragma unroll 1
    for (int k = 0; k < 4; ++k) {
        const int yo = 16 * vg + 4 * k;   // four outputs: tile rows yo .. yo + 3
        if (y0 + yo >= H) break;
        float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        float w[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) w[j] = s_t[(yo + j) * kSmoothTile + vx];
        for (int i = 0; i < T; i += 4) {
#pragma unroll
            for (int j = 0; j < 4; ++j) w[4 + j] = (yo + i + 4 + j < rows) ? s_t[(yo + i + 4 + j) * kSmoothTile + vx] : 0.0f;
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                if (i + m < T) {
                    const float tap = s_taps[i + m];
#pragma unroll
                    for (int o = 0; o < 4; ++o) acc[o] = __fmaf_rn(tap, w[o + m], acc[o]);
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) w[j] = w[4 + j];
        }
#pragma unroll
        for (int o = 0; o < 4; ++o)
            if (y0 + yo + o < H) __builtin_nontemporal_store(acc[o], &d[(size_t)(y0 + yo + o) * W + x0 + vx]);
    }
}

hipError_t launch_smooth(const float *src, float *dst, int N, int C, int C_mem, int H, int W, const float *taps,
                         int n_taps, hipStream_t s)
{
    const int r = (n_taps - 1) / 2;
    const size_t lds = sizeof(float) * (size_t)(kSmoothTile + 2 * r) * kSmoothTile;
    // grid.z carries the planes: at most 65535 per launch
    for (int p0 = 0; p0 < N * C; p0 += 65535 / C * C) {
        const int planes = min(N * C - p0, 65535 / C * C);
        const size_t off = (size_t)(p0 / C) * C_mem * H * W;
        const dim3 grid((W + kSmoothTile - 1) / kSmoothTile, (H + kSmoothTile - 1) / kSmoothTile, planes);
        HP_KERNEL(k_smooth, grid, dim3(kBlock), lds, s, src + off, dst + off, C, C_mem, H, W, taps, n_taps);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace hp
