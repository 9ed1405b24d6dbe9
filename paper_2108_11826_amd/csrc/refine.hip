// Optional sub-pixel refinement of peak positions: per axis, the vertex of the parabola through the peak's
// value and its two neighbours' values on the map the peaks were found on (fp32, operation by operation as
// written at hp_refine_peaks in hp.h).  One thread per stored peak; five scattered reads each.
#include "hp_dev.h"

namespace hp {

__device__ __forceinline__ float refine_axis(float a, float b, float c)
{
    const float den = (a + c) - (b + b);
    if (!(den < 0.0f)) return 0.0f;
    const float off = (0.5f * (a - c)) / den;
    return fminf(fmaxf(off, -0.5f), 0.5f);
}

__global__ __launch_bounds__(kBlock) void k_refine(const float *__restrict__ maps, int C_mem, int K, int H, int W,
                                                   const int32_t *__restrict__ px, const int32_t *__restrict__ py,
                                                   const int32_t *__restrict__ count, int cap, float *__restrict__ xf,
                                                   float *__restrict__ yf)
{
    const int n = blockIdx.z, c = blockIdx.y;
    const int k = blockIdx.x * kBlock + threadIdx.x;
    const int list = n * K + c;
    if (k >= min(count[list], cap)) return;
    const size_t e = (size_t)list * cap + k;
    const int x = px[e], y = py[e];
    if (x < 0 || x >= W || y < 0 || y >= H) return;   // not a position on this map: nothing to read
    const float *u = maps + ((size_t)n * C_mem + c) * H * W;
    const float b = u[(size_t)y * W + x];
    float ox = 0.0f, oy = 0.0f;
    if (x > 0 && x < W - 1) ox = refine_axis(u[(size_t)y * W + x - 1], b, u[(size_t)y * W + x + 1]);
    if (y > 0 && y < H - 1) oy = refine_axis(u[(size_t)(y - 1) * W + x], b, u[(size_t)(y + 1) * W + x]);
    xf[e] = (float)x + ox;
    yf[e] = (float)y + oy;
}

hipError_t launch_refine(const float *maps, int N, int C_mem, int K, int H, int W, const hp_peaks &pk, float *xf, float *yf,
                         hipStream_t s)
{
    // grid.z carries the images: at most 65535 per launch
    for (int n0 = 0; n0 < N; n0 += 65535) {
        const int nn = min(N - n0, 65535);
        const size_t lists = (size_t)n0 * K, entries = lists * pk.cap;
        HP_KERNEL(k_refine, dim3((pk.cap + kBlock - 1) / kBlock, K, nn), dim3(kBlock), 0, s,
                  maps + (size_t)n0 * C_mem * H * W, C_mem, K, H, W, pk.x + entries, pk.y + entries, pk.count + lists, pk.cap,
                  xf + entries, yf + entries);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace hp
