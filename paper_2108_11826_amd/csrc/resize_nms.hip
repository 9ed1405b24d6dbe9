// Upsampling (x8 half-pixel bilinear) with optional materialisation and fused peak
// detection, peak detection on materialised maps, and the ordering of peak lists.
//
// These are the "resizing" and the first half of the post-processing operator of the
// paper's inference engine (Section 2.2, Section 2.2.1 operator 4).  The arithmetic is
// the one stated at hp_resize / hp_find_peaks in hp.h.
#include "hp_dev.h"

namespace hp {

typedef float v4f __attribute__((ext_vector_type(4)));

__global__ void k_init(int32_t *a, int na, int32_t *b, int nb, int32_t *status)
{
    int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g < na) a[g] = 0;
    if (g < nb) b[g] = 0;
    if (g == 0 && status) *status = 0;
}

hipError_t launch_init(int32_t *a, int na, int32_t *b, int nb, int32_t *status, hipStream_t s)
{
    int n = na > nb ? na : nb;
    if (n < 1) n = 1;
    HP_KERNEL(k_init, dim3((n + kBlock - 1) / kBlock), dim3(kBlock), 0, s, a, na, b, nb, status);
    return hipGetLastError();
}

__device__ __forceinline__ void emit_peak(int32_t *counts, uint64_t *stage, int plane, int cap, int cap2,
                                          int key, float u)
{
    int slot = atomicAdd(&counts[plane * kCtrStride], 1);
    if (slot < cap)
        stage[(size_t)plane * cap2 + slot] = ((uint64_t)(uint32_t)key << 32) | (uint64_t)__float_as_uint(u);
}

// The unit of work of the peak search is the 8-row x 4-column hi-res tile rows [8j, 8j+8), columns [8m+4hf, 8m+4hf+4)
// of one plane: the tile plus a one-pixel halo (10 x 6 values) is a function of the 3x3 lo-res
// neighbourhood of node (j, m).
//
// Column X = 8m + t (t = -1..8) reads nodes (m-1, m) with weight (2t+9)/16 for t <= 3 and
// nodes (m, m+1) with weight (2t-7)/16 for t >= 4; left of node 0 the weight is 0 and right
// of node w-1 the upper node is clamped.  Rows alike.

// The nine nodes around node (j, m) = node t of a plane (t = j w + m): offsets from the plane's first node, no multiply.
template <typename T>
__device__ __forceinline__ void load_nodes(const T *pl, int h, int w, int j, int m, int t, float (&lo9)[3][3])
{
    const int row[3] = {j > 0 ? t - m - w : t - m, t - m, j < h - 1 ? t - m + w : t - m};
    const int mc[3] = {max(m - 1, 0), m, min(m + 1, w - 1)};
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int k = 0; k < 3; ++k) lo9[r][k] = ld(pl + (unsigned)(row[r] + mc[k]));
}

// Every value of a tile and its halo is a convex combination of its nine nodes, formed with
// four roundings at most: none exceeds max9 * (1 + 2^-24)^4.  If even that stays below a
// positive threshold the tile holds no peak (a non-positive max9 gives non-positive values).
__device__ __forceinline__ bool tile_may_peak(const float (&lo9)[3][3], float thr)
{
    if (!(thr > 0.0f)) return true;
    float mx = lo9[0][0];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int k = 0; k < 3; ++k) mx = fmaxf(mx, lo9[r][k]);
    return !(mx * 1.000001f < thr);
}

// Upsamples one tile (with halo) from its nine nodes into v[10][6]: v[r+1][k] is row 8j+r,
// column 8m+4hf-1+k.  Column k = 0 always reads nodes (m-1, m), column 5 always (m, m+1); columns 1..4 read
// (m-1, m) in the left half tile (hf = 0) and (m, m+1) in the right one, so the half decides a pair of nodes per
// source row and six weights once, instead of every column choosing its nodes for itself.
__device__ __forceinline__ void upsample_tile(const float (&lo9)[3][3], int j, int m, int hf, float (&v)[10][6])
{
    const bool right = hf != 0, edge = m == 0;     // left of node 0 the weight is 0
    float fx[6];
    fx[0] = edge ? 0.0f : (right ? 15.0f : 7.0f) * 0.0625f;
#pragma unroll
    for (int k = 1; k <= 4; ++k) fx[k] = right ? (float)(2 * k - 1) * 0.0625f : (edge ? 0.0f : (float)(2 * k + 7) * 0.0625f);
    fx[5] = right ? 9.0f * 0.0625f : 0.0625f;
    float hr[3][6];
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const float p = right ? lo9[r][1] : lo9[r][0], q = right ? lo9[r][2] : lo9[r][1];
        hr[r][0] = __fmaf_rn(fx[0], lo9[r][1], (1.0f - fx[0]) * lo9[r][0]);
#pragma unroll
        for (int k = 1; k <= 4; ++k) hr[r][k] = __fmaf_rn(fx[k], q, (1.0f - fx[k]) * p);
        hr[r][5] = __fmaf_rn(fx[5], lo9[r][2], (1.0f - fx[5]) * lo9[r][1]);
    }
#pragma unroll
    for (int r = -1; r <= 8; ++r) {
        const bool top = r <= 3;
        const float gconst = top ? (float)(2 * r + 9) * 0.0625f : (float)(2 * r - 7) * 0.0625f;
        const float gy = (top && j == 0) ? 0.0f : gconst;
#pragma unroll
        for (int k = 0; k < 6; ++k) {
            const float a = top ? hr[0][k] : hr[1][k];
            const float b = top ? hr[1][k] : hr[2][k];
            v[r + 1][k] = __fmaf_rn(gy, b, (1.0f - gy) * a);
        }
    }
}

// 3x3 test on the 8 x 4 interior of v; halo entries outside the map must not take part.
// A pixel is a peak when it exceeds thr and its earlier neighbours (row above, left) and is
// not below its later ones (right, row below).
__device__ __forceinline__ void tile_peaks(float (&v)[10][6], int j, int h, int X0, int Y0, int W, float thr,
                                           int32_t *counts, uint64_t *stage, int plane, int cap, int cap2)
{
    const float ninf = -__builtin_huge_valf();
    if (X0 == 0) {
#pragma unroll
        for (int r = 0; r < 10; ++r) v[r][0] = ninf;
    }
    if (X0 + 4 >= W) {
#pragma unroll
        for (int r = 0; r < 10; ++r) v[r][5] = ninf;
    }
    if (j == 0) {
#pragma unroll
        for (int k = 0; k < 6; ++k) v[0][k] = ninf;
    }
    if (j == h - 1) {
#pragma unroll
        for (int k = 0; k < 6; ++k) v[9][k] = ninf;
    }
    float h3[10][4];     // maximum of the three horizontal neighbours centred on column k+1
#pragma unroll
    for (int r = 0; r < 10; ++r)
#pragma unroll
        for (int k = 0; k < 4; ++k) h3[r][k] = fmaxf(fmaxf(v[r][k], v[r][k + 1]), v[r][k + 2]);
    // A tile seldom holds a peak and hardly ever two, and an append costs a memory round trip (the counter comes
    // back before the entry can be stored).  So the test only notes which pixels are peaks and keeps the last one
    // found; lanes with exactly one peak then append together, one round trip for the wavefront, and the rare lane
    // with several walks through them one by one.
    uint32_t found = 0;
    int last_pos = 0;
    float last_u = 0.0f;
#pragma unroll
    for (int r = 1; r <= 8; ++r) {
#pragma unroll
        for (int k = 1; k <= 4; ++k) {
            const float u = v[r][k];
            const float early = fmaxf(fmaxf(h3[r - 1][k - 1], v[r][k - 1]), thr);
            const float late = fmaxf(h3[r + 1][k - 1], v[r][k + 1]);
            const bool is_peak = u > early && u >= late;
            found |= is_peak ? 1u << ((r - 1) * 4 + (k - 1)) : 0u;
            last_pos = is_peak ? (r - 1) * 4 + (k - 1) : last_pos;
            last_u = is_peak ? u : last_u;
        }
    }
    if (found) {
        if ((found & (found - 1)) == 0) {
            emit_peak(counts, stage, plane, cap, cap2, (Y0 + (last_pos >> 2)) * W + X0 + (last_pos & 3), last_u);
        } else {
#pragma unroll
            for (int r = 1; r <= 8; ++r) {
#pragma unroll
                for (int k = 1; k <= 4; ++k) {
                    if (found & (1u << ((r - 1) * 4 + (k - 1))))
                        emit_peak(counts, stage, plane, cap, cap2, (Y0 + r - 1) * W + X0 + k - 1, v[r][k]);
                }
            }
        }
    }
}

// Materialising form.  One thread produces one 16-byte group of four pixels of one row and
// issues exactly one non-temporal store; a workgroup is a 2-D block (column groups of a row) x
// (R consecutive rows) of one plane, workgroups are numbered in memory order (row groups of a
// plane, then planes), so consecutive wavefronts write consecutive kilobytes.  Measured on
// MI355X this order streams at the rate of a plain fill, while threads that each write several
// rows (a tile per thread) lose a quarter of it and threads that write two adjacent groups lose
// more than half.  With one store per thread the instruction count per thread decides whether
// the kernel stays memory-bound: sizes are folded on the host, products use 24-bit multiplies.
// The four columns of a group share one pair of source nodes, the row one pair of source rows:
// four loads (L1/L2 hits) per thread.  The grid is (row groups [x column parts], channels,
// images), the channels counted over [0, Ca) of tensor a followed by the Cb channels of tensor
// b, so that a workgroup finds its plane from its block index with a compare and two
// multiplications on the scalar unit, without a division in front of every wavefront's loads.
//
// The source is 64 times smaller than the output, but a workgroup that finds its source rows
// in no cache waits a full memory round trip before its only store, and with every workgroup
// of the write front in that state the kernel runs a third slower (measured after a kernel
// that had swept the caches: 94 us instead of 65 us for 447 MB).  So the first `warm_blocks`
// workgroups, which are dispatched first, begin by streaming both source tensors through the
// caches, 16 bytes per thread and step (`vec_a`, `vec_b` 16-byte units; 0 = skip); every later
// workgroup then finds its rows in the shared cache.
template <typename T>
__global__ __launch_bounds__(1024) void k_resize_write(const T *__restrict__ lo_a, const T *__restrict__ lo_b,
                                                       float *__restrict__ hi_a, float *__restrict__ hi_b,
                                                       int c0, int n0, int Ca, int Ca_mem, int Cb, int h, int w,
                                                       int W4, int H, int xparts, int bx, int rows, int grid_x,
                                                       int grid_y, unsigned vec_a, unsigned vec_b,
                                                       unsigned warm_blocks)
{
    // Every wavefront lives for one load and one store, so what stands between its start and its
    // loads counts: the block shape comes as arguments (not from the dispatch packet), and all
    // four pointers are brought into registers with the first batch of argument loads instead of
    // where a branch first needs them.
    asm volatile("" ::"s"(lo_a), "s"(lo_b), "s"(hi_a), "s"(hi_b));
    // blockIdx.x: row group (times the column parts of rows wider than a workgroup), y: channel, z: image
    const unsigned block_linear = (blockIdx.z * grid_y + blockIdx.y) * grid_x + blockIdx.x;
    if (block_linear < warm_blocks) {
        const unsigned nthr = bx * rows;
        const unsigned stride = warm_blocks * nthr;
        const unsigned first = block_linear * nthr + threadIdx.y * bx + threadIdx.x;
        uint32_t seen = 0;
        for (unsigned i = first; i < vec_a; i += stride) {
            const uint4 v = ((const uint4 *)lo_a)[i];
            seen |= (v.x ^ v.y) | (v.z ^ v.w);
        }
        for (unsigned i = first; i < vec_b; i += stride) {
            const uint4 v = ((const uint4 *)lo_b)[i];
            seen |= (v.x ^ v.y) | (v.z ^ v.w);
        }
        asm volatile("" ::"v"(seen));        // the loads are wanted for their effect on the caches
    }
    const int group = xparts == 1 ? (int)blockIdx.x : (int)(blockIdx.x / xparts);
    const int xpart = xparts == 1 ? 0 : (int)(blockIdx.x - group * xparts);
    const int x4 = xpart * bx + threadIdx.x;
    const int Y = group * rows + threadIdx.y;
    if (x4 >= W4 || Y >= H) return;

    // plane -> tensor, uniform over the workgroup
    const int c = c0 + blockIdx.y, n = n0 + blockIdx.z;
    const bool in_a = c < Ca;
    const size_t plane_mem = (size_t)n * (in_a ? Ca_mem : Cb) + (in_a ? c : c - Ca);
    const T *p = (in_a ? lo_a : lo_b) + plane_mem * (size_t)(h * w);
    float *q = (in_a ? hi_a : hi_b) + plane_mem * (size_t)H * (size_t)(4 * W4);

    const int numy = 2 * Y - 7;
    const int y0 = numy < 0 ? 0 : numy >> 4;
    const float gy = numy < 0 ? 0.0f : (float)(numy & 15) * 0.0625f;
    const int y1 = min(y0 + 1, h - 1);
    const int numx = 8 * x4 - 7;                  // first column X = 4 * x4
    const int x0 = numx < 0 ? 0 : numx >> 4;
    const int x1 = min(x0 + 1, w - 1);
    const float f0 = (float)(numx & 15) * 0.0625f;
    const unsigned o0 = (unsigned)__mul24(y0, w), o1 = (unsigned)__mul24(y1, w);
    const float a0 = ld(p + (o0 + x0)), b0 = ld(p + (o0 + x1));
    const float a1 = ld(p + (o1 + x0)), b1 = ld(p + (o1 + x1));
    const float g1 = 1.0f - gy;
    v4f o;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float f = numx < 0 ? 0.0f : f0 + 0.125f * (float)k;     // k/16 steps of 2: exact
        const float r0 = __fmaf_rn(f, b0, (1.0f - f) * a0);
        const float r1 = __fmaf_rn(f, b1, (1.0f - f) * a1);
        o[k] = __fmaf_rn(gy, r1, g1 * r0);
    }
    const unsigned off = (unsigned)__mul24(Y, W4) + (unsigned)x4;     // in 16-byte units, < 2^29 by the host's check
    __builtin_nontemporal_store(o, (v4f *)q + off);
}

// Fused form: nothing is written but peaks.  Every wavefront works by itself on NP * 64 consecutive lo-res nodes
// of one searched plane (no workgroup barrier; the plane comes from the block index, channel and image).  Phase 1,
// NP nodes per lane, their loads in flight together: can the node's two tiles hold a peak at all?  The nodes that can
// are compacted, with their nine values, into a list in the wavefront's own piece of LDS (places from ballots);
// phase 2 spreads the list's tiles densely over the lanes, so the upsampling and the 3x3 test are only paid where the
// map rises to the threshold, and a wavefront whose nodes are all below it leaves after one round of loads.
// The kernel issues 4 M vector instructions a launch at the benchmark's size and is bound by that more than by
// anything else, so the index arithmetic is kept small: a node's row and column come from one single-precision
// quotient put right by its remainder (three integer divisions a node, for column, row and plane, were a third of
// phase 1), and its neighbours' offsets from additions.
// (Six wavefronts per SIMD: the 80 registers that leaves still hold a tile without spilling.)
constexpr int kNmsWaves = kBlock / kWave;
constexpr int kEntWords = 11;        // 9 values + row, column; odd stride: no LDS bank conflicts

template <typename T, int NP>
__global__ __launch_bounds__(kBlock, 6) void k_resize_nms(const T *__restrict__ lo, int K, int C_mem, int h, int w,
                                                       float thr, int32_t *counts, uint64_t *stage, int cap,
                                                       int cap2, int32_t *status)
{
    __shared__ uint32_t ent_all[kNmsWaves][NP * kWave][kEntWords];
    // first kernel of hp_postprocess: it clears the status word (no kernel of this launch sets bits)
    if (status && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0) *status = 0;
    const int lane = threadIdx.x & (kWave - 1), wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t(*ent)[kEntWords] = ent_all[wv];
    const int hw = h * w;
    const int t0 = (blockIdx.x * kNmsWaves + wv) * (NP * kWave);          // first node of this wavefront in its plane
    if (t0 >= hw) return;
    const int c = blockIdx.y, n = blockIdx.z, plane = n * K + c;
    const T *pl = lo + ((size_t)n * C_mem + c) * (size_t)hw;
    const unsigned long long below = (1ull << lane) - 1ull;
    const float inv_w = 1.0f / (float)w;
    const bool exact_in_float = hw <= (1 << 24);                          // every node index is a float then

    // two nodes per lane at a time: their loads are in flight together and the registers still hold a tile later
    constexpr int kPer = NP < 2 ? NP : 2;
    int n_ent = 0;
    for (int u0 = 0; u0 < NP; u0 += kPer) {
        float lo9[kPer][3][3];
        int jj[kPer], mm[kPer];
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            // nodes beyond the plane's end repeat its last one (their verdict is dropped)
            const int t = min(t0 + (u0 + u) * kWave + lane, hw - 1);
            int j, m;
            if (exact_in_float) {
                // t / w to within one unit; the remainder says which way
                j = (int)((float)t * inv_w);
                m = t - __mul24(j, w);
                if (m < 0) {
                    --j;
                    m += w;
                }
                if (m >= w) {
                    ++j;
                    m -= w;
                }
            } else {
                j = t / w;
                m = t - j * w;
            }
            jj[u] = j;
            mm[u] = m;
            load_nodes(pl, h, w, j, m, t, lo9[u]);
        }
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const bool act = t0 + (u0 + u) * kWave + lane < hw && tile_may_peak(lo9[u], thr);
            const unsigned long long mk = __ballot(act);
            if (act) {
                uint32_t *e = ent[n_ent + __popcll(mk & below)];
#pragma unroll
                for (int r = 0; r < 3; ++r)
#pragma unroll
                    for (int k = 0; k < 3; ++k) e[3 * r + k] = __float_as_uint(lo9[u][r][k]);
                e[9] = (uint32_t)jj[u];
                e[10] = (uint32_t)mm[u];
            }
            n_ent += __popcll(mk);
        }
    }
    if (n_ent == 0) return;
    // the list is written and read by the lanes of this wavefront only
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    const int W = 8 * w;
    for (int task = lane; task < 2 * n_ent; task += kWave) {
        const uint32_t *e = ent[task >> 1];
        const int hf = task & 1;
        float v9[3][3];
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int k = 0; k < 3; ++k) v9[r][k] = __uint_as_float(e[3 * r + k]);
        const int j = (int)e[9], m = (int)e[10];
        float v[10][6];
        upsample_tile(v9, j, m, hf, v);
        tile_peaks(v, j, h, 8 * m + 4 * hf, 8 * j, W, thr, counts, stage, plane, cap, cap2);
    }
}

template <typename T>
static hipError_t launch_resize_write_t(const T *lo_a, const T *lo_b, float *hi_a, float *hi_b, int N, int Ca,
                                        int Ca_mem, int Cb, int h, int w, hipStream_t s)
{
    const int W4 = 2 * w, H = 8 * h;
    if ((long long)H * W4 >= (1LL << 29) || H >= (1 << 24) || W4 >= (1 << 24)) return hipErrorInvalidValue;
    // block = (column groups, rows): a whole row and as many rows as fit 1024 threads (8 at most);
    // rows wider than 1024 groups are split into column parts
    const int bx = W4 <= 1024 ? W4 : 1024;
    int R = 1024 / bx;
    if (R > 8) R = 8;
    const int xparts = (W4 + bx - 1) / bx, groups = (H + R - 1) / R;
    const int Cg = Ca + Cb;
    if (N <= 0 || Cg <= 0 || (long long)groups * xparts >= (1LL << 31)) return hipErrorInvalidValue;
    // source tensors in 16-byte units for the cache-warming pass of the first launch (a hint:
    // skipped for a pointer that is not 16-byte aligned; a tail shorter than 16 bytes is left out)
    auto units = [&](const T *p, long long channels) -> unsigned {
        if (!p || ((uintptr_t)p & 15) != 0) return 0u;
        return (unsigned)((unsigned long long)N * channels * h * w * sizeof(T) / 16);    // < 2^28 by check_dims
    };
    const unsigned vec_a = units(lo_a, Ca_mem), vec_b = units(lo_b, Cb);
    // the workgroups that share that pass: about two per compute unit
    const long long first_blocks = (long long)groups * xparts * (Cg < 65535 ? Cg : 65535) * (N < 65535 ? N : 65535);
    const unsigned warm = (vec_a | vec_b) == 0u ? 0u : (unsigned)(first_blocks < 512 ? first_blocks : 512);
    bool first = true;
    for (int n0 = 0; n0 < N; n0 += 65535) {
        const int nn = N - n0 < 65535 ? N - n0 : 65535;
        for (int c0 = 0; c0 < Cg; c0 += 65535) {
            const int nc = Cg - c0 < 65535 ? Cg - c0 : 65535;
            HP_KERNEL((k_resize_write<T>), dim3(groups * xparts, nc, nn), dim3(bx, R), 0, s, lo_a, lo_b, hi_a,
                               hi_b, c0, n0, Ca, Ca_mem, Cb, h, w, W4, H, xparts, bx, R, groups * xparts, nc, vec_a, vec_b,
                               first ? warm : 0u);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
            first = false;
        }
    }
    return hipSuccess;
}

hipError_t launch_resize_write(const void *lo_a, const void *lo_b, hp_dtype dt, float *hi_a, float *hi_b, int N,
                               int Ca, int Ca_mem, int Cb, int h, int w, hipStream_t s)
{
    if (dt == HP_F16)
        return launch_resize_write_t((const __half *)lo_a, (const __half *)lo_b, hi_a, hi_b, N, Ca, Ca_mem, Cb, h, w, s);
    return launch_resize_write_t((const float *)lo_a, (const float *)lo_b, hi_a, hi_b, N, Ca, Ca_mem, Cb, h, w, s);
}

template <typename T>
static hipError_t launch_resize_nms_t(const T *lo, int N, int K, int C_mem, int h, int w, float thr, int32_t *counts,
                                      uint64_t *stage, int cap, int cap2, int32_t *status, hipStream_t s)
{
    const long long hw = (long long)h * w;
    if (hw <= 0 || hw >= (1LL << 31) - 4 * kBlock || h >= (1 << 24) || w >= (1 << 24) || K <= 0 || K > 65535 || N <= 0 ||
        N > 65535)
        return hipErrorInvalidValue;
    // two nodes per lane: measured against one, four and eight on the five workloads (equal on the small ones, 13-19 %
    // faster on the large ones, where the tiles of a wavefront's survivors fill its lanes better)
    constexpr int NP = 2;
    constexpr int per_block = kBlock * NP;
    HP_KERNEL((k_resize_nms<T, NP>), dim3((unsigned)((hw + per_block - 1) / per_block), K, N), dim3(kBlock), 0, s, lo, K, C_mem,
              h, w, thr, counts, stage, cap, cap2, status);
    return hipGetLastError();
}

hipError_t launch_resize_nms(const void *lo, hp_dtype dt, int N, int K, int C_mem, int h, int w, float thr,
                             int32_t *counts, uint64_t *stage, int cap, int cap2, int32_t *status, hipStream_t s)
{
    if (dt == HP_F16)
        return launch_resize_nms_t((const __half *)lo, N, K, C_mem, h, w, thr, counts, stage, cap, cap2, status, s);
    return launch_resize_nms_t((const float *)lo, N, K, C_mem, h, w, thr, counts, stage, cap, cap2, status, s);
}

__global__ void k_zero(uint32_t *p, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = 0u;
}

hipError_t launch_zero(void *p, size_t bytes, hipStream_t s)
{
    const size_t n = bytes / 4;
    size_t blocks = (n + kBlock - 1) / kBlock;
    if (blocks > 65536) blocks = 65536;
    if (blocks < 1) blocks = 1;
    HP_KERNEL(k_zero, dim3((unsigned)blocks), dim3(kBlock), 0, s, (uint32_t *)p, n);
    return hipGetLastError();
}

// Peak detection on a materialised map.  One thread owns an 8-row x 4-column tile and reads
// it with a one-pixel halo; pixels outside the map read as -inf.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_nms_hi(const float *__restrict__ cm, int total, int C_cm, int K,
                                                   int H, int W, int tiles_x, int tiles_y, float thr,
                                                   int32_t *counts, uint64_t *stage, int cap, int cap2,
                                                   int32_t *status)
{
    int g = blockIdx.x * kBlock + threadIdx.x;
    // first kernel of hp_find_peaks: it clears the status word (the ordering kernel that follows sets bits)
    if (status && g == 0) *status = 0;
    if (g >= total) return;
    int q = g;
    int tx = q % tiles_x; q /= tiles_x;
    int ty = q % tiles_y; q /= tiles_y;
    int c = q % K;
    int n = q / K;
    const float *pl = cm + ((size_t)n * C_cm + c) * (size_t)H * W;
    const float ninf = -__builtin_huge_valf();
    const int X0 = 4 * tx, Y0 = 8 * ty;

    float v[10][6];
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        int Y = Y0 + r - 1;
        bool yin = Y >= 0 && Y < H;
        const float *row = pl + (size_t)(yin ? Y : 0) * W;
        if (VEC) {
            // W % 4 == 0: the four centre columns are in bounds and 16-byte aligned
            v4f cvec = yin ? *(const v4f *)(row + X0) : (v4f){ninf, ninf, ninf, ninf};
            v[r][1] = cvec.x; v[r][2] = cvec.y; v[r][3] = cvec.z; v[r][4] = cvec.w;
            v[r][0] = (yin && X0 > 0) ? row[X0 - 1] : ninf;
            v[r][5] = (yin && X0 + 4 < W) ? row[X0 + 4] : ninf;
        } else {
#pragma unroll
            for (int k = 0; k < 6; ++k) {
                int X = X0 + k - 1;
                v[r][k] = (yin && X >= 0 && X < W) ? row[X] : ninf;
            }
        }
    }
    const int plane = n * K + c;
#pragma unroll
    for (int r = 1; r <= 8; ++r) {
#pragma unroll
        for (int k = 1; k <= 4; ++k) {
            float u = v[r][k];
            float early = fmaxf(fmaxf(v[r - 1][k - 1], v[r - 1][k]), fmaxf(v[r - 1][k + 1], v[r][k - 1]));
            float late = fmaxf(fmaxf(v[r + 1][k - 1], v[r + 1][k]), fmaxf(v[r + 1][k + 1], v[r][k + 1]));
            // a pixel outside the map holds -inf and never exceeds thr
            if (u > thr && u > early && u >= late)
                emit_peak(counts, stage, plane, cap, cap2, (Y0 + r - 1) * W + X0 + k - 1, u);
        }
    }
}

// Peak detection on a materialised map whose rows are whole 16-byte groups: the memory-bound
// form.  A wavefront owns a strip of R rows x 62 column groups (248 pixels): lane l reads group
// 62 * strip_column - 1 + l, one 16-byte load per row and R + 2 rows, all issued
// before the first use.  The pixel left of a group and the pixel right of it come from the
// neighbouring lanes, so lanes 0 and 63 only supply those and produce no output (their groups
// belong to the next strips); groups and rows outside the map read as -inf.
//
// At 8 TB/s a pixel is worth 0.5 ns of one compute unit's time... the instruction budget is a
// dozen vector instructions per pixel, so the test is arranged to need few: the 3x3 maximum m
// comes from horizontal 3-maxima shared by three rows (4 max per pixel), a pixel is a
// candidate when u >= m and u > thr (2 compares), and only candidates (a fraction of a
// percent) go on to the tie-break against their four earlier neighbours.  Everything that is
// the same for a whole wavefront (strip position, row addresses, edge cases) is computed on
// the scalar unit: the strip comes from the block index, never from a division.
constexpr int kStripRows = 16, kStripGroups = kWave - 2, kStripsPerBlock = 4;

template <int R, bool EDGE>
__device__ __forceinline__ void strip_peaks(const float *__restrict__ pl, int H, int W, int W4, int sx, int Y0, int lane,
                                            float thr, int32_t *counts, uint64_t *stage, int plane, int cap, int cap2)
{
    const float ninf = -__builtin_huge_valf();
    const int cg = sx * kStripGroups - 1 + lane;
    const bool inb = !EDGE || (cg >= 0 && cg < W4);
    const unsigned lane_off = 4u * (unsigned)(inb ? cg : 0);
    v4f v[R + 2];
#pragma unroll
    for (int r = 0; r < R + 2; ++r) {
        const int Y = Y0 + r - 1;                                  // uniform
        const float *row = pl + (size_t)(unsigned)(EDGE ? min(max(Y, 0), H - 1) : Y) * (unsigned)W;
        v[r] = *(const v4f *)(row + lane_off);       // cached loads: the halo rows are read again by the strips next door
        if (EDGE && !(inb && Y >= 0 && Y < H)) v[r] = (v4f){ninf, ninf, ninf, ninf};
    }
    // window of three rows: horizontal 3-maxima of the row above (ha), the row (hc) and the row
    // below (hb); left / right neighbour pixels of the row above (la, ra) and of the row (lc, rc).
    // Lane 0 and lane 63 get their own value back from the shuffles: never used.
    float ha[4], hc[4], hb[4], la, ra, lc, rc, lb, rb;
    auto row_max3 = [&](const v4f &x, float (&h3)[4], float &l, float &r) {
        l = __shfl_up(x.w, 1);
        r = __shfl_down(x.x, 1);
        h3[0] = fmaxf(fmaxf(l, x.x), x.y);
        h3[1] = fmaxf(fmaxf(x.x, x.y), x.z);
        h3[2] = fmaxf(fmaxf(x.y, x.z), x.w);
        h3[3] = fmaxf(fmaxf(x.z, x.w), r);
    };
    row_max3(v[0], ha, la, ra);
    row_max3(v[1], hc, lc, rc);
    const bool out_lane = inb && lane != 0 && lane != kWave - 1;
    const int key0 = Y0 * W + 4 * cg;
#pragma unroll
    for (int r = 1; r <= R; ++r) {
        row_max3(v[r + 1], hb, lb, rb);             // every lane of the wavefront takes part in the shuffles
        bool cand[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float u = v[r][k];
            const float m = fmaxf(fmaxf(ha[k], hc[k]), hb[k]);
            cand[k] = (u >= m) & (u > thr);         // rows and groups outside the map hold -inf: never candidates
        }
        if (out_lane & (cand[0] | cand[1] | cand[2] | cand[3])) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if (!cand[k]) continue;
                // not below any neighbour; a peak if it also exceeds the four earlier ones
                const float u = v[r][k];
                const float ul = k == 0 ? la : v[r - 1][k - 1], ur = k == 3 ? ra : v[r - 1][k + 1];
                const float lft = k == 0 ? lc : v[r][k - 1];
                const float early = fmaxf(fmaxf(ul, v[r - 1][k]), fmaxf(ur, lft));
                if (u > early) emit_peak(counts, stage, plane, cap, cap2, key0 + (r - 1) * W + k, u);
            }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            ha[k] = hc[k];
            hc[k] = hb[k];
        }
        la = lc; ra = rc;
        lc = lb; rc = rb;
    }
}

// block = (64, kStripsPerBlock): one wavefront per strip, strips below each other;
// grid = (strips across, groups of strips down, planes)
template <int R>
__global__ __launch_bounds__(kWave *kStripsPerBlock) void k_nms_hi_strip(const float *__restrict__ cm, int plane0,
                                                                         int C_cm, int K, int H, int W, int W4,
                                                                         float thr, int32_t *counts, uint64_t *stage,
                                                                         int cap, int cap2, int32_t *status)
{
    const int lane = threadIdx.x;
    const int sx = blockIdx.x;
    // first kernel of hp_find_peaks: it clears the status word (the ordering kernel that follows sets bits)
    if (status && (blockIdx.x | blockIdx.y | blockIdx.z | threadIdx.y) == 0 && lane == 0) *status = 0;
    const int sy = blockIdx.y * kStripsPerBlock + __builtin_amdgcn_readfirstlane(threadIdx.y);
    const int Y0 = sy * R;
    if (Y0 >= H) return;
    const int plane = plane0 + blockIdx.z;
    const int n = plane / K, c = plane - n * K;
    const float *pl = cm + ((size_t)n * C_cm + c) * (size_t)H * W;
    const bool edge = sx == 0 || (sx + 1) * kStripGroups + 1 > W4 || Y0 == 0 || Y0 + R + 1 > H;
    if (edge)
        strip_peaks<R, true>(pl, H, W, W4, sx, Y0, lane, thr, counts, stage, plane, cap, cap2);
    else
        strip_peaks<R, false>(pl, H, W, W4, sx, Y0, lane, thr, counts, stage, plane, cap, cap2);
}

hipError_t launch_nms_hi(const float *cm_hi, int N, int C_cm, int K, int H, int W, float thr,
                         int32_t *counts, uint64_t *stage, int cap, int cap2, int32_t *status, hipStream_t s)
{
    if (W % 4 == 0 && ((uintptr_t)cm_hi % 16) == 0) {
        constexpr int R = kStripRows;
        const int W4 = W / 4;
        const int strips_x = (W4 + kStripGroups - 1) / kStripGroups, strips_y = (H + R - 1) / R;
        const int groups_y = (strips_y + kStripsPerBlock - 1) / kStripsPerBlock;
        const long long planes = (long long)N * K;
        if (planes <= 0 || planes >= (1LL << 31) || groups_y > 65535 || (long long)H * W >= (1LL << 31))
            return hipErrorInvalidValue;
        for (long long p0 = 0; p0 < planes; p0 += 65535) {
            const long long np = planes - p0 < 65535 ? planes - p0 : 65535;
            HP_KERNEL((k_nms_hi_strip<R>), dim3(strips_x, groups_y, (unsigned)np), dim3(kWave, kStripsPerBlock), 0,
                               s, cm_hi, (int)p0, C_cm, K, H, W, W4, thr, counts, stage, cap, cap2,
                               p0 == 0 ? status : (int32_t *)nullptr);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    int tiles_x = (W + 3) / 4, tiles_y = (H + 7) / 8;
    long long total64 = (long long)N * K * tiles_x * tiles_y;
    if (total64 <= 0 || total64 >= (1LL << 31) - kBlock) return hipErrorInvalidValue;
    int total = (int)total64;
    dim3 grid((total + kBlock - 1) / kBlock), block(kBlock);
    HP_KERNEL((k_nms_hi<false>), grid, block, 0, s, cm_hi, total, C_cm, K, H, W, tiles_x, tiles_y, thr,
                       counts, stage, cap, cap2, status);
    return hipGetLastError();
}

// Orders the staged peaks of every (image, part) by raster key.  Keys are distinct, so the
// place of a peak is the number of smaller keys: a workgroup loads the list's keys into LDS and
// each of its threads counts for one peak, reading four keys per LDS access (all lanes read the
// same address).  grid = (planes, list parts of kBlock peaks): a long list is ranked by several
// workgroups at once, n^2 / 64 wavefront-compares spread over as many compute units (a bitonic
// sort by one workgroup took 41 us for the 1024-peak lists of the 1080p workload).
// The first workgroup of a plane publishes the count; the append counter is left at zero for
// the next call by whichever workgroup of the plane is the last to have read it (a ticket in
// the counter's own cache line).
__global__ __launch_bounds__(kBlock) void k_sort_peaks(int32_t *ctr, const uint64_t *__restrict__ stage, int cap,
                                                       int cap2, int W, int32_t *counts, int32_t *px, int32_t *py,
                                                       float *ps, int32_t *status)
{
    extern __shared__ uint32_t lds_keys[];            // [n rounded up to 4]
    const int plane = blockIdx.x, part = blockIdx.y;
    const int cnt = ctr[plane * kCtrStride];
    __syncthreads();                                  // every thread has read the counter
    if (threadIdx.x == 0) {
        if (part == 0) {
            counts[plane] = cnt;
            if (cnt > cap) atomicOr(status, (int)HP_STATUS_PEAK_OVERFLOW);
        }
        if (atomicAdd(&ctr[plane * kCtrStride + 1], 1) == (int)gridDim.y - 1) {
            ctr[plane * kCtrStride] = 0;
            ctr[plane * kCtrStride + 1] = 0;
        }
    }
    const int n = max(min(cnt, cap), 0);
    if (part * kBlock >= n) return;
    const uint64_t *g = stage + (size_t)plane * cap2;
    const int n4 = (n + 3) & ~3;
    for (int t = threadIdx.x; t < n4; t += kBlock) lds_keys[t] = t < n ? (uint32_t)(g[t] >> 32) : 0xffffffffu;
    __syncthreads();
    const int idx = part * kBlock + threadIdx.x;
    if (idx >= n) return;
    const uint64_t e = g[idx];
    const uint32_t key = (uint32_t)(e >> 32);
    int r = 0;
    const uint4 *k4 = reinterpret_cast<const uint4 *>(lds_keys);
    for (int u = 0; u < n4 / 4; ++u) {
        const uint4 k = k4[u];
        r += (k.x < key) + (k.y < key) + (k.z < key) + (k.w < key);
    }
    const size_t o = (size_t)plane * cap + r;
    const int y = (int)key / W;
    px[o] = (int)key - y * W;
    py[o] = y;
    ps[o] = __uint_as_float((uint32_t)e);
}

hipError_t launch_sort_peaks(int32_t *ctr, uint64_t *stage, int cap, int cap2, int planes, int W,
                             const hp_peaks &pk, int32_t *status, hipStream_t s)
{
    const int parts = (cap + kBlock - 1) / kBlock;
    const size_t lds = sizeof(uint32_t) * (size_t)((cap + 3) & ~3);         // <= 64 KB: cap <= HP_MAX_CAP
    HP_KERNEL(k_sort_peaks, dim3(planes, parts), dim3(kBlock), lds, s, ctr, stage, cap, cap2, W, pk.count, pk.x,
                       pk.y, pk.score, status);
    return hipGetLastError();
}

}  // namespace hp
