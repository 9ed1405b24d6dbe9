// Optional smoothing of the upsampled confidence maps before the peak search: a separable
// correlation with a caller-supplied odd-length tap vector, edge pixels repeated beyond the
// borders, fp32, horizontal pass first, every sum accumulated from 0 in ascending tap order with
// one fused multiply-add per tap (so the result is defined bit for bit).
//
// One workgroup produces a tile of 64 x 64 outputs in one launch, the horizontally filtered rows
// living only in LDS.  Horizontal pass: the tile's source rows (64 + 2r of them, 64 + 2r wide) are
// staged in LDS 32 at a time, sixteen loads per lane in flight, one coalesced row per wavefront
// load; a thread filters four neighbouring outputs of a row from a sliding window held in
// registers (two 16-byte LDS reads per four taps, sixteen multiply-adds).  Vertical pass: a thread
// walks down one column of the filtered rows, four outputs at a time, with the same window scheme,
// and stores rows 256 bytes wide.  The usual tap counts (5, 9, 13, 17, 25) are compiled in: the
// loops over taps unroll completely and the taps stay in scalar registers, which took the 17-tap
// case from 170 to 104 us; any other odd count up to 65 runs the same code with run-time loops.
// With 17 taps the kernel does 38 multiply-adds and moves 8 bytes per output pixel and reaches
// about 40 % of both the fp32 vector rate and the HBM peak; switching one phase off at a time shows
// loading, the horizontal and the vertical pass adding up rather than overlapping.
#include <algorithm>
#include <type_traits>

#include "hp_dev.h"

namespace hp {

constexpr int kSmoothTile = 64;      // outputs per tile row: 16 threads x 4 (horizontal pass), 64 threads (vertical pass)
constexpr int kSmoothTileH = 64;     // output rows per tile (measured at 17 taps, 8 x 18 maps of 368 x 656: 64 x 32 tiles
                                     // 96-113 us, 64 x 64 and 64 x 128 tiles 87 us with 512 threads, 103 us with 256)
constexpr int kSmoothBlock = 512;    // threads per workgroup
constexpr int kSmoothWaves = kSmoothBlock / kWave;
constexpr int kSmoothHRows = kSmoothBlock / 16;     // rows filtered per step of the horizontal pass (16 threads a row)
constexpr int kSmoothVRows = kSmoothTileH / kSmoothWaves;   // output rows per thread in the vertical pass
static_assert(kSmoothVRows % 4 == 0, "the vertical pass produces four outputs at a time");
constexpr int kSmoothMaxR = 32;      // largest radius: 65 taps
constexpr int kSmoothStageFloats = 4096;   // LDS given to the staged source rows: 32 rows at a time (with room for the
                                           // whole tile, 32 KB, a compute unit held a workgroup less and the kernel took 104 us
                                           // instead of 87)

// TC: the number of taps when it is known at compile time (the loops over taps then unroll completely and the taps
// stay in scalar registers), 0 for any number of taps.
template <int TC>
__global__ __launch_bounds__(kSmoothBlock) void k_smooth(const float *__restrict__ src, float *__restrict__ dst, int C,
                                                   int C_mem, int H, int W, const float *__restrict__ taps, int T_any)
{
    const int T = TC ? TC : T_any;
    __shared__ __attribute__((aligned(16))) float s_taps[2 * kSmoothMaxR + 4];   // read four at a time
    extern __shared__ __attribute__((aligned(16))) float s_dyn[];
    float *s_t = s_dyn;                                   // [tile rows + 2r][64] horizontally filtered rows
    float *s_src = s_dyn + (kSmoothTileH + 2 * ((T - 1) >> 1)) * kSmoothTile;   // [stage rows][pitch] source rows (+ 8 floats)

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
    const int r = (T - 1) >> 1;
    const int plane = blockIdx.z;
    const size_t plane_off = ((size_t)(plane / C) * C_mem + plane % C) * H * W;
    const float *s = src + plane_off;
    float *d = dst + plane_off;
    const int x0 = blockIdx.x * kSmoothTile, y0 = blockIdx.y * kSmoothTileH;
    const int rows = kSmoothTileH + 2 * r, cols = kSmoothTile + 2 * r;

    if (tid < 2 * kSmoothMaxR + 4) s_taps[tid] = tid < T ? taps[tid] : 0.0f;

    // ---- horizontal pass into s_t -------------------------------------------------------------
    // rows staged at a time: a multiple of the rows filtered per step (16 threads x 4 outputs a row); the pitch is a multiple
    // of 4 floats so that windows are read 16 bytes at a time, and the last window's unused tail (up to 7 floats
    // beyond a row) stays inside the array
    const int pitch = (cols + 3) & ~3;
    const int stage = min((kSmoothStageFloats / pitch) & ~(kSmoothHRows - 1), (rows + kSmoothHRows - 1) & ~(kSmoothHRows - 1));
    const int hr = tid >> 4, hx = 4 * (tid & 15);   // this thread's row of a step and its four outputs
    for (int rs = 0; rs < rows; rs += stage) {
        __syncthreads();   // the previous stage has been consumed (and s_taps is in place)
        // a wavefront stages rows wv, wv + 4, ...: eight rows (sixteen loads per lane) are in flight at a time
        const int xa = min(max(x0 - r + lane, 0), W - 1), xb = min(max(x0 - r + lane + kWave, 0), W - 1);
        const bool second = lane + kWave < cols;   // a staged row is 64 + 2r <= 128 floats: at most two per lane
        for (int rr0 = wv; rr0 < stage && rs + rr0 < rows; rr0 += 8 * kSmoothWaves) {
            float va[8], vb[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int rr = rr0 + u * kSmoothWaves;
                const float *line = s + (size_t)min(max(y0 - r + rs + rr, 0), H - 1) * W;   // clamped: always readable
                va[u] = line[xa];
                vb[u] = second ? line[xb] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int rr = rr0 + u * kSmoothWaves;
                if (rr < stage && rs + rr < rows) {
                    s_src[rr * pitch + lane] = va[u];
                    if (second) s_src[rr * pitch + lane + kWave] = vb[u];
                }
            }
        }
        __syncthreads();
        for (int row = hr; row < stage && rs + row < rows; row += kSmoothHRows) {
            float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            const float *win = &s_src[row * pitch + hx];
            float4 lo = *(const float4 *)win;
#pragma unroll
            for (int i = 0; i < T; i += 4) {
                const float4 hi = *(const float4 *)(win + i + 4);
                const float4 t4 = *(const float4 *)&s_taps[i];
                const float w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                const float tp[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    if (i + m < T) {   // the same for every thread
                        const float tap = TC ? taps[TC ? i + m : 0] : tp[m];
#pragma unroll
                        for (int o = 0; o < 4; ++o) acc[o] = __fmaf_rn(tap, w[o + m], acc[o]);
                    }
                }
                lo = hi;
            }
            *(float4 *)&s_t[(rs + row) * kSmoothTile + hx] = make_float4(acc[0], acc[1], acc[2], acc[3]);
        }
    }
    __syncthreads();

    // ---- vertical pass out of s_t ----------------------------------------------------------------
    const int vx = tid & (kSmoothTile - 1), vg = tid >> 6;   // this thread's column and its rows
    if (x0 + vx >= W) return;
#pragma unroll 1
    for (int k = 0; k < kSmoothVRows / 4; ++k) {
        const int yo = kSmoothVRows * vg + 4 * k;   // four outputs: tile rows yo .. yo + 3
        if (y0 + yo >= H) break;
        float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        float w[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) w[j] = s_t[(yo + j) * kSmoothTile + vx];
#pragma unroll
        for (int i = 0; i < T; i += 4) {
#pragma unroll
            for (int j = 0; j < 4; ++j) w[4 + j] = (yo + i + 4 + j < rows) ? s_t[(yo + i + 4 + j) * kSmoothTile + vx] : 0.0f;
            const float4 t4 = *(const float4 *)&s_taps[i];
            const float tp[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                if (i + m < T) {
                    const float tap = TC ? taps[TC ? i + m : 0] : tp[m];
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

// The marching form, for the usual tap counts on maps whose rows are whole 16-byte groups.  A wavefront owns a
// strip of a band of rows and walks down it one source row at a time; its 64 lanes hold 256 neighbouring columns, four
// a lane, of which the outer rp on either side (r rounded up to whole 16-byte pieces) are only read: neighbouring
// strips overlap by that much, so a lane never fetches anything but its own piece.  A step: the row's 16-byte pieces
// (fetched kMarchAhead steps earlier into registers) go to a row buffer in the wavefront's
// own LDS; every lane reads back its window of 4 + 2 rp values and filters its four outputs horizontally; the
// filtered values are then added, tap by tap, to the T output rows they belong to, whose running sums live in
// registers; the output row whose last tap this was is stored.  A sum receives its taps in the order the source rows
// arrive, which is ascending tap order, starting from 0: the same bits as the definition.
// The row loop is unrolled T-fold (a multiple of it for few taps) so that every register has a fixed name, and a
// step is straight-line code, the same for every lane (columns outside the map read the clamped piece and repeat its
// edge pixel), so that the loads of later rows stay in flight across it.  No workgroup barrier, one LDS write and
// (4 + 2 rp) / 4 LDS reads per row and lane against 8 T multiply-adds, no horizontally filtered row is computed twice
// except the 2r rows between two bands, and the stores are whole rows.
// (With separate loads for the pieces left and right of a strip, kept in registers like the others, the 17-tap kernel
// needed 276 registers: one wavefront a SIMD, 95 us for the benchmark's maps.)
constexpr int kMarchBlock = 256, kMarchWaves = kMarchBlock / kWave;

// f(integral_constant<0>), f(integral_constant<1>), ...: a loop whose counter is a constant in every round
template <int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(std::integral_constant<int, N - 1>{});
    }
}

constexpr int kMarchAhead = 6;        // rows a wavefront has under way: a row is fetched this many steps before its turn
template <int T>
__global__ __launch_bounds__(kMarchBlock) __attribute__((amdgpu_waves_per_eu(1, 3))) void k_smooth_march(const float *__restrict__ src, float *__restrict__ dst, int C,
                                                              int C_mem, int H, int W, const float *__restrict__ taps,
                                                              int strips, int sw, int bands, int band)
{
    constexpr int r = (T - 1) / 2, rp = (r + 3) & ~3, o0 = rp - r;
    constexpr int U = T * ((10 + T - 1) / T);            // rows per pass through the unrolled loop (16 bytes x U in registers)
    constexpr int kWin = 2 * rp + 4;                     // floats a lane reads back per row
    constexpr int kBuf = 4 * kWave + 2 * rp;             // floats per row buffer: rp never written on either side
    __shared__ __attribute__((aligned(16))) float bufs[kMarchWaves][kBuf];
    const int lane = threadIdx.x & (kWave - 1), wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int task = blockIdx.x * kMarchWaves + wv;
    if (task >= strips * bands) return;
    const int strip = task % strips, bandi = task / strips;
    const int plane = blockIdx.z;
    const size_t plane_off = ((size_t)(plane / C) * C_mem + plane % C) * H * W;
    const float *s = src + plane_off;
    float *d = dst + plane_off;
    const int x0 = strip * sw, y_start = bandi * band;   // the strip's first output column, the band's first row
    if (x0 >= W || y_start >= H) return;
    const int y_end = min(y_start + band, H);
    const int sw_valid = min(sw, W - x0);                // output columns: a multiple of 4, at least 4
    const int X = x0 - rp + 4 * lane;                    // this lane's four columns
    const bool writes = X >= x0 && X < x0 + sw_valid;
    // a piece lies wholly inside the map or wholly outside it; outside, the edge pixel is repeated
    const bool before = X < 0, beyond = X >= W;
    const int x_ld = min(max(X, 0), W - 4);
    float *buf = bufs[wv];

    typedef float v4f __attribute__((ext_vector_type(4)));
    v4f pre[U];
    auto load_row = [&](int yy, v4f &m) { m = *(const v4f *)(s + (size_t)min(max(yy, 0), H - 1) * W + x_ld); };
    auto edge_fix = [&](const v4f &m) {
        const float e = before ? m.x : m.w;
        const v4f rep = {e, e, e, e};
        return (before || beyond) ? rep : m;
    };
    const int n_steps = (y_end - y_start) + 2 * r;       // source rows y_start - r .. y_end - 1 + r, clamped to the map
    constexpr int P = kMarchAhead;
    static_assert(P <= U, "a slot is refilled after its turn");
#pragma unroll
    for (int u = 0; u < P; ++u) load_row(y_start - r + u, pre[u]);

    float ring[T][4];
#pragma unroll
    for (int j = 0; j < T; ++j)
#pragma unroll
        for (int o = 0; o < 4; ++o) ring[j][o] = 0.0f;

    for (int base = 0; base < n_steps; base += U) {
        static_for<U>([&](auto uc) {
            constexpr int u = decltype(uc)::value;
            const int step = base + u;                   // steps beyond n_steps (the last pass of a band) store nothing
            *(v4f *)&buf[rp + 4 * lane] = edge_fix(pre[u]);
            load_row(y_start - r + step + P, pre[(u + P) % U]);
            // LDS serves a wavefront's requests in order: the reads below see the writes above
            __builtin_amdgcn_wave_barrier();
            float win[kWin];
#pragma unroll
            for (int q = 0; q < kWin / 4; ++q) {
                const v4f v = *(const v4f *)&buf[4 * lane + 4 * q];
                win[4 * q] = v.x;
                win[4 * q + 1] = v.y;
                win[4 * q + 2] = v.z;
                win[4 * q + 3] = v.w;
            }
            __builtin_amdgcn_wave_barrier();
            float t4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int i = 0; i < T; ++i) {
                const float tap = taps[i];
#pragma unroll
                for (int o = 0; o < 4; ++o) t4[o] = __fmaf_rn(tap, win[o0 + o + i], t4[o]);
            }
            // this row is tap j of the output row that started j steps ago
#pragma unroll
            for (int j = 0; j < T; ++j) {
                const float tap = taps[j];
                constexpr int kBig = 4 * T;
                const int slot = (u % T - j + kBig) % T;     // a constant once the loop over j is unrolled
#pragma unroll
                for (int o = 0; o < 4; ++o) ring[slot][o] = __fmaf_rn(tap, t4[o], j == 0 ? 0.0f : ring[slot][o]);
            }
            if (step >= 2 * r && step < n_steps && writes) {
                const int slot = (u % T + 1) % T;        // the row that has just received its last tap
                const v4f out = {ring[slot][0], ring[slot][1], ring[slot][2], ring[slot][3]};
                __builtin_nontemporal_store(out, (v4f *)&d[(size_t)(y_start + step - 2 * r) * W + X]);
            }
        });
    }
}

// Rows staged at a time and the floats between staged rows, for radius r (the kernel derives the same two numbers).
static void smooth_stage(int r, int &stage, int &pitch)
{
    const int rows = kSmoothTileH + 2 * r, cols = kSmoothTile + 2 * r;
    pitch = (cols + 3) & ~3;
    stage = std::min((kSmoothStageFloats / pitch) & ~(kSmoothHRows - 1), (rows + kSmoothHRows - 1) & ~(kSmoothHRows - 1));
}

hipError_t launch_smooth(const float *src, float *dst, int N, int C, int C_mem, int H, int W, const float *taps,
                         int n_taps, hipStream_t s)
{
    const int r = (n_taps - 1) / 2;
    // The marching kernel serves the tap counts it is compiled for (measured on 8 x 18 maps of 368 x 656 / 4 x 18 maps of
    // 1080 x 1920, tile kernel -> marching kernel): 5 taps 62 -> 46 / 267 -> 238 us, 9 taps 68 -> 52 / 279 -> 244, 13 taps
    // 75 -> 58 / 304 -> 247, 17 taps 87 -> 74 / 355 -> 270 (161 registers a lane).
    const bool march_pays = n_taps == 5 || n_taps == 9 || n_taps == 13 || n_taps == 17;
    if (march_pays && W % 4 == 0 && ((((uintptr_t)src) | ((uintptr_t)dst)) & 15) == 0) {
        // strips of equal width (a multiple of 4; with the columns read on either side, at most 256); bands so that
        // about two wavefronts per SIMD are under way: fewer would leave the memory system idle, more would filter more
        // rows twice (2r per band)
        const int rp = (r + 3) & ~3, sw_max = 4 * kWave - 2 * rp;
        const int strips = (W + sw_max - 1) / sw_max;
        const int sw = ((W + strips - 1) / strips + 3) & ~3;
        for (int p0 = 0; p0 < N * C; p0 += 65535 / C * C) {
            const int planes = std::min(N * C - p0, 65535 / C * C);
            const size_t off = (size_t)(p0 / C) * C_mem * H * W;
            // two wavefronts per SIMD, 2048 on 256 compute units, measured best although three fit at 17 taps and more
            // at fewer: 5, 6 and 7 bands on the first of the shapes above (2160, 2592, 3024 wavefronts) took 88, 75 and
            // 93 us against 74 with 4 bands (1728)
            const long long columns = (long long)strips * planes;
            int bands = (int)std::min<long long>((H + 15) / 16, std::max<long long>(1, 2048 / columns));
            const int band = (H + bands - 1) / bands;
            bands = (H + band - 1) / band;
            const dim3 grid((strips * bands + kMarchWaves - 1) / kMarchWaves, 1, planes);
#define HP_MARCH_CASE(T_)                                                                                             \
    case T_:                                                                                                         \
        HP_KERNEL(k_smooth_march<T_>, grid, dim3(kMarchBlock), 0, s, src + off, dst + off, C, C_mem, H, W, taps, strips, sw, \
                  bands, band);                                                                                      \
        break;
            switch (n_taps) {
                HP_MARCH_CASE(5)
                HP_MARCH_CASE(9)
                HP_MARCH_CASE(13)
                HP_MARCH_CASE(17)
            }
#undef HP_MARCH_CASE
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    int stage, pitch;
    smooth_stage(r, stage, pitch);
    const size_t lds = sizeof(float) * ((size_t)(kSmoothTileH + 2 * r) * kSmoothTile + (size_t)stage * pitch + 8);
    // grid.z carries the planes: at most 65535 per launch
    for (int p0 = 0; p0 < N * C; p0 += 65535 / C * C) {
        const int planes = std::min(N * C - p0, 65535 / C * C);
        const size_t off = (size_t)(p0 / C) * C_mem * H * W;
        const dim3 grid((W + kSmoothTile - 1) / kSmoothTile, (H + kSmoothTileH - 1) / kSmoothTileH, planes);
#define HP_SMOOTH_CASE(TC_)                                                                                            \
    case TC_:                                                                                                      \
        HP_KERNEL(k_smooth<TC_>, grid, dim3(kSmoothBlock), lds, s, src + off, dst + off, C, C_mem, H, W, taps, n_taps); \
        break;
        switch (n_taps) {
            HP_SMOOTH_CASE(5)
            HP_SMOOTH_CASE(9)
            HP_SMOOTH_CASE(13)
            HP_SMOOTH_CASE(17)
            HP_SMOOTH_CASE(25)
        default:
            HP_KERNEL(k_smooth<0>, grid, dim3(kSmoothBlock), lds, s, src + off, dst + off, C, C_mem, H, W, taps, n_taps);
        }
#undef HP_SMOOTH_CASE
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace hp
