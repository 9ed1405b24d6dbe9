// Visualisation operator (Section 2.2.1, operator 5): the parsed poses drawn onto the frames.
//
// A limb is the capsule of pixels within thickness / 2 of the segment between its two parts, a part
// the disc of pixels within `radius`; primitives are ordered (person, then the person's limbs in
// table order, then its parts) and a pixel shows the last one that covers it, else the source
// pixel.  All geometry is exact integer arithmetic on frame pixel coordinates.
//
// Two launches.  k_draw_list, one workgroup per image, walks the person table once and writes the
// image's primitives, in painter's order, as 16-byte records (end points in frame coordinates, id,
// and the largest cross product a covered pixel can have) into the workspace, plus one bit per
// frame tile that says whether any primitive can touch it.  k_draw_tiles, one workgroup per tile
// of 64 x 16 pixels, copies untouched tiles and rasterises the others primitive by primitive
// instead of testing every pixel against every primitive: the records are read 512 at a time
// (coalesced), those whose bounding box and line can meet the tile are kept in LDS, and each
// thread then takes (record, row) pairs: the covered pixels of a row are an interval (a capsule
// is convex) whose ends follow exactly from two integer square roots and four exact integer
// divisions, and the thread raises the owner word of each pixel in it to (rank of the record,
// colour id) with an LDS atomic max, which is the painter's order.  A thread finally owns four
// neighbouring pixels, looks up their owners and writes them once.  Testing the pixels of a strip
// against every record that touches it (the first version of this kernel) cost 200 instructions
// per (strip, record) pair for the sixteen or so pixels a thin limb covers there, and that
// arithmetic, not memory, set the kernel's duration.
#include <string.h>

#include "hp_dev.h"

namespace hp {

constexpr int kTileW = 64, kTileH = 16;   // pixels a workgroup paints; a thread owns four neighbouring pixels of a row
static_assert(kTileW * kTileH == 4 * kBlock, "four pixels per thread");

// Per-primitive tables, indexed by id = limb index, or n_limbs + part index.  Passed by value and copied to LDS
// through constant indices: a kernel argument indexed per lane would be unpacked by long select chains.
struct DrawTables {
    uint32_t rgb[HP_MAX_LIMBS + HP_MAX_PARTS];   // r | g << 8 | b << 16
    uint8_t a[HP_MAX_LIMBS], b[HP_MAX_LIMBS];    // the two parts of a limb
};

struct DrawParams {
    int Hf, Wf, H, W, K, L, cap, pcap;
    int thickness, radius;
    int th2_quarter;   // floor(thickness^2 / 4): 4 |u|^2 <= thickness^2 for integer |u|^2
    int reach;         // pixels a limb can extend beyond its end points
    int list_cap;      // records per image in the workspace
    int tiles_x, tiles_y, mask_words;   // tiles of a frame and the 32-bit words of its tile mask
};

// A primitive as the tile kernel reads it.
struct DrawRecord {
    int a, b;     // end points, x | y << 16 in frame pixels (equal for a part)
    int id;       // limb index, or n_limbs + part index
    int cmax;     // limbs: floor(sqrt(thickness^2 |B - A|^2 / 4)), the largest |(P - A) x (B - A)| of a covered pixel
};

// Frame pixel that contains the centre of map pixel x: floor((2x + 1) n_frame / (2 n_map)).  With x inside the map
// (a peak is; anything else is clamped so that the arithmetic stays in range) the product is below 2^30.
__device__ __forceinline__ int to_frame(int x, int n_map, int n_frame)
{
    x = min(max(x, 0), n_map - 1);
    return (int)((unsigned)((2 * x + 1) * n_frame) / (unsigned)(2 * n_map));
}

// End points are frame coordinates below 16384, packed as x | y << 16.
__device__ __forceinline__ int pack_xy(int x, int y) { return x | (y << 16); }
__device__ __forceinline__ int px_of(int v) { return v & 0xFFFF; }
__device__ __forceinline__ int py_of(int v) { return (int)((unsigned)v >> 16); }

// Does the bounding box of segment (a, b), grown by `reach`, meet the rectangle [x0, x0 + w) x [y0, y0 + h)?
__device__ __forceinline__ bool box_meets(int a, int b, int reach, int x0, int y0, int w, int h)
{
    const int ax = px_of(a), ay = py_of(a), bx = px_of(b), by = py_of(b);
    return min(ax, bx) - reach < x0 + w && max(ax, bx) + reach >= x0 && min(ay, by) - reach < y0 + h &&
           max(ay, by) + reach >= y0;
}

// Conservative rejection of a whole rectangle against a limb.  A pixel of the capsule lies within thickness / 2 of
// the line through (a, b), so its cross product with the direction, |(P - A) x (B - A)|, is at most cmax.
// (cx2, cy2) is twice the rectangle's centre, (ex2, ey2) twice its half extents: over the rectangle twice the
// cross product moves by at most ex2 |dy| + ey2 |dx| from its value at the centre.
// Every factor is a difference of coordinates below 16384 (or twice one), so the products are taken with the
// full-rate 24-bit multiplier (a 32-bit integer multiply issues at a quarter of that rate).
__device__ __forceinline__ bool far_from_line(int a, int b, int cmax, int cx2, int cy2, int ex2, int ey2)
{
    const int dx = px_of(b) - px_of(a), dy = py_of(b) - py_of(a);
    const int cross2 = __mul24(cx2 - 2 * px_of(a), dy) - __mul24(cy2 - 2 * py_of(a), dx);
    return abs(cross2) > 2 * cmax + __mul24(ex2, abs(dy)) + __mul24(ey2, abs(dx));
}

constexpr int kListBlock = 1024;   // one workgroup per image walks its persons: as wide as a workgroup gets

__global__ __launch_bounds__(kListBlock) void k_draw_list(const int32_t *__restrict__ peak_x, const int32_t *__restrict__ peak_y,
                                                      const int32_t *__restrict__ slots,
                                                      const int32_t *__restrict__ pose_count, DrawTables tab, DrawParams P,
                                                      DrawRecord *__restrict__ records, int32_t *__restrict__ record_count,
                                                      uint32_t *__restrict__ tile_mask)
{
    __shared__ uint8_t s_part_a[HP_MAX_LIMBS], s_part_b[HP_MAX_LIMBS];
    __shared__ int s_scan[kListBlock / kWave + 1];
    extern __shared__ uint32_t s_mask[];   // one bit per tile: can any primitive touch it?
    const int n = blockIdx.x, tid = threadIdx.x;
    if (tid == 0) {
#pragma unroll
        for (int i = 0; i < HP_MAX_LIMBS; ++i) {
            s_part_a[i] = tab.a[i];
            s_part_b[i] = tab.b[i];
        }
    }
    for (int i = tid; i < P.mask_words; i += kListBlock) s_mask[i] = 0;
    __syncthreads();
    const int per_person = P.L + P.K;
    const int items = min(pose_count[n], P.pcap) * per_person;
    DrawRecord *out = records + (size_t)n * P.list_cap;
    int total = 0;
    for (int base = 0; base < items; base += kListBlock) {
        const int q = base + tid;
        bool keep = false;
        DrawRecord rec = {0, 0, 0, 0};
        if (q < items) {
            const int p = q / per_person;
            rec.id = q - p * per_person;
            const bool limb = rec.id < P.L;
            const int32_t *sl = slots + ((size_t)n * P.pcap + p) * P.K;
            const int a = limb ? s_part_a[rec.id] : rec.id - P.L;
            const int b = limb ? s_part_b[rec.id] : a;
            const int ia = sl[a], ib = sl[b];
            if (ia >= 0 && ib >= 0 && ia < P.cap && ib < P.cap) {
                keep = true;
                const size_t oa = ((size_t)n * P.K + a) * P.cap + ia, ob = ((size_t)n * P.K + b) * P.cap + ib;
                const int ax = to_frame(peak_x[oa], P.W, P.Wf), ay = to_frame(peak_y[oa], P.H, P.Hf);
                const int bx = to_frame(peak_x[ob], P.W, P.Wf), by = to_frame(peak_y[ob], P.H, P.Hf);
                rec.a = pack_xy(ax, ay);
                rec.b = pack_xy(bx, by);
                if (limb) {
                    // an integer cross product c satisfies 4 c^2 <= thickness^2 |B - A|^2 if and only if |c| <= cmax
                    const int dx = bx - ax, dy = by - ay;
                    const long long v = ((long long)P.thickness * P.thickness * (dx * dx + dy * dy)) >> 2;
                    long long r = (long long)sqrt((double)v);
                    while (r * r > v) --r;
                    while ((r + 1) * (r + 1) <= v) ++r;
                    rec.cmax = (int)r;
                }
                const int reach = limb ? P.reach : P.radius;
                const int tx0 = max(min(ax, bx) - reach, 0) / kTileW, tx1 = min((max(ax, bx) + reach) / kTileW, P.tiles_x - 1);
                const int ty0 = max(min(ay, by) - reach, 0) / kTileH, ty1 = min((max(ay, by) + reach) / kTileH, P.tiles_y - 1);
                for (int ty = ty0; ty <= ty1; ++ty)
                    for (int tx = tx0; tx <= tx1; ++tx) {
                        if (limb && far_from_line(rec.a, rec.b, rec.cmax, 2 * tx * kTileW + kTileW - 1,
                                                  2 * ty * kTileH + kTileH - 1, kTileW - 1, kTileH - 1))
                            continue;
                        const int t = ty * P.tiles_x + tx;
                        atomicOr(&s_mask[t >> 5], 1u << (t & 31));
                    }
            }
        }
        int kept;
        const int pos = total + block_flag_scan(keep, s_scan, kept);
        if (keep) out[pos] = rec;
        total += kept;
    }
    if (tid == 0) record_count[n] = total;
    __syncthreads();
    for (int i = tid; i < P.mask_words; i += kListBlock) tile_mask[(size_t)n * P.mask_words + i] = s_mask[i];
}

// floor(n / d) for d > 0, exact: the quotient of two 32-bit integers is either an integer (then the double
// division is exact) or at least 1 / d away from one, far more than a double's rounding error.
__device__ __forceinline__ int floor_div(int n, int d) { return (int)floor((double)n / (double)d); }

// Largest h >= 0 with h * h <= v (v >= 0, below 2^31).
__device__ __forceinline__ int isqrt(int v)
{
    int h = (int)sqrtf((float)v);
    while (h * h > v) --h;
    while ((h + 1) * (h + 1) <= v) ++h;
    return h;
}

// Pixels of row y covered by a record: the interval [xl, xr] (empty when xl > xr), exact.
//   part: |x - ax| <= isqrt(radius^2 - (y - ay)^2);
//   limb: the union of the two end discs (radius^2 -> floor(thickness^2 / 4); a pixel in an end disc is within
//   thickness / 2 of the segment wherever its projection falls) and of the middle part, 0 < t < L2 and |c| <= cmax
//   with t = (P - A).(B - A) and c = (P - A) x (B - A), both linear in x.  The capsule is convex, so the union is
//   one interval: its ends are the smallest left end and the largest right end of the parts present.
__device__ __forceinline__ void row_interval(const DrawRecord &rec, bool limb, int y, int th2_quarter, int r2,
                                             int &xl, int &xr)
{
    const int ax = px_of(rec.a), ay = py_of(rec.a), bx = px_of(rec.b), by = py_of(rec.b);
    xl = 1 << 20;
    xr = -(1 << 20);
    const int uy = y - ay;
    const int remA = (limb ? th2_quarter : r2) - uy * uy;
    if (remA >= 0) {
        const int h = isqrt(remA);
        xl = ax - h;
        xr = ax + h;
    }
    if (!limb) return;
    const int vy = y - by, remB = th2_quarter - vy * vy;
    if (remB >= 0) {
        const int h = isqrt(remB);
        xl = min(xl, bx - h);
        xr = max(xr, bx + h);
    }
    // middle part, in k = x - ax:  -cmax <= k dy - uy dx <= cmax  and  0 < k dx + uy dy < L2
    const int dx = bx - ax, dy = by - ay, L2 = dx * dx + dy * dy;
    const int e = uy * dx, g = uy * dy;
    int lo = -(1 << 20), hi = 1 << 20;
    if (dy > 0) {
        lo = max(lo, -floor_div(rec.cmax - e, dy));       // ceil((e - cmax) / dy)
        hi = min(hi, floor_div(rec.cmax + e, dy));
    } else if (dy < 0) {
        lo = max(lo, -floor_div(rec.cmax + e, -dy));      // ceil((-cmax - e) / -dy)
        hi = min(hi, floor_div(rec.cmax - e, -dy));
    } else if (abs(e) > rec.cmax) {
        return;
    }
    if (dx > 0) {
        lo = max(lo, floor_div(-g, dx) + 1);              // k dx > -g
        hi = min(hi, -floor_div(g - L2, dx) - 1);         // k dx < L2 - g
    } else if (dx < 0) {
        lo = max(lo, floor_div(g - L2, -dx) + 1);         // k (-dx) > g - L2
        hi = min(hi, -floor_div(-g, -dx) - 1);            // k (-dx) < g
    } else if (g <= 0 || g >= L2) {
        return;
    }
    if (lo <= hi) {
        xl = min(xl, ax + lo);
        xr = max(xr, ax + hi);
    }
}

template <int C, bool VEC>
__global__ __launch_bounds__(kBlock) void k_draw_tiles(const uint8_t *src, uint8_t *dst,   // may be the same buffer
                                                       const DrawRecord *__restrict__ records,
                                                       const int32_t *__restrict__ record_count,
                                                       const uint32_t *__restrict__ tile_mask, DrawTables tab,
                                                       DrawParams P)
{
    constexpr int kRound = 2 * kBlock;   // records looked at per round: two per thread, one memory round trip
    __shared__ uint32_t s_rgb[HP_MAX_LIMBS + HP_MAX_PARTS];
    __shared__ DrawRecord s_rec[kRound];            // records that can meet the tile
    __shared__ int s_rank[kRound];                  // their ranks in painter's order
    __shared__ int s_owner[kTileW * kTileH];        // per pixel: (rank + 1) << 7 | id of the last primitive covering it
    __shared__ int s_kept;

    const int n = blockIdx.z;
    const int tid = threadIdx.x;
    const int tile_x0 = blockIdx.x * kTileW, tile_y0 = blockIdx.y * kTileH;
    const int x0 = tile_x0 + 4 * (tid & 15), y = tile_y0 + (tid >> 4);   // this thread's four pixels
    const bool inside = y < P.Hf && x0 < P.Wf;
    const int r2 = P.radius * P.radius;
    // tiles no primitive can touch (most of them) skip the records altogether
    const int tile = blockIdx.y * P.tiles_x + blockIdx.x;
    const int listed = record_count[n];   // read whether needed or not: one memory round trip for both words
    const bool touched = (tile_mask[(size_t)n * P.mask_words + (tile >> 5)] >> (tile & 31)) & 1u;
    const int count = touched ? min(listed, P.list_cap) : 0;
    const DrawRecord *list = records + (size_t)n * P.list_cap;

    // this thread's pixels are on their way while the records are looked at
    const size_t row = ((size_t)n * P.Hf + y) * P.Wf;
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    uint32_t w[4] = {0, 0, 0, 0};
    if (VEC && inside) {
        if (C == 3) {
            const uint32_t *s = (const uint32_t *)(src + (row + x0) * 3);
            w[0] = __builtin_nontemporal_load(s);
            w[1] = __builtin_nontemporal_load(s + 1);
            w[2] = __builtin_nontemporal_load(s + 2);
        } else {
            const v4u v = __builtin_nontemporal_load((const v4u *)(src + (row + x0) * 4));
            w[0] = v[0];
            w[1] = v[1];
            w[2] = v[2];
            w[3] = v[3];
        }
    }

    if (count > 0) {   // the same for every thread
        if (tid == 0) {
            // colours by id; tab is a kernel argument, so the copy goes through constant indices
#pragma unroll
            for (int i = 0; i < HP_MAX_LIMBS + HP_MAX_PARTS; ++i) s_rgb[i] = tab.rgb[i];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) s_owner[4 * tid + j] = 0;
        for (int base = 0; base < count; base += kRound) {
            if (tid == 0) s_kept = 0;
            __syncthreads();
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int q = base + half * kBlock + tid;
                if (q < count) {
                    const DrawRecord rec = list[q];
                    const bool limb = rec.id < P.L;
                    if (box_meets(rec.a, rec.b, limb ? P.reach : P.radius, tile_x0, tile_y0, kTileW, kTileH) &&
                        !(limb && far_from_line(rec.a, rec.b, rec.cmax, 2 * tile_x0 + kTileW - 1,
                                                2 * tile_y0 + kTileH - 1, kTileW - 1, kTileH - 1))) {
                        const int pos = atomicAdd(&s_kept, 1);
                        s_rec[pos] = rec;
                        s_rank[pos] = q;
                    }
                }
            }
            __syncthreads();
            // (record, row) pairs: the covered interval of the row, clipped to the tile, raises the owners
            const int pairs = s_kept * kTileH;
            for (int task = tid; task < pairs; task += kBlock) {
                const int k = task / kTileH, r = task - k * kTileH;
                const DrawRecord rec = s_rec[k];
                int xl, xr;
                row_interval(rec, rec.id < P.L, tile_y0 + r, P.th2_quarter, r2, xl, xr);
                xl = max(xl, tile_x0);
                xr = min(xr, tile_x0 + kTileW - 1);
                const int value = ((s_rank[k] + 1) << 7) | rec.id;
                for (int x = xl; x <= xr; ++x) atomicMax(&s_owner[r * kTileW + x - tile_x0], value);
            }
            __syncthreads();
        }
    }

    if (!inside) return;
    int best[4] = {-1, -1, -1, -1};   // colour id per pixel
    if (count > 0) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int o = s_owner[4 * tid + j];
            best[j] = o ? (o & 127) : -1;
        }
    }
    if (VEC) {
        // four whole pixels: 12 or 16 bytes at a 4-byte (C = 3) or 16-byte (C = 4) aligned address
        if (C == 3) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (best[j] < 0) continue;
                const uint32_t rgb = s_rgb[best[j]];
#pragma unroll
                for (int ch = 0; ch < 3; ++ch) {
                    const int byte = 3 * j + ch;
                    w[byte >> 2] = (w[byte >> 2] & ~(0xFFu << (8 * (byte & 3)))) |
                                   (((rgb >> (8 * ch)) & 0xFFu) << (8 * (byte & 3)));
                }
            }
            uint32_t *d = (uint32_t *)(dst + (row + x0) * 3);
            __builtin_nontemporal_store(w[0], d);
            __builtin_nontemporal_store(w[1], d + 1);
            __builtin_nontemporal_store(w[2], d + 2);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (best[j] >= 0) w[j] = (w[j] & 0xFF000000u) | s_rgb[best[j]];
            v4u v = {w[0], w[1], w[2], w[3]};
            __builtin_nontemporal_store(v, (v4u *)(dst + (row + x0) * 4));
        }
    } else {
        for (int j = 0; j < 4 && x0 + j < P.Wf; ++j) {
            const uint8_t *s = src + (row + x0 + j) * C;
            uint8_t *d = dst + (row + x0 + j) * C;
            uint8_t v[C];
#pragma unroll
            for (int ch = 0; ch < C; ++ch) v[ch] = s[ch];
            if (best[j] >= 0) {
                const uint32_t rgb = s_rgb[best[j]];
#pragma unroll
                for (int ch = 0; ch < 3; ++ch) v[ch] = (uint8_t)(rgb >> (8 * ch));
            }
#pragma unroll
            for (int ch = 0; ch < C; ++ch) d[ch] = v[ch];
        }
    }
}

// Workspace: [N record counts][N tile masks][N x list_cap records], each part on a 256-byte boundary.
static size_t pad256(size_t v) { return (v + 255) / 256 * 256; }
static uint32_t *mask_of(void *workspace, int N) { return (uint32_t *)((char *)workspace + pad256((size_t)N * sizeof(int32_t))); }
static DrawRecord *records_of(void *workspace, int N, int mask_words)
{
    return (DrawRecord *)((char *)mask_of(workspace, N) + pad256((size_t)N * mask_words * sizeof(uint32_t)));
}

size_t draw_workspace_bytes(int N, int K, int L, int pcap, int Hf, int Wf)
{
    const size_t tiles = (size_t)((Wf + kTileW - 1) / kTileW) * ((Hf + kTileH - 1) / kTileH);
    return pad256((size_t)N * sizeof(int32_t)) + pad256((size_t)N * ((tiles + 31) / 32) * sizeof(uint32_t)) +
           (size_t)N * pcap * (K + L) * sizeof(DrawRecord);
}

static void draw_setup(int Hf, int Wf, int H, int W, const LimbTable &T, int K, int L, const hp_peaks &pk,
                       const hp_poses &poses, const uint8_t *limb_rgb, const uint8_t *part_rgb, int thickness, int radius,
                       DrawTables &tab, DrawParams &P)
{
    memset(&tab, 0, sizeof(tab));
    for (int l = 0; l < L; ++l) {
        tab.rgb[l] = limb_rgb[3 * l] | (limb_rgb[3 * l + 1] << 8) | (limb_rgb[3 * l + 2] << 16);
        tab.a[l] = (uint8_t)T.a[l];
        tab.b[l] = (uint8_t)T.b[l];
    }
    for (int c = 0; c < K; ++c) tab.rgb[L + c] = part_rgb[3 * c] | (part_rgb[3 * c + 1] << 8) | (part_rgb[3 * c + 2] << 16);
    P.Hf = Hf;
    P.Wf = Wf;
    P.H = H;
    P.W = W;
    P.K = K;
    P.L = L;
    P.cap = pk.cap;
    P.pcap = poses.cap;
    P.thickness = thickness;
    P.radius = radius;
    P.th2_quarter = (int)(((long long)thickness * thickness) / 4);
    P.reach = (thickness + 1) / 2;
    P.list_cap = poses.cap * (K + L);
    P.tiles_x = (Wf + kTileW - 1) / kTileW;
    P.tiles_y = (Hf + kTileH - 1) / kTileH;
    P.mask_words = (P.tiles_x * P.tiles_y + 31) / 32;
}

hipError_t launch_draw_list(int N, int Hf, int Wf, int H, int W, const LimbTable &T, int K, int L, const hp_peaks &pk,
                            const hp_poses &poses, int thickness, int radius, void *workspace, hipStream_t s)
{
    DrawTables tab;
    DrawParams P;
    const uint8_t none[3 * (HP_MAX_LIMBS + HP_MAX_PARTS)] = {0};   // the list holds no colours
    draw_setup(Hf, Wf, H, W, T, K, L, pk, poses, none, none, thickness, radius, tab, P);
    HP_KERNEL(k_draw_list, dim3(N), dim3(kListBlock), P.mask_words * sizeof(uint32_t), s, pk.x, pk.y, poses.slots, poses.count, tab, P,
              records_of(workspace, N, P.mask_words), (int32_t *)workspace, mask_of(workspace, N));
    return hipGetLastError();
}

hipError_t launch_draw_tiles(const uint8_t *src, uint8_t *dst, int N, int Hf, int Wf, int C, int H, int W,
                             const LimbTable &T, int K, int L, const hp_peaks &pk, const hp_poses &poses,
                             const uint8_t *limb_rgb, const uint8_t *part_rgb, int thickness, int radius,
                             const void *workspace, hipStream_t s)
{
    DrawTables tab;
    DrawParams P;
    draw_setup(Hf, Wf, H, W, T, K, L, pk, poses, limb_rgb, part_rgb, thickness, radius, tab, P);
    const DrawRecord *records = records_of((void *)workspace, N, P.mask_words);
    const int32_t *record_count = (const int32_t *)workspace;
    const uint32_t *tile_mask = mask_of((void *)workspace, N);
    const dim3 grid((Wf + kTileW - 1) / kTileW, (Hf + kTileH - 1) / kTileH, N);
    const uintptr_t bits = (uintptr_t)src | (uintptr_t)dst;
    const bool vec = (Wf % 4) == 0 && (bits & (C == 4 ? 15 : 3)) == 0;
    if (C == 3) {
        if (vec)
            HP_KERNEL((k_draw_tiles<3, true>), grid, dim3(kBlock), 0, s, src, dst, records, record_count, tile_mask, tab, P);
        else
            HP_KERNEL((k_draw_tiles<3, false>), grid, dim3(kBlock), 0, s, src, dst, records, record_count, tile_mask, tab, P);
    } else {
        if (vec)
            HP_KERNEL((k_draw_tiles<4, true>), grid, dim3(kBlock), 0, s, src, dst, records, record_count, tile_mask, tab, P);
        else
            HP_KERNEL((k_draw_tiles<4, false>), grid, dim3(kBlock), 0, s, src, dst, records, record_count, tile_mask, tab, P);
    }
    return hipGetLastError();
}

}  // namespace hp
