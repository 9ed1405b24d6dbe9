// Visualisation operator (Section 2.2.1, operator 5): the parsed poses drawn onto the frames.
//
// A limb is the capsule of pixels within thickness / 2 of the segment between its two parts, a part
// the disc of pixels within `radius`; primitives are ordered (person, then the person's limbs in
// table order, then its parts) and a pixel shows the last one that covers it, else the source
// pixel.  All geometry is exact integer arithmetic on frame pixel coordinates.
//
// Two launches.  k_draw_list, one workgroup per image, walks the person table once and writes the
// image's primitives, in painter's order, as 16-byte records (end points in frame coordinates, id,
// and the largest cross product a covered pixel can have) into the workspace; it also hands each
// record, with its rank in that order, to every frame tile its capsule can touch (a count and up
// to kTileCap records per tile).  k_draw_tiles, one workgroup per tile of 128 x 16 pixels, copies
// tiles nothing was handed to and rasterises the others primitive by primitive instead of testing
// every pixel against every primitive: each thread takes (record, row) pairs: the covered pixels
// of a row are an interval (a capsule is convex) whose ends follow exactly from two integer square
// roots and four exact integer divisions, and the thread raises the owner word of each pixel in it
// to (rank of the record, colour id) with an LDS atomic max, which is the painter's order.  A
// thread finally looks up the owners of its own pixels and writes them once.  A
// tile that was handed more records than it can hold goes through the image's whole list instead,
// 512 records at a time, keeping those whose bounding box and line can meet it (every touched tile
// did that at first: with a thousand records an image the tests were 10 us of arithmetic, and the
// list cost a tile a second memory round trip).  Testing the pixels of a strip against every
// record that touches it (the first version of this kernel) cost 200 instructions per (strip,
// record) pair for the sixteen or so pixels a thin limb covers there.
#include <string.h>

#include "hp_dev.h"

namespace hp {

// Frames are read and written with ordinary loads and stores: non-temporal ones took a sixth longer (17.9 against
// 15.1 us for the benchmark's 64 frames with nothing to draw).
#define DRAW_ST(v, p) (*(p) = (v))
#define DRAW_LD(p) (*(p))

// Pixels a workgroup paints.  A thread owns kTileGroups groups of four neighbouring pixels, 64 pixels apart in a
// row and 16 rows apart: sixteen threads fetch 64 neighbouring pixels of a row at a time.  (The kernel waits for its
// pixels once per workgroup: a tile of 64 x 16 took the benchmark's frames 25 us, one of 128 x 16 21 us.)
constexpr int kTileW = 128, kTileH = 16, kTileGroupsX = kTileW / 64, kTileGroups = kTileGroupsX * (kTileH / 16);
static_assert(kTileW * kTileH == 4 * kTileGroups * kBlock, "kTileGroups groups of four pixels a thread");
constexpr int kTileCap = 64;              // records a tile can be handed; with more it reads the image's list itself
constexpr int kListBinTiles = 8192;       // k_draw_list counts a frame's tiles in LDS up to this many, else in the workspace
static_assert(kTileCap <= kBlock && HP_MAX_LIMBS + HP_MAX_PARTS <= kBlock, "a thread fetches one of its tile's records and one colour");

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
    int tiles_x, tiles_y, tiles;        // tiles of a frame
};

// A primitive as the tile kernel reads it.
struct DrawRecord {
    int a, b;     // end points, x | y << 16 in frame pixels (equal for a part)
    int id;       // limb index, or n_limbs + part index; in a tile's records: id | rank in painter's order << 7
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
                                                      int32_t *__restrict__ tile_count, DrawRecord *__restrict__ tile_records,
                                                      uint32_t *__restrict__ rgb_table)
{
    __shared__ uint8_t s_part_a[HP_MAX_LIMBS], s_part_b[HP_MAX_LIMBS];
    __shared__ int s_scan[kListBlock / kWave + 1];
    extern __shared__ int s_tiles[];   // records handed to each tile so far (frames of up to kListBinTiles tiles)
    const int n = blockIdx.x, tid = threadIdx.x;
    if (tid == 0) {
#pragma unroll
        for (int i = 0; i < HP_MAX_LIMBS; ++i) {
            s_part_a[i] = tab.a[i];
            s_part_b[i] = tab.b[i];
        }
        if (n == 0) {
            // the colours by id, where every tile can fetch them with its first loads
#pragma unroll
            for (int i = 0; i < HP_MAX_LIMBS + HP_MAX_PARTS; ++i) rgb_table[i] = tab.rgb[i];
        }
    }
    int32_t *const tile_count_n = tile_count + (size_t)n * P.tiles;
    const bool in_lds = P.tiles <= kListBinTiles;
    int *const handed = in_lds ? s_tiles : tile_count_n;
    for (int i = tid; i < P.tiles; i += kListBlock) handed[i] = 0;
    if (!in_lds) __threadfence();   // the zeros are in place before another thread's atomic finds the word
    __syncthreads();
    const int per_person = P.L + P.K;
    const int items = min(pose_count[n], P.pcap) * per_person;
    DrawRecord *out = records + (size_t)n * P.list_cap;
    int total = 0;
    for (int base = 0; base < items; base += kListBlock) {
        const int q = base + tid;
        bool keep = false;
        DrawRecord rec = {0, 0, 0, 0};
        int ax = 0, ay = 0, bx = 0, by = 0;
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
                ax = to_frame(peak_x[oa], P.W, P.Wf), ay = to_frame(peak_y[oa], P.H, P.Hf);
                bx = to_frame(peak_x[ob], P.W, P.Wf), by = to_frame(peak_y[ob], P.H, P.Hf);
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
            }
        }
        int kept;
        const int pos = total + block_flag_scan(keep, s_scan, kept);
        total += kept;
        if (keep) {
            out[pos] = rec;
            // the tiles its bounding box meets, less those its line stays clear of, get it with its rank
            const bool limb = rec.id < P.L;
            DrawRecord ranked = rec;
            ranked.id = rec.id | (pos << 7);
            const int reach = limb ? P.reach : P.radius;
            const int tx0 = max(min(ax, bx) - reach, 0) / kTileW, tx1 = min((max(ax, bx) + reach) / kTileW, P.tiles_x - 1);
            const int ty0 = max(min(ay, by) - reach, 0) / kTileH, ty1 = min((max(ay, by) + reach) / kTileH, P.tiles_y - 1);
            for (int ty = ty0; ty <= ty1; ++ty)
                for (int tx = tx0; tx <= tx1; ++tx) {
                    if (limb && far_from_line(rec.a, rec.b, rec.cmax, 2 * tx * kTileW + kTileW - 1,
                                              2 * ty * kTileH + kTileH - 1, kTileW - 1, kTileH - 1))
                        continue;
                    const int t = ty * P.tiles_x + tx;
                    const int at = atomicAdd(&handed[t], 1);
                    if (at < kTileCap) tile_records[((size_t)n * P.tiles + t) * kTileCap + at] = ranked;
                }
        }
    }
    if (tid == 0) record_count[n] = total;
    if (in_lds) {
        __syncthreads();
        for (int i = tid; i < P.tiles; i += kListBlock) tile_count_n[i] = s_tiles[i];
    }
}

// floor(n / d) for d > 0, exact: the quotient of two 32-bit integers is either an integer (then the double
// division is exact) or at least 1 / d away from one, far more than a double's rounding error.  (A single-precision
// estimate put right by the remainder was no faster: the kernel does not wait for this arithmetic.)
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
                                                       const int32_t *__restrict__ tile_count,
                                                       const DrawRecord *__restrict__ tile_records,
                                                       const uint32_t *__restrict__ rgb_table, DrawParams P)
{
    constexpr int kRound = 2 * kBlock;   // records of the image's list looked at per round: two per thread
    __shared__ uint32_t s_rgb[HP_MAX_LIMBS + HP_MAX_PARTS];
    __shared__ DrawRecord s_rec[kRound];            // records that can meet the tile
    __shared__ int s_rank[kRound];                  // their ranks in painter's order
    __shared__ int s_owner[kTileW * kTileH];        // per pixel: (rank + 1) << 7 | id of the last primitive covering it
    __shared__ int s_kept;

    const int n = blockIdx.z;
    const int tid = threadIdx.x;
    const int tile_x0 = blockIdx.x * kTileW, tile_y0 = blockIdx.y * kTileH;
    // this thread's pixels: group g is (gx(g) + 0..3, gy(g))
    auto gx = [&](int g) { return tile_x0 + 4 * (tid & 15) + 64 * (g % kTileGroupsX); };
    auto gy = [&](int g) { return tile_y0 + (tid >> 4) + 16 * (g / kTileGroupsX); };
    auto grow = [&](int g) { return ((size_t)n * P.Hf + gy(g)) * P.Wf + gx(g); };   // pixel index of the group's first
    const int r2 = P.radius * P.radius;
    // what the tile was handed: the count, and one record a thread, fetched whether it exists or not (the slot does),
    // so that one memory round trip brings the count, the records and the pixels
    const size_t tile = (size_t)n * P.tiles + blockIdx.y * P.tiles_x + blockIdx.x;
    const int handed = tile_count[tile];
    DrawRecord mine = {0, 0, 0, 0};
    if (tid < kTileCap) mine = tile_records[tile * kTileCap + tid];
    const uint32_t colour = tid < HP_MAX_LIMBS + HP_MAX_PARTS ? rgb_table[tid] : 0u;   // r | g << 8 | b << 16 of id `tid`

    // this thread's pixels are on their way meanwhile
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    uint32_t w[kTileGroups][4];
#pragma unroll
    for (int g = 0; g < kTileGroups; ++g) {
        w[g][0] = w[g][1] = w[g][2] = w[g][3] = 0;
        if (VEC && gy(g) < P.Hf && gx(g) < P.Wf) {
            if (C == 3) {
                const uint32_t *s = (const uint32_t *)(src + grow(g) * 3);
                w[g][0] = DRAW_LD(s);
                w[g][1] = DRAW_LD(s + 1);
                w[g][2] = DRAW_LD(s + 2);
            } else {
                const v4u v = DRAW_LD((const v4u *)(src + grow(g) * 4));
                w[g][0] = v[0];
                w[g][1] = v[1];
                w[g][2] = v[2];
                w[g][3] = v[3];
            }
        }
    }

    // (record, row) pairs of the first `kept` records in LDS: the covered interval of the row, clipped to the tile,
    // raises the owners
    auto paint = [&](int kept) {
        const int pairs = kept * kTileH;
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
    };

    if (handed > 0) {   // the same for every thread
        if (tid < HP_MAX_LIMBS + HP_MAX_PARTS) s_rgb[tid] = colour;
#pragma unroll
        for (int j = 0; j < 4 * kTileGroups; ++j) s_owner[j * kBlock + tid] = 0;
        if (handed <= kTileCap) {
            if (tid < handed) {
                s_rank[tid] = mine.id >> 7;
                mine.id &= 127;
                s_rec[tid] = mine;
            }
            __syncthreads();
            paint(handed);
            __syncthreads();
        } else {
            // more than the tile could hold: the image's whole list, a round at a time
            const int count = min(record_count[n], P.list_cap);
            const DrawRecord *list = records + (size_t)n * P.list_cap;
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
                paint(s_kept);
                __syncthreads();
            }
        }
    }

#pragma unroll
    for (int g = 0; g < kTileGroups; ++g) {
        const int xg = gx(g);
        if (xg >= P.Wf || gy(g) >= P.Hf) continue;
        const size_t row = grow(g) - xg;
        int best[4] = {-1, -1, -1, -1};   // colour id per pixel
        if (handed > 0) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int o = s_owner[(gy(g) - tile_y0) * kTileW + xg - tile_x0 + j];
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
                        w[g][byte >> 2] = (w[g][byte >> 2] & ~(0xFFu << (8 * (byte & 3)))) |
                                          (((rgb >> (8 * ch)) & 0xFFu) << (8 * (byte & 3)));
                    }
                }
                uint32_t *d = (uint32_t *)(dst + (row + xg) * 3);
                DRAW_ST(w[g][0], d);
                DRAW_ST(w[g][1], d + 1);
                DRAW_ST(w[g][2], d + 2);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (best[j] >= 0) w[g][j] = (w[g][j] & 0xFF000000u) | s_rgb[best[j]];
                v4u v = {w[g][0], w[g][1], w[g][2], w[g][3]};
                DRAW_ST(v, (v4u *)(dst + (row + xg) * 4));
            }
        } else {
            for (int j = 0; j < 4 && xg + j < P.Wf; ++j) {
                const uint8_t *s = src + (row + xg + j) * C;
                uint8_t *d = dst + (row + xg + j) * C;
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
}

// Workspace: [colours by id][N record counts][N x tiles tile counts][N x list_cap records][N x tiles x kTileCap tile records], each
// part on a 256-byte boundary.
static size_t pad256(size_t v) { return (v + 255) / 256 * 256; }
static size_t frame_tiles(int Hf, int Wf) { return (size_t)((Wf + kTileW - 1) / kTileW) * ((Hf + kTileH - 1) / kTileH); }
struct DrawWork {
    uint32_t *rgb_table;
    int32_t *record_count, *tile_count;
    DrawRecord *records, *tile_records;
    size_t bytes;
};
static DrawWork draw_layout(void *workspace, int N, int list_cap, size_t tiles)
{
    DrawWork w;
    char *p = (char *)workspace;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *q = p ? p + off : nullptr;
        off += pad256(bytes);
        return q;
    };
    w.rgb_table = (uint32_t *)take((HP_MAX_LIMBS + HP_MAX_PARTS) * sizeof(uint32_t));
    w.record_count = (int32_t *)take((size_t)N * sizeof(int32_t));
    w.tile_count = (int32_t *)take((size_t)N * tiles * sizeof(int32_t));
    w.records = (DrawRecord *)take((size_t)N * list_cap * sizeof(DrawRecord));
    w.tile_records = (DrawRecord *)take((size_t)N * tiles * kTileCap * sizeof(DrawRecord));
    w.bytes = off;
    return w;
}

size_t draw_workspace_bytes(int N, int K, int L, int pcap, int Hf, int Wf)
{
    return draw_layout(nullptr, N, pcap * (K + L), frame_tiles(Hf, Wf)).bytes;
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
    P.tiles = P.tiles_x * P.tiles_y;
}

hipError_t launch_draw_list(int N, int Hf, int Wf, int H, int W, const LimbTable &T, int K, int L, const hp_peaks &pk,
                            const hp_poses &poses, const uint8_t *limb_rgb, const uint8_t *part_rgb, int thickness,
                            int radius, void *workspace, hipStream_t s)
{
    DrawTables tab;
    DrawParams P;
    draw_setup(Hf, Wf, H, W, T, K, L, pk, poses, limb_rgb, part_rgb, thickness, radius, tab, P);
    const DrawWork ws = draw_layout(workspace, N, P.list_cap, (size_t)P.tiles);
    const size_t lds = P.tiles <= kListBinTiles ? (size_t)P.tiles * sizeof(int) : 0;
    HP_KERNEL(k_draw_list, dim3(N), dim3(kListBlock), lds, s, pk.x, pk.y, poses.slots, poses.count, tab, P, ws.records,
              ws.record_count, ws.tile_count, ws.tile_records, ws.rgb_table);
    return hipGetLastError();
}

hipError_t launch_draw_tiles(const uint8_t *src, uint8_t *dst, int N, int Hf, int Wf, int C, int H, int W,
                             const LimbTable &T, int K, int L, const hp_peaks &pk, const hp_poses &poses, int thickness,
                             int radius, const void *workspace, hipStream_t s)
{
    DrawTables tab;   // the colours are in the workspace by now
    DrawParams P;
    const uint8_t none[3 * (HP_MAX_LIMBS + HP_MAX_PARTS)] = {0};
    draw_setup(Hf, Wf, H, W, T, K, L, pk, poses, none, none, thickness, radius, tab, P);
    const DrawWork ws = draw_layout((void *)workspace, N, P.list_cap, (size_t)P.tiles);
    const dim3 grid((Wf + kTileW - 1) / kTileW, (Hf + kTileH - 1) / kTileH, N);
    const uintptr_t bits = (uintptr_t)src | (uintptr_t)dst;
    const bool vec = (Wf % 4) == 0 && (bits & (C == 4 ? 15 : 3)) == 0;
    if (C == 3) {
        if (vec)
            HP_KERNEL((k_draw_tiles<3, true>), grid, dim3(kBlock), 0, s, src, dst, ws.records, ws.record_count, ws.tile_count,
                      ws.tile_records, ws.rgb_table, P);
        else
            HP_KERNEL((k_draw_tiles<3, false>), grid, dim3(kBlock), 0, s, src, dst, ws.records, ws.record_count, ws.tile_count,
                      ws.tile_records, ws.rgb_table, P);
    } else {
        if (vec)
            HP_KERNEL((k_draw_tiles<4, true>), grid, dim3(kBlock), 0, s, src, dst, ws.records, ws.record_count, ws.tile_count,
                      ws.tile_records, ws.rgb_table, P);
        else
            HP_KERNEL((k_draw_tiles<4, false>), grid, dim3(kBlock), 0, s, src, dst, ws.records, ws.record_count, ws.tile_count,
                      ws.tile_records, ws.rgb_table, P);
    }
    return hipGetLastError();
}

}  // namespace hp
