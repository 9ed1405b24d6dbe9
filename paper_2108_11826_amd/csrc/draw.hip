// Visualisation operator (Section 2.2.1, operator 5): the parsed poses drawn onto the frames.
//
// A limb is the capsule of pixels within thickness / 2 of the segment between its two parts, a part
// the disc of pixels within `radius`; primitives are ordered (person, then the person's limbs in
// table order, then its parts) and a pixel shows the last one that covers it, else the source
// pixel.  All geometry is exact integer arithmetic on frame pixel coordinates.
//
// Two launches.  k_draw_list, one workgroup per image, walks the person table once and writes the
// image's primitives, in painter's order, as 16-byte records (end points in frame coordinates, id,
// and the largest cross product a covered pixel can have) into the workspace.  k_draw_tiles, one
// workgroup per tile of 64 x 16 pixels, reads the records 256 at a time (coalesced), keeps those
// whose bounding box and line can meet the tile, packed in order in LDS, and then every wavefront
// paints one strip of 64 x 4 pixels: 64 lanes test 64 kept records at a time against the strip, the
// few that can touch it are broadcast from lane to scalar registers, newest first, and each lane
// decides its four neighbouring pixels with 32-bit integer tests.  Most tiles keep nothing and only
// copy their pixels.  Crowded places cost a wavefront a walk over one strip's records only, which
// keeps the longest wavefront short: with larger regions per workgroup the few crowded ones decided
// the kernel's duration (measured: 2 to 5 times slower).
#include <string.h>

#include "hp_dev.h"

namespace hp {

#ifndef HP_DRAW_STRIPS
#define HP_DRAW_STRIPS 1
#endif
constexpr int kStrips = HP_DRAW_STRIPS;       // strips a wavefront paints, one after the other (measured: 1 is best
                                              // on crowded frames, where the longest wavefront decides)
constexpr int kStripH = 4;                    // rows of a strip: one per 16 lanes
constexpr int kTileW = 64, kTileH = kStripH * kStrips * (kBlock / kWave);   // pixels a workgroup paints
static_assert(kStripH * 16 == kWave && kTileW == 4 * 16, "a lane paints four neighbouring pixels of one row");

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

// Frame pixel that contains the centre of map pixel x.
__device__ __forceinline__ int to_frame(int x, int n_map, int n_frame)
{
    return (int)(((long long)(2 * x + 1) * n_frame) / (2LL * n_map));
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

__global__ __launch_bounds__(kBlock) void k_draw_list(const int32_t *__restrict__ peak_x, const int32_t *__restrict__ peak_y,
                                                      const int32_t *__restrict__ slots,
                                                      const int32_t *__restrict__ pose_count, DrawTables tab, DrawParams P,
                                                      DrawRecord *__restrict__ records, int32_t *__restrict__ record_count,
                                                      uint32_t *__restrict__ tile_mask)
{
    __shared__ uint8_t s_part_a[HP_MAX_LIMBS], s_part_b[HP_MAX_LIMBS];
    __shared__ int s_scan[kBlock / kWave + 1];
    extern __shared__ uint32_t s_mask[];   // one bit per tile: can any primitive touch it?
    const int n = blockIdx.x, tid = threadIdx.x;
    if (tid == 0) {
#pragma unroll
        for (int i = 0; i < HP_MAX_LIMBS; ++i) {
            s_part_a[i] = tab.a[i];
            s_part_b[i] = tab.b[i];
        }
    }
    for (int i = tid; i < P.mask_words; i += kBlock) s_mask[i] = 0;
    __syncthreads();
    const int per_person = P.L + P.K;
    const int items = min(pose_count[n], P.pcap) * per_person;
    DrawRecord *out = records + (size_t)n * P.list_cap;
    int total = 0;
    for (int base = 0; base < items; base += kBlock) {
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
                // a peak of the map lands inside the frame; the clamps only keep the integer geometry
                // within range should the lists hold anything else
                const int ax = min(max(to_frame(peak_x[oa], P.W, P.Wf), 0), P.Wf - 1);
                const int ay = min(max(to_frame(peak_y[oa], P.H, P.Hf), 0), P.Hf - 1);
                const int bx = min(max(to_frame(peak_x[ob], P.W, P.Wf), 0), P.Wf - 1);
                const int by = min(max(to_frame(peak_y[ob], P.H, P.Hf), 0), P.Hf - 1);
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
    for (int i = tid; i < P.mask_words; i += kBlock) tile_mask[(size_t)n * P.mask_words + i] = s_mask[i];
}

template <int C, bool VEC>
__global__ __launch_bounds__(kBlock) void k_draw_tiles(const uint8_t *src, uint8_t *dst,   // may be the same buffer
                                                       const DrawRecord *__restrict__ records,
                                                       const int32_t *__restrict__ record_count,
                                                       const uint32_t *__restrict__ tile_mask, DrawTables tab,
                                                       DrawParams P)
{
    constexpr int kChunk = 2 * kBlock;   // records looked at per round: two per thread, one memory round trip
    __shared__ uint32_t s_rgb[HP_MAX_LIMBS + HP_MAX_PARTS];
    __shared__ int t_a[kChunk], t_b[kChunk], t_id[kChunk], t_cmax[kChunk];
    __shared__ int s_scan[kBlock / kWave + 1];

    const int n = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
    const int tile_x0 = blockIdx.x * kTileW, tile_y0 = blockIdx.y * kTileH;
    const int x0 = tile_x0 + 4 * (lane & 15);
    const int r2 = P.radius * P.radius;
    // tiles no primitive can touch (most of them) skip the records altogether
    const int tile = blockIdx.y * P.tiles_x + blockIdx.x;
    const int listed = record_count[n];   // read whether needed or not: one memory round trip for both words
    const bool touched = (tile_mask[(size_t)n * P.mask_words + (tile >> 5)] >> (tile & 31)) & 1u;
    const int count = touched ? min(listed, P.list_cap) : 0;
    const DrawRecord *list = records + (size_t)n * P.list_cap;

    // this thread's pixels are on their way while the records are looked at
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    uint32_t w[kStrips][4];
    bool inside[kStrips];
#pragma unroll
    for (int i = 0; i < kStrips; ++i) {
        const int y = tile_y0 + (wv * kStrips + i) * kStripH + (lane >> 4);
        inside[i] = y < P.Hf && x0 < P.Wf;
        w[i][0] = w[i][1] = w[i][2] = w[i][3] = 0;
        if (VEC && inside[i]) {
            const size_t row = ((size_t)n * P.Hf + y) * P.Wf;
            if (C == 3) {
                const uint32_t *s = (const uint32_t *)(src + (row + x0) * 3);
                w[i][0] = __builtin_nontemporal_load(s);
                w[i][1] = __builtin_nontemporal_load(s + 1);
                w[i][2] = __builtin_nontemporal_load(s + 2);
            } else {
                const v4u v = __builtin_nontemporal_load((const v4u *)(src + (row + x0) * 4));
                w[i][0] = v[0];
                w[i][1] = v[1];
                w[i][2] = v[2];
                w[i][3] = v[3];
            }
        }
    }
    if (count > 0 && tid == 0) {
        // colours by id; tab is a kernel argument, so the copy goes through constant indices
#pragma unroll
        for (int i = 0; i < HP_MAX_LIMBS + HP_MAX_PARTS; ++i) s_rgb[i] = tab.rgb[i];
    }

    int best[kStrips][4];   // id of the last primitive covering each of the lane's pixels
#pragma unroll
    for (int i = 0; i < kStrips; ++i) best[i][0] = best[i][1] = best[i][2] = best[i][3] = -1;

    auto meets_tile = [&](const DrawRecord &rec) {
        const bool limb = rec.id < P.L;
        return box_meets(rec.a, rec.b, limb ? P.reach : P.radius, tile_x0, tile_y0, kTileW, kTileH) &&
               !(limb && far_from_line(rec.a, rec.b, rec.cmax, 2 * tile_x0 + kTileW - 1, 2 * tile_y0 + kTileH - 1,
                                       kTileW - 1, kTileH - 1));
    };

    for (int base = 0; base < count; base += kChunk) {
        // the records that can meet the tile, packed in order
        const int q0 = base + tid, q1 = base + kBlock + tid;
        DrawRecord rec0 = {0, 0, 0, 0}, rec1 = {0, 0, 0, 0};
        if (q0 < count) rec0 = list[q0];
        if (q1 < count) rec1 = list[q1];
        const bool keep0 = q0 < count && meets_tile(rec0), keep1 = q1 < count && meets_tile(rec1);
        int kept0, kept1 = 0, pos1 = 0;
        const int pos0 = block_flag_scan(keep0, s_scan, kept0);
        if (base + kBlock < count) pos1 = block_flag_scan(keep1, s_scan, kept1);   // the same for every thread
        const int kept = kept0 + kept1;
        if (kept == 0) continue;   // the same for every thread
        if (keep0) {
            t_a[pos0] = rec0.a;
            t_b[pos0] = rec0.b;
            t_id[pos0] = rec0.id;
            t_cmax[pos0] = rec0.cmax;
        }
        if (keep1) {
            t_a[kept0 + pos1] = rec1.a;
            t_b[kept0 + pos1] = rec1.b;
            t_id[kept0 + pos1] = rec1.id;
            t_cmax[kept0 + pos1] = rec1.cmax;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kStrips; ++i) {
            // One strip of the wavefront: the kept records are walked backwards, 64 at a time.  Every lane tests one
            // record against the strip; those that can touch it are broadcast (lane to scalar registers), newest first.
            const int strip_y0 = tile_y0 + (wv * kStrips + i) * kStripH, y = strip_y0 + (lane >> 4);
            int open = inside[i] ? 0xF : 0;   // pixels this round has not decided yet; a later round overrides an earlier one
            for (int k0 = (kept - 1) & ~(kWave - 1); k0 >= 0 && __ballot(open != 0); k0 -= kWave) {
                const int k = k0 + lane;
                int ea = 0, eb = 0, eid = 0, ecmax = 0;
                bool touches = false;
                if (k < kept) {
                    ea = t_a[k];
                    eb = t_b[k];
                    eid = t_id[k];
                    ecmax = t_cmax[k];
                    const int reach = eid < P.L ? P.reach : P.radius;
                    touches = !(strip_y0 + kStripH - 1 < min(py_of(ea), py_of(eb)) - reach ||
                                strip_y0 > max(py_of(ea), py_of(eb)) + reach) &&
                              !(eid < P.L && far_from_line(ea, eb, ecmax, 2 * tile_x0 + kTileW - 1,
                                                           2 * strip_y0 + kStripH - 1, kTileW - 1, kStripH - 1));
                }
                unsigned long long m = __ballot(touches);
                while (m) {
                    const int from_lane = 63 - __builtin_clzll(m);
                    m &= ~(1ull << from_lane);
                    const int a = __builtin_amdgcn_readlane(ea, from_lane), b = __builtin_amdgcn_readlane(eb, from_lane);
                    const int cid = __builtin_amdgcn_readlane(eid, from_lane);
                    const int cmax = __builtin_amdgcn_readlane(ecmax, from_lane);
                    const int ax = px_of(a), ay = py_of(a), bx = px_of(b), by = py_of(b);
                    const bool limb = cid < P.L;
                    const int reach = limb ? P.reach : P.radius;
                    // the lane's four pixels
                    if (!open || x0 + 3 < min(ax, bx) - reach || x0 > max(ax, bx) + reach) continue;
                    const int ux = x0 - ax, uy = y - ay;
                    // squared distances of the lane's first pixel to the end points; pixel j adds j (2 u + j)
                    const int dA = __mul24(ux, ux) + __mul24(uy, uy);
                    if (limb) {
                        // exact, in 32 bits: t = (P - A).(B - A) selects an end cap or the middle, where the pixel is
                        // inside when |(P - A) x (B - A)| <= cmax
                        const int dx = bx - ax, dy = by - ay, L2 = __mul24(dx, dx) + __mul24(dy, dy);
                        const int vx = x0 - bx, vy = y - by;
                        const int dB = __mul24(vx, vx) + __mul24(vy, vy);
                        const int t0 = __mul24(ux, dx) + __mul24(uy, dy), c0 = __mul24(ux, dy) - __mul24(uy, dx);
                        if (abs(2 * c0 + 3 * dy) > 2 * cmax + 3 * abs(dy) && t0 > 0 && t0 + 3 * dx > 0 && t0 < L2 &&
                            t0 + 3 * dx < L2)
                            continue;   // all four lie beside the middle part and too far from the line
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int t = t0 + j * dx, c = c0 + j * dy;
                            const bool in = (t <= 0) & (dA + j * (2 * ux + j) <= P.th2_quarter) |
                                            (t >= L2) & (dB + j * (2 * vx + j) <= P.th2_quarter) |
                                            (t > 0) & (t < L2) & (abs(c) <= cmax);
                            const int take = (int)in & (open >> j);   // bit 0: covered and not decided yet
                            best[i][j] = (take & 1) ? cid : best[i][j];
                            open &= ~((take & 1) << j);
                        }
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int take = (int)(dA + j * (2 * ux + j) <= r2) & (open >> j);
                            best[i][j] = (take & 1) ? cid : best[i][j];
                            open &= ~((take & 1) << j);
                        }
                    }
                }
            }
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < kStrips; ++i) {
        if (!inside[i]) continue;
        const int y = tile_y0 + (wv * kStrips + i) * kStripH + (lane >> 4);
        const size_t row = ((size_t)n * P.Hf + y) * P.Wf;
        if (VEC) {
            // four whole pixels: 12 or 16 bytes at a 4-byte (C = 3) or 16-byte (C = 4) aligned address
            if (C == 3) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (best[i][j] < 0) continue;
                    const uint32_t rgb = s_rgb[best[i][j]];
#pragma unroll
                    for (int ch = 0; ch < 3; ++ch) {
                        const int byte = 3 * j + ch;
                        w[i][byte >> 2] = (w[i][byte >> 2] & ~(0xFFu << (8 * (byte & 3)))) |
                                          (((rgb >> (8 * ch)) & 0xFFu) << (8 * (byte & 3)));
                    }
                }
                uint32_t *d = (uint32_t *)(dst + (row + x0) * 3);
                __builtin_nontemporal_store(w[i][0], d);
                __builtin_nontemporal_store(w[i][1], d + 1);
                __builtin_nontemporal_store(w[i][2], d + 2);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (best[i][j] >= 0) w[i][j] = (w[i][j] & 0xFF000000u) | s_rgb[best[i][j]];
                v4u v = {w[i][0], w[i][1], w[i][2], w[i][3]};
                __builtin_nontemporal_store(v, (v4u *)(dst + (row + x0) * 4));
            }
        } else {
            for (int j = 0; j < 4 && x0 + j < P.Wf; ++j) {
                const uint8_t *s = src + (row + x0 + j) * C;
                uint8_t *d = dst + (row + x0 + j) * C;
                uint8_t v[C];
#pragma unroll
                for (int ch = 0; ch < C; ++ch) v[ch] = s[ch];
                if (best[i][j] >= 0) {
                    const uint32_t rgb = s_rgb[best[i][j]];
#pragma unroll
                    for (int ch = 0; ch < 3; ++ch) v[ch] = (uint8_t)(rgb >> (8 * ch));
                }
#pragma unroll
                for (int ch = 0; ch < C; ++ch) d[ch] = v[ch];
            }
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
    HP_KERNEL(k_draw_list, dim3(N), dim3(kBlock), P.mask_words * sizeof(uint32_t), s, pk.x, pk.y, poses.slots, poses.count, tab, P,
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
