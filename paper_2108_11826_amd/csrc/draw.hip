// Visualisation operator (Section 2.2.1, operator 5): the parsed poses drawn onto the frames.
//
// A limb is the capsule of pixels within thickness / 2 of the segment between its two parts, a part
// the disc of pixels within `radius`; primitives are ordered (person, then the person's limbs in
// table order, then its parts) and a pixel shows the last one that covers it, else the source
// pixel.  All geometry is exact integer arithmetic on frame pixel coordinates.
//
// One workgroup owns a tile of 64 x 16 pixels, one thread four neighbouring pixels of a row.  The
// image's primitives are walked 256 at a time: every thread builds one (two gathers from the person
// table, two from the peak lists), keeps it if its bounding box meets the tile, and the kept ones
// are packed in order into LDS; each thread then walks the packed list backwards until its four
// pixels are decided.  A later chunk overrides an earlier one.  Most tiles keep no primitive at all
// and only copy their pixels, so the kernel moves the frames at memory speed.
#include <string.h>

#include "hp_dev.h"

namespace hp {

constexpr int kDrawTileW = 64, kDrawTileH = 16;

struct DrawColours {
    uint8_t limb[HP_MAX_LIMBS][3];
    uint8_t part[HP_MAX_PARTS][3];
};

struct DrawParams {
    int Hf, Wf, H, W, K, L, cap, pcap;
    int thickness, radius;
    int th2_quarter;   // floor(thickness^2 / 4): 4 |u|^2 <= thickness^2 for integer |u|^2
    int reach;         // pixels a primitive can extend beyond its end points
};

// Frame pixel that contains the centre of map pixel x.
__device__ __forceinline__ int to_frame(int x, int n_map, int n_frame)
{
    return (int)(((long long)(2 * x + 1) * n_frame) / (2LL * n_map));
}

__device__ __forceinline__ bool in_capsule(int px, int py, int ax, int ay, int bx, int by, int th2_quarter,
                                           long long th2)
{
    const int dx = bx - ax, dy = by - ay;
    const int ux = px - ax, uy = py - ay;
    const int t = ux * dx + uy * dy;          // |t| <= 2 * 16384^2 < 2^31
    if (t <= 0) return ux * ux + uy * uy <= th2_quarter;
    const int L2 = dx * dx + dy * dy;
    if (t >= L2) {
        const int vx = px - bx, vy = py - by;
        return vx * vx + vy * vy <= th2_quarter;
    }
    const long long cross = (long long)ux * dy - (long long)uy * dx;
    return 4 * cross * cross <= th2 * L2;     // squared distance to the line = cross^2 / L2
}

template <int C, bool VEC>
__global__ __launch_bounds__(kBlock) void k_draw(const uint8_t *src, uint8_t *dst,   // may be the same buffer
                                                 const int32_t *__restrict__ peak_x, const int32_t *__restrict__ peak_y,
                                                 const int32_t *__restrict__ slots, const int32_t *__restrict__ pose_count,
                                                 LimbTable T, DrawColours col, DrawParams P)
{
    __shared__ int s_ax[kBlock], s_ay[kBlock], s_bx[kBlock], s_by[kBlock], s_id[kBlock];
    __shared__ int s_scan[kBlock / kWave + 1];

    const int n = blockIdx.z;
    const int tid = threadIdx.x;
    const int tile_x0 = blockIdx.x * kDrawTileW, tile_y0 = blockIdx.y * kDrawTileH;
    const int x0 = tile_x0 + 4 * (tid & 15), y = tile_y0 + (tid >> 4);
    const int per_person = P.L + P.K;
    const int n_persons = min(pose_count[n], P.pcap);
    const int items = n_persons * per_person;
    const long long th2 = (long long)P.thickness * P.thickness;
    const int r2 = P.radius * P.radius;

    int best[4] = {-1, -1, -1, -1};   // colour index of the last primitive covering each pixel
    for (int base = 0; base < items; base += kBlock) {
        const int q = base + tid;
        bool keep = false;
        int ax = 0, ay = 0, bx = 0, by = 0, id = 0;
        if (q < items) {
            const int p = q / per_person;
            id = q - p * per_person;
            const int32_t *sl = slots + ((size_t)n * P.pcap + p) * P.K;
            const int a = id < P.L ? T.a[id] : id - P.L;
            const int b = id < P.L ? T.b[id] : a;
            const int ia = sl[a], ib = sl[b];
            if (ia >= 0 && ib >= 0 && ia < P.cap && ib < P.cap) {
                const size_t oa = ((size_t)n * P.K + a) * P.cap + ia, ob = ((size_t)n * P.K + b) * P.cap + ib;
                // a peak of the map lands inside the frame; the clamps only keep the integer geometry below
                // within range should the lists hold anything else
                ax = min(max(to_frame(peak_x[oa], P.W, P.Wf), 0), P.Wf - 1);
                ay = min(max(to_frame(peak_y[oa], P.H, P.Hf), 0), P.Hf - 1);
                bx = min(max(to_frame(peak_x[ob], P.W, P.Wf), 0), P.Wf - 1);
                by = min(max(to_frame(peak_y[ob], P.H, P.Hf), 0), P.Hf - 1);
                const int reach = id < P.L ? P.reach : P.radius;
                keep = min(ax, bx) - reach < tile_x0 + kDrawTileW && max(ax, bx) + reach >= tile_x0 &&
                       min(ay, by) - reach < tile_y0 + kDrawTileH && max(ay, by) + reach >= tile_y0;
            }
        }
        int kept;
        const int pos = block_flag_scan(keep, s_scan, kept);
        if (keep) {
            s_ax[pos] = ax;
            s_ay[pos] = ay;
            s_bx[pos] = bx;
            s_by[pos] = by;
            s_id[pos] = id;
        }
        __syncthreads();
        int open = 0xF;    // pixels not yet decided within this chunk
        for (int k = kept - 1; k >= 0 && open; --k) {
            const int cax = s_ax[k], cay = s_ay[k], cbx = s_bx[k], cby = s_by[k], cid = s_id[k];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (!(open >> j & 1)) continue;
                bool in;
                if (cid < P.L) {
                    in = in_capsule(x0 + j, y, cax, cay, cbx, cby, P.th2_quarter, th2);
                } else {
                    const int ux = x0 + j - cax, uy = y - cay;
                    in = ux * ux + uy * uy <= r2;
                }
                if (in) {
                    best[j] = cid;
                    open &= ~(1 << j);
                }
            }
        }
        __syncthreads();
    }

    if (y >= P.Hf || x0 >= P.Wf) return;
    const size_t row = ((size_t)n * P.Hf + y) * P.Wf;
    auto colour = [&](int id, int ch) -> uint32_t { return id < P.L ? col.limb[id][ch] : col.part[id - P.L][ch]; };
    if (VEC) {
        // four whole pixels: 12 or 16 bytes at a 4-byte (C = 3) or 16-byte (C = 4) aligned address
        if (C == 3) {
            const uint32_t *s = (const uint32_t *)(src + (row + x0) * 3);
            uint32_t w[3] = {__builtin_nontemporal_load(s), __builtin_nontemporal_load(s + 1),
                             __builtin_nontemporal_load(s + 2)};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (best[j] < 0) continue;
#pragma unroll
                for (int ch = 0; ch < 3; ++ch) {
                    const int byte = 3 * j + ch;
                    w[byte >> 2] = (w[byte >> 2] & ~(0xFFu << (8 * (byte & 3)))) | (colour(best[j], ch) << (8 * (byte & 3)));
                }
            }
            uint32_t *d = (uint32_t *)(dst + (row + x0) * 3);
            __builtin_nontemporal_store(w[0], d);
            __builtin_nontemporal_store(w[1], d + 1);
            __builtin_nontemporal_store(w[2], d + 2);
        } else {
            typedef uint32_t v4u __attribute__((ext_vector_type(4)));
            v4u w = __builtin_nontemporal_load((const v4u *)(src + (row + x0) * 4));
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (best[j] < 0) continue;
                w[j] = (w[j] & 0xFF000000u) | colour(best[j], 0) | (colour(best[j], 1) << 8) | (colour(best[j], 2) << 16);
            }
            __builtin_nontemporal_store(w, (v4u *)(dst + (row + x0) * 4));
        }
    } else {
        for (int j = 0; j < 4 && x0 + j < P.Wf; ++j) {
            const uint8_t *s = src + (row + x0 + j) * C;
            uint8_t *d = dst + (row + x0 + j) * C;
            uint8_t v[C];
#pragma unroll
            for (int ch = 0; ch < C; ++ch) v[ch] = s[ch];
            if (best[j] >= 0) {
#pragma unroll
                for (int ch = 0; ch < 3; ++ch) v[ch] = (uint8_t)colour(best[j], ch);
            }
#pragma unroll
            for (int ch = 0; ch < C; ++ch) d[ch] = v[ch];
        }
    }
}

hipError_t launch_draw(const uint8_t *src, uint8_t *dst, int N, int Hf, int Wf, int C, int H, int W, const LimbTable &T,
                       int K, int L, const hp_peaks &pk, const hp_poses &poses, const uint8_t *limb_rgb,
                       const uint8_t *part_rgb, int thickness, int radius, hipStream_t s)
{
    DrawColours col = {};
    for (int l = 0; l < L; ++l)
        for (int ch = 0; ch < 3; ++ch) col.limb[l][ch] = limb_rgb[3 * l + ch];
    for (int c = 0; c < K; ++c)
        for (int ch = 0; ch < 3; ++ch) col.part[c][ch] = part_rgb[3 * c + ch];
    DrawParams P;
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
    const dim3 grid((Wf + kDrawTileW - 1) / kDrawTileW, (Hf + kDrawTileH - 1) / kDrawTileH, N);
    const uintptr_t bits = (uintptr_t)src | (uintptr_t)dst;
    const bool vec = (Wf % 4) == 0 && (bits & (C == 4 ? 15 : 3)) == 0;
    if (C == 3) {
        if (vec)
            HP_KERNEL((k_draw<3, true>), grid, dim3(kBlock), 0, s, src, dst, pk.x, pk.y, poses.slots, poses.count, T, col, P);
        else
            HP_KERNEL((k_draw<3, false>), grid, dim3(kBlock), 0, s, src, dst, pk.x, pk.y, poses.slots, poses.count, T, col, P);
    } else {
        if (vec)
            HP_KERNEL((k_draw<4, true>), grid, dim3(kBlock), 0, s, src, dst, pk.x, pk.y, poses.slots, poses.count, T, col, P);
        else
            HP_KERNEL((k_draw<4, false>), grid, dim3(kBlock), 0, s, src, dst, pk.x, pk.y, poses.slots, poses.count, T, col, P);
    }
    return hipGetLastError();
}

}  // namespace hp
