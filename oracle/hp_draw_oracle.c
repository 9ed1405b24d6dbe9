/*
 * CPU oracle for the visualisation operator.
 *
 * TEST INFRASTRUCTURE ONLY.  The slow, plain statement of what operator 5 of
 * the paper's inference dataflow computes (Section 2.2.1: the parsed pose
 * topology is placed onto the original image).  It shares no code with the
 * HIP library and must never be called from the product path.
 *
 * The paper says what the operator is for and nothing about how the topology
 * is drawn, so the rules are this build's reading, all in integer arithmetic:
 *   V1 frames are 8-bit, interleaved (height, width, channel), C = 3 or 4; the
 *      first three channels receive colour, a fourth one is left as it is;
 *   V2 a peak at map pixel (x, y) of a W x H map lands on frame pixel
 *      (floor((2x + 1) Wf / (2 W)), floor((2y + 1) Hf / (2 H))): the frame pixel
 *      that contains the centre of the map pixel;
 *   V3 a limb whose two parts a person holds is the set of pixels whose centre
 *      lies within thickness / 2 of the segment between the two parts' frame
 *      pixels (a capsule); a part a person holds is the disc of pixels within
 *      `radius` of its frame pixel.  Distances are Euclidean between integer
 *      pixel coordinates and compared exactly (no rounding anywhere);
 *   V4 painter's order: persons in list order, for each person its limbs in
 *      table order, then its parts in index order; a pixel shows the colour of
 *      the last primitive that covers it, and the source pixel if none does.
 *      Colours are opaque, one per limb and one per part.
 *
 * The distance test is written as the closest-point definition: the point of
 * the segment nearest to P is A + (t / L2)(B - A) with t = clamp((P - A).(B - A),
 * 0, L2), L2 = |B - A|^2, so 4 |L2 (P - A) - t (B - A)|^2 <= thickness^2 L2^2,
 * evaluated in 128-bit integers.
 *
 * Parity pins (tests/test_oracle_draw.py): lattice-point counts of discs
 * (1, 5, 13, 29, 49, 81 for radius 0..5), axis-aligned and diagonal hairlines,
 * capsule areas in closed form, a float64 distance computation on random
 * segments away from the boundary, reflection / transposition symmetry, the
 * painter's order on overlapping primitives, and the coordinate map at
 * integer scale factors.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>

typedef __int128 wide;

/* V2 */
static int hpv_to_frame(int x, int n_map, int n_frame)
{
    return (int)(((int64_t)(2 * x + 1) * n_frame) / (2 * (int64_t)n_map));
}

/* V3: is pixel (px, py) within thickness / 2 of segment (ax, ay)-(bx, by)? */
int hpv_in_capsule(int px, int py, int ax, int ay, int bx, int by, int thickness)
{
    const wide dx = bx - ax, dy = by - ay;
    const wide ux = px - ax, uy = py - ay;
    const wide L2 = dx * dx + dy * dy;
    const wide th2 = (wide)thickness * thickness;
    if (L2 == 0) return 4 * (ux * ux + uy * uy) <= th2;
    wide t = ux * dx + uy * dy;
    if (t < 0) t = 0;
    if (t > L2) t = L2;
    const wide ex = L2 * ux - t * dx, ey = L2 * uy - t * dy;
    return 4 * (ex * ex + ey * ey) <= th2 * L2 * L2;
}

int hpv_in_disc(int px, int py, int cx, int cy, int radius)
{
    const int64_t ux = px - cx, uy = py - cy;
    return ux * ux + uy * uy <= (int64_t)radius * radius;
}

static void hpv_paint(uint8_t *img, int Hf, int Wf, int C, const uint8_t *rgb, int kind, int ax, int ay, int bx,
                      int by, int size)
{
    /* nothing further than `size` pixels from the primitive's bounding box can be covered */
    if (kind != 0) {
        bx = ax;
        by = ay;
    }
    const int x_lo = (ax < bx ? ax : bx) - size, x_hi = (ax > bx ? ax : bx) + size;
    const int y_lo = (ay < by ? ay : by) - size, y_hi = (ay > by ? ay : by) + size;
    for (int y = (y_lo < 0 ? 0 : y_lo); y < Hf && y <= y_hi; ++y)
        for (int x = (x_lo < 0 ? 0 : x_lo); x < Wf && x <= x_hi; ++x) {
            const int in = kind == 0 ? hpv_in_capsule(x, y, ax, ay, bx, by, size) : hpv_in_disc(x, y, ax, ay, size);
            if (in) memcpy(img + ((size_t)y * Wf + x) * C, rgb, 3);
        }
}

/*
 * One frame.  src / dst: [Hf][Wf][C]; px / py: peak coordinates [K][cap] on a W x H map; slots: [n_persons][K]
 * (peak rank or -1); limb_rgb: [L][3], part_rgb: [K][3].
 */
void hpv_draw(const uint8_t *src, uint8_t *dst, int Hf, int Wf, int C, int H, int W, int K, int L,
              const int32_t *limb_a, const int32_t *limb_b, const int32_t *px, const int32_t *py, int cap,
              const int32_t *slots, int n_persons, const uint8_t *limb_rgb, const uint8_t *part_rgb,
              int thickness, int radius)
{
    memmove(dst, src, (size_t)Hf * Wf * C);
    for (int p = 0; p < n_persons; ++p) {
        const int32_t *s = slots + (size_t)p * K;
        for (int l = 0; l < L; ++l) {
            const int a = limb_a[l], b = limb_b[l];
            if (s[a] < 0 || s[b] < 0) continue;
            hpv_paint(dst, Hf, Wf, C, limb_rgb + 3 * l, 0,
                      hpv_to_frame(px[(size_t)a * cap + s[a]], W, Wf), hpv_to_frame(py[(size_t)a * cap + s[a]], H, Hf),
                      hpv_to_frame(px[(size_t)b * cap + s[b]], W, Wf), hpv_to_frame(py[(size_t)b * cap + s[b]], H, Hf),
                      thickness);
        }
        for (int c = 0; c < K; ++c) {
            if (s[c] < 0) continue;
            hpv_paint(dst, Hf, Wf, C, part_rgb + 3 * c, 1, hpv_to_frame(px[(size_t)c * cap + s[c]], W, Wf),
                      hpv_to_frame(py[(size_t)c * cap + s[c]], H, Hf), 0, 0, radius);
        }
    }
}
