"""Seeded generator of synthetic network outputs (CM and PAF tensors).

Stands in for the activation maps that the inference operator hands to the
post-processing operator (paper Section 2.2.1, operators 3 and 4): the video
and the trained networks of the paper's evaluation (Section 3.2) are not
available, so people are planted from a skeleton template instead.

Recipe, per image (all randomness from numpy's PCG64, seed =
20210811 + 1000 * config_index + image_index, draws in the order below):
  1. cluster centres (clustered placement only): 3 x U(image).
  2. per person: scale ~ U(scale_lo, scale_hi) [hi-res px, person height],
     centre (uniform over the image; over the image grown by scale/2 when
     truncation is on; cluster centre + N(0, 150 px) when clustered; a fixed
     lattice when placement == "grid"), then joint jitter N(0, jitter_sd) per
     coordinate, then one U(0,1) per joint for dropout.
  3. spurious peaks: (part channel, x, y, amplitude ~ U(0.05, 0.3)) each.
  4. noise: one N(0, noise_sd) per CM element, then per PAF element.
Rendering is done at lo-res pixel centres: lo-res pixel (i, j) stands for the
hi-res point (s*j + (s-1)/2, s*i + (s-1)/2).
  CM[c]  = max over people of exp(-d^2 / (2 sigma^2)), d in hi-res px,
           truncated to zero beyond 64 px; spurious peaks joined by max;
           background channel = 1 - max_c CM[c]; then noise on every channel.
  PAF[2l], PAF[2l+1] = average, over the people whose limb l covers the pixel,
           of the unit vector A->B; a limb covers the points whose projection
           on AB lies within the segment and whose distance to the line is at
           most limb_halfwidth; rendered only if both ends are present; then
           noise.
Values are generated in float64 and cast once to the storage dtype.
"""
from dataclasses import dataclass, replace
import numpy as np

from .skeletons import Skeleton, COCO18, BODY25

SEED_BASE = 20210811


@dataclass(frozen=True)
class Params:
    """Post-processing thresholds (inputs to both implementations)."""
    peak_thr: float = 0.05
    paf_thr: float = 0.05
    n_samples: int = 10
    min_valid_ratio: float = 0.8
    min_parts: int = 3
    scale: int = 8


DEFAULT_PARAMS = Params()

# Output capacities (peaks per (image, part), candidates per (image, limb), persons per image) that the
# benchmark provisions for each workload; the parity tests run the same launch configuration.
BENCH_CAPS = {0: (64, 256, 64), 1: (128, 512, 128), 2: (128, 1024, 128), 3: (2048, 4096, 1024), 4: (1024, 4096, 512)}


@dataclass(frozen=True)
class SynthConfig:
    index: int                  # enters the seed
    skeleton: Skeleton
    batch: int
    h: int                      # lo-res rows
    w: int                      # lo-res cols
    n_people: int
    scale_lo: float = 40.0
    scale_hi: float = 120.0
    jitter_sd: float = 3.0
    noise_sd: float = 0.01
    dropout: float = 0.0
    n_spurious: int = 0
    truncation: bool = False    # centres may fall outside the image
    clustered: bool = False
    placement: str = "random"   # "random" | "grid"
    dtype: str = "float32"      # storage dtype of the tensors
    sigma: float = 7.0
    limb_halfwidth: float = 8.0
    scale: int = 8              # upsampling factor s

    @property
    def H(self):
        return self.h * self.scale

    @property
    def W(self):
        return self.w * self.scale

    def small(self, **kw):
        return replace(self, **kw)


CONFIGS = (
    SynthConfig(0, COCO18, 1, 46, 46, 3, noise_sd=0.01),
    SynthConfig(1, COCO18, 1, 46, 54, 10, noise_sd=0.02, truncation=True),
    SynthConfig(2, COCO18, 8, 46, 82, 20, noise_sd=0.02, dropout=0.15, n_spurious=30),
    SynthConfig(3, COCO18, 4, 135, 240, 30, scale_lo=30.0, scale_hi=300.0,
                noise_sd=0.03, clustered=True),
    SynthConfig(4, BODY25, 16, 90, 160, 40, scale_lo=40.0 * 720 / 368, scale_hi=120.0 * 720 / 368,
                noise_sd=0.03, dropout=0.2, n_spurious=60, dtype="float16"),
)


@dataclass
class SynthBatch:
    config: SynthConfig
    cm: np.ndarray              # [N, K+1, h, w] storage dtype
    paf: np.ndarray             # [N, 2L, h, w] storage dtype
    people: list                # per image: float64 [P, K, 2] hi-res (x, y), NaN = absent


def _place_people(cfg, rng):
    sk = cfg.skeleton
    K = sk.n_parts
    H, W = cfg.H, cfg.W
    tmpl = sk.template_xy
    clusters = None
    if cfg.clustered:
        clusters = np.stack([rng.uniform(0, W, 3), rng.uniform(0, H, 3)], axis=1)
    people = np.full((cfg.n_people, K, 2), np.nan)
    if cfg.placement == "grid":
        cols = int(np.ceil(np.sqrt(cfg.n_people * W / H)))
        rows = int(np.ceil(cfg.n_people / cols))
    for p in range(cfg.n_people):
        scale = rng.uniform(cfg.scale_lo, cfg.scale_hi)
        if cfg.placement == "grid":
            cx = (p % cols + 0.5) * W / cols
            cy = (p // cols + 0.5) * H / rows
        elif cfg.clustered:
            k = rng.integers(0, 3)
            cx = clusters[k, 0] + rng.normal(0.0, 150.0)
            cy = clusters[k, 1] + rng.normal(0.0, 150.0)
        elif cfg.truncation:
            cx = rng.uniform(-0.5 * scale, W + 0.5 * scale)
            cy = rng.uniform(-0.5 * scale, H + 0.5 * scale)
        else:
            cx = rng.uniform(0, W)
            cy = rng.uniform(0, H)
        joints = np.array([cx, cy]) + scale * tmpl
        joints = joints + rng.normal(0.0, cfg.jitter_sd, size=joints.shape)
        drop = rng.uniform(0, 1, K) < cfg.dropout
        inside = (joints[:, 0] >= 0) & (joints[:, 0] <= W - 1) & (joints[:, 1] >= 0) & (joints[:, 1] <= H - 1)
        keep = inside & ~drop
        people[p, keep] = joints[keep]
    return people


def _render_image(cfg, rng):
    sk = cfg.skeleton
    K, L = sk.n_parts, sk.n_limbs
    h, w, s = cfg.h, cfg.w, cfg.scale
    people = _place_people(cfg, rng)
    gx = s * np.arange(w) + (s - 1) / 2.0
    gy = s * np.arange(h) + (s - 1) / 2.0
    cm = np.zeros((K + 1, h, w))
    two_sig2 = 2.0 * cfg.sigma ** 2
    rad = 64.0

    def splat(c, x, y, amp):
        j0 = max(int(np.floor((x - rad - gx[0]) / s)), 0)
        j1 = min(int(np.ceil((x + rad - gx[0]) / s)) + 1, w)
        i0 = max(int(np.floor((y - rad - gy[0]) / s)), 0)
        i1 = min(int(np.ceil((y + rad - gy[0]) / s)) + 1, h)
        if j0 >= j1 or i0 >= i1:
            return
        d2 = (gx[None, j0:j1] - x) ** 2 + (gy[i0:i1, None] - y) ** 2
        g = amp * np.exp(-d2 / two_sig2)
        g[d2 > rad * rad] = 0.0
        np.maximum(cm[c, i0:i1, j0:j1], g, out=cm[c, i0:i1, j0:j1])

    for p in range(people.shape[0]):
        for c in range(K):
            x, y = people[p, c]
            if not np.isnan(x):
                splat(c, x, y, 1.0)
    for _ in range(cfg.n_spurious):
        c = int(rng.integers(0, K))
        x = rng.uniform(0, cfg.W)
        y = rng.uniform(0, cfg.H)
        amp = rng.uniform(0.05, 0.3)
        splat(c, x, y, amp)
    cm[K] = 1.0 - cm[:K].max(axis=0)

    paf_sum = np.zeros((2 * L, h, w))
    paf_cnt = np.zeros((L, h, w))
    hw = cfg.limb_halfwidth
    for p in range(people.shape[0]):
        for l, (a, b) in enumerate(sk.limbs):
            ax, ay = people[p, a]
            bx, by = people[p, b]
            if np.isnan(ax) or np.isnan(bx):
                continue
            length = np.hypot(bx - ax, by - ay)
            if length < 1e-6:
                continue
            ux, uy = (bx - ax) / length, (by - ay) / length
            j0 = max(int(np.floor((min(ax, bx) - hw - gx[0]) / s)), 0)
            j1 = min(int(np.ceil((max(ax, bx) + hw - gx[0]) / s)) + 1, w)
            i0 = max(int(np.floor((min(ay, by) - hw - gy[0]) / s)), 0)
            i1 = min(int(np.ceil((max(ay, by) + hw - gy[0]) / s)) + 1, h)
            if j0 >= j1 or i0 >= i1:
                continue
            rx = gx[None, j0:j1] - ax
            ry = gy[i0:i1, None] - ay
            along = rx * ux + ry * uy
            perp = np.abs(rx * uy - ry * ux)
            m = (along >= 0) & (along <= length) & (perp <= hw)
            paf_sum[2 * l, i0:i1, j0:j1] += m * ux
            paf_sum[2 * l + 1, i0:i1, j0:j1] += m * uy
            paf_cnt[l, i0:i1, j0:j1] += m
    cnt = np.maximum(paf_cnt, 1.0)
    paf = paf_sum / np.repeat(cnt, 2, axis=0)

    if cfg.noise_sd > 0:
        cm += rng.normal(0.0, cfg.noise_sd, size=cm.shape)
        paf += rng.normal(0.0, cfg.noise_sd, size=paf.shape)
    return cm, paf, people


def generate(cfg: SynthConfig, images=None) -> SynthBatch:
    """Render `cfg.batch` images (or the image indices in `images`)."""
    idx = list(range(cfg.batch)) if images is None else list(images)
    sk = cfg.skeleton
    dt = np.dtype(cfg.dtype)
    cm = np.empty((len(idx), sk.n_parts + 1, cfg.h, cfg.w), dtype=dt)
    paf = np.empty((len(idx), 2 * sk.n_limbs, cfg.h, cfg.w), dtype=dt)
    people = []
    for k, n in enumerate(idx):
        rng = np.random.Generator(np.random.PCG64(SEED_BASE + 1000 * cfg.index + n))
        c, p, pp = _render_image(cfg, rng)
        cm[k] = c.astype(dt)
        paf[k] = p.astype(dt)
        people.append(pp)
    return SynthBatch(cfg, cm, paf, people)


def gaussian_taps(sigma, radius):
    """2 * radius + 1 samples of a Gaussian of standard deviation `sigma` (pixels), normalised to sum 1 in float64 and
    rounded to fp32: the tap vector handed to the smoothing step by the tests and the benchmark (an input, like the maps)."""
    k = np.arange(-radius, radius + 1, dtype=np.float64)
    t = np.exp(-k * k / (2.0 * sigma * sigma))
    return (t / t.sum()).astype(np.float32)
