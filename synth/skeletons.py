"""Skeleton tables (inputs to both implementations).

The paper names the PAF/OpenPose family (Section 2.3) but prints no part or
limb table.  The tables below are this build's own: parts are listed head to
feet, limbs breadth-first from the neck so that, when limbs are folded into
persons in table order, the parent part of a tree limb is already attached.
The last two limbs close cycles (ear-shoulder) and are redundant on purpose.

`template` is a unit-height standing figure (x to the right, y down, origin
near the hip line) used only to plant synthetic people.
"""
from dataclasses import dataclass
import numpy as np


@dataclass(frozen=True)
class Skeleton:
    name: str
    part_names: tuple
    limbs: tuple            # ((a, b), ...) part indices, a -> b
    template: tuple         # ((x, y), ...) one per part, unit height

    @property
    def n_parts(self):
        return len(self.part_names)

    @property
    def n_limbs(self):
        return len(self.limbs)

    @property
    def limb_a(self):
        return np.array([a for a, _ in self.limbs], dtype=np.int32)

    @property
    def limb_b(self):
        return np.array([b for _, b in self.limbs], dtype=np.int32)

    @property
    def template_xy(self):
        return np.array(self.template, dtype=np.float64)


_COCO_PARTS = (
    "nose", "neck", "r_shoulder", "r_elbow", "r_wrist", "l_shoulder", "l_elbow",
    "l_wrist", "r_hip", "r_knee", "r_ankle", "l_hip", "l_knee", "l_ankle",
    "r_eye", "l_eye", "r_ear", "l_ear",
)

_COCO_TEMPLATE = (
    (0.00, -0.42),   # nose
    (0.00, -0.30),   # neck
    (-0.12, -0.30),  # r_shoulder
    (-0.16, -0.14),  # r_elbow
    (-0.19, 0.02),   # r_wrist
    (0.12, -0.30),   # l_shoulder
    (0.16, -0.14),   # l_elbow
    (0.19, 0.02),    # l_wrist
    (-0.08, 0.02),   # r_hip
    (-0.10, 0.26),   # r_knee
    (-0.12, 0.48),   # r_ankle
    (0.08, 0.02),    # l_hip
    (0.10, 0.26),    # l_knee
    (0.12, 0.48),    # l_ankle
    (-0.06, -0.48),  # r_eye
    (0.06, -0.48),   # l_eye
    (-0.13, -0.43),  # r_ear
    (0.13, -0.43),   # l_ear
)

_COCO_LIMBS = (
    (1, 0), (1, 2), (1, 5), (1, 8), (1, 11),
    (2, 3), (5, 6), (8, 9), (11, 12), (0, 14), (0, 15),
    (3, 4), (6, 7), (9, 10), (12, 13), (14, 16), (15, 17),
    (16, 2), (17, 5),
)

COCO18 = Skeleton("coco18", _COCO_PARTS, _COCO_LIMBS, _COCO_TEMPLATE)

_BODY25_PARTS = _COCO_PARTS + (
    "mid_hip", "r_big_toe", "r_small_toe", "r_heel", "l_big_toe", "l_small_toe", "l_heel",
)

_BODY25_TEMPLATE = _COCO_TEMPLATE + (
    (0.00, 0.045),    # mid_hip
    (-0.20, 0.50),    # r_big_toe
    (-0.285, 0.50),   # r_small_toe
    (-0.06, 0.54),    # r_heel
    (0.20, 0.50),     # l_big_toe
    (0.285, 0.50),    # l_small_toe
    (0.06, 0.54),     # l_heel
)

_BODY25_LIMBS = (
    (1, 0), (1, 2), (1, 5), (1, 18),
    (18, 8), (18, 11), (2, 3), (5, 6),
    (8, 9), (11, 12), (0, 14), (0, 15), (3, 4), (6, 7),
    (9, 10), (12, 13), (14, 16), (15, 17),
    (10, 19), (10, 21), (13, 22), (13, 24),
    (19, 20), (22, 23),
    (16, 2), (17, 5),
)

BODY25 = Skeleton("body25", _BODY25_PARTS, _BODY25_LIMBS, _BODY25_TEMPLATE)
