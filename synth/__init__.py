"""Seeded synthetic inputs for bottom-up pose post-processing.

This package holds only input construction: skeleton tables (which both the
CPU oracle and the HIP library receive as an argument) and a generator of
confidence maps (CM) and part-affinity fields (PAF) shaped like the network
outputs that the post-processing operator of the paper's inference engine
consumes (Section 2.2.1, operator 4).  None of the post-processing arithmetic
lives here.
"""
from .skeletons import Skeleton, COCO18, BODY25
from .pose_proposal import PPConfig, PP_CONFIGS, PP_COCO19, generate_pp
from .composite_fields import CFConfig, CF_CONFIGS, CF_COCO17, generate_cf
from .generate import SynthConfig, CONFIGS, generate, Params, DEFAULT_PARAMS, BENCH_CAPS, gaussian_taps

__all__ = ["CFConfig", "CF_CONFIGS", "CF_COCO17", "generate_cf", "PPConfig", "PP_CONFIGS", "PP_COCO19", "generate_pp", "gaussian_taps", "Skeleton", "COCO18", "BODY25", "SynthConfig", "CONFIGS", "generate",
           "Params", "DEFAULT_PARAMS", "BENCH_CAPS"]
