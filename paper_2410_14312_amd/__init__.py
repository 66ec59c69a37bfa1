"""MI355X-native stage-training hot path of TiMePReSt (arXiv 2410.14312).

Thin ctypes binding over libtmps.so (C ABI in include/tmps.h).  All arithmetic runs in the HIP
kernels of the library; this package only marshals arguments and gets device memory and streams
from PyTorch.  There is no CPU fallback: without the built library every entry point raises.
"""
from .binding import (KERNEL_CLASSES, profile_enable, profile_read, LayerDesc, Pipeline, Stage, StageCfg, TmpsError, lib, load_library,  # noqa: F401
                      schedule_plan, schedule_plan_1f1b, schedule_shadow_versions, schedule_stash_groups, version_diff_formula,
                      version_diff_simulated)
