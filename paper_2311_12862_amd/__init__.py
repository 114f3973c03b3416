"""MI355X-native sparse 3-D convolution (implicit GEMM) behind a C ABI.

The work is done by libspconv.so (hand-written HIP for gfx950, built by
`python -m paper_2311_12862_amd.build`); this package only marshals arguments.
Importing it without the built library raises: there is no fallback path.
"""
from .binding import (  # noqa: F401
    Config, KMap, SpconvError, build_kmap, dgrad, fwd, fwd_noalloc, lib_path, load_library, tune, tune_group, wgrad,
    OP_FWD, OP_DGRAD, OP_WGRAD, FLAG_SLABS, EW_RELU, EW_ADD, EW_ADD_RELU, EW_RELU_BWD, ew, copy_cols, set_allocator, measure_peaks, describe_launch, LaunchInfo,
)
