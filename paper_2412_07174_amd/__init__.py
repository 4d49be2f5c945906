"""MI355X-native sparse fully-connected layer of SCAP (arXiv 2412.07174).

Thin ctypes binding over ``libscap.so`` (hand-written HIP for gfx950, C ABI in ``include/scap.h``).
The binding only marshals arguments: torch tensors supply device memory and the current stream,
every step of the path runs inside the library's kernels.  There is no CPU fallback: if the
library has not been built, loading fails loudly.
"""
from .binding import (  # noqa: F401
    BF16, CFG_ACCUMULATE, CFG_DEVICE_SCOPE_LOADS, CFG_GENERAL_KERNEL, CFG_PARK_SLICES, CFG_PARTIAL_SUMS, F16, I8, MODE_HIST, STATIC_SCRATCH_BYTES, MODE_MEAN, MODE_MEDIAN, MODE_ZERO, LaunchCfg, ScapError, Workspace,
    calibrate, dense_fc, fold_bias, lib_path, load_library, pack_gate_up, read_probe, sparse_fc, sparse_fc_static, status_string,
    swiglu_block, swiglu_workspace_bytes, version, workspace_bytes,
)
