"""ctypes binding of libscap.so.  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libscap.so")

F16, BF16, I8 = 0, 1, 2
MODE_ZERO, MODE_MEAN, MODE_MEDIAN, MODE_HIST = 0, 1, 2, 3
MAX_TOKENS = 16
CFG_DEVICE_SCOPE_LOADS, CFG_GENERAL_KERNEL, CFG_ACCUMULATE, CFG_PARTIAL_SUMS, CFG_PARK_SLICES = 1, 2, 4, 8, 16

_TORCH_CODE = {torch.float16: F16, torch.bfloat16: BF16, torch.int8: I8}

EXPORTS = (
    "scap_status_string", "scap_version", "scap_workspace_bytes", "scap_workspace_init", "scap_calibrate",
    "scap_fold_bias", "scap_sparse_fc", "scap_sparse_fc_ex", "scap_sparse_fc_static", "scap_dense_fc", "scap_read_probe",
    "scap_pack_gate_up", "scap_swiglu_workspace_bytes", "scap_swiglu_block", "scap_swiglu_block_ex",
    "scap_swiglu_block_residual",
)


class ScapError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class LaunchCfg(ctypes.Structure):
    _fields_ = [("waves_per_group", ctypes.c_int32), ("rows_per_group", ctypes.c_int32),
                ("unroll", ctypes.c_int32), ("lanes_per_row", ctypes.c_int32), ("flags", ctypes.c_int32)]


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load libscap.so from the package directory.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it first (python -m paper_2412_07174_amd.build, or "
            "__graft_entry__.build()).  There is no fallback path.")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i64, i32, f32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.scap_status_string.restype = ctypes.c_char_p
    lib.scap_status_string.argtypes = [i32]
    lib.scap_version.restype = i32
    lib.scap_version.argtypes = []
    lib.scap_workspace_bytes.restype = sz
    lib.scap_workspace_bytes.argtypes = [i64, i64, i64]
    lib.scap_workspace_init.restype = i32
    lib.scap_workspace_init.argtypes = [vp, sz, vp]
    lib.scap_calibrate.restype = i32
    lib.scap_calibrate.argtypes = [vp, i64, i64, i32, f32, i32, ctypes.POINTER(f32), ctypes.POINTER(f32), vp, sz, vp]
    lib.scap_fold_bias.restype = i32
    lib.scap_fold_bias.argtypes = [vp, vp, i64, i64, i32, vp, f32, vp, vp, sz, vp]
    fc = [vp, vp, i64, i64, i32, vp, i32, i64, f32, f32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.scap_sparse_fc.restype = i32
    lib.scap_sparse_fc.argtypes = fc
    lib.scap_sparse_fc_ex.restype = i32
    lib.scap_sparse_fc_ex.argtypes = fc + [ctypes.POINTER(LaunchCfg)]
    lib.scap_sparse_fc_static.restype = i32
    lib.scap_sparse_fc_static.argtypes = fc[:-3] + [vp]
    lib.scap_dense_fc.restype = i32
    lib.scap_dense_fc.argtypes = [vp, vp, i64, i64, i32, vp, i32, i64, vp, vp, vp, sz, vp, ctypes.POINTER(LaunchCfg)]
    lib.scap_pack_gate_up.restype = i32
    lib.scap_pack_gate_up.argtypes = [vp, vp, i64, i64, i32, vp, vp]
    lib.scap_swiglu_workspace_bytes.restype = sz
    lib.scap_swiglu_workspace_bytes.argtypes = [i64, i64, i64, i64]
    lib.scap_swiglu_block.restype = i32
    lib.scap_swiglu_block.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, vp, i32, i64, f32, f32, vp, f32, f32, vp, vp,
                                      vp, vp, vp, vp, sz, vp]
    lib.scap_swiglu_block_residual.restype = i32
    lib.scap_swiglu_block_residual.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, vp, i32, i64, f32, f32, vp, f32, f32, vp, vp,
                                      vp, vp, vp, vp, sz, vp]
    lib.scap_swiglu_block_ex.restype = i32
    lib.scap_swiglu_block_ex.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, vp, i32, i64, f32, f32, vp, f32, f32, vp, vp,
                                      vp, vp, vp, vp, sz, vp, vp]
    lib.scap_read_probe.restype = i32
    lib.scap_read_probe.argtypes = [vp, sz, vp, vp]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().scap_status_string(int(status)).decode()


def version() -> int:
    return int(load_library().scap_version())


def workspace_bytes(K: int, N: int, B: int = 1) -> int:
    return int(load_library().scap_workspace_bytes(K, N, B))


def swiglu_workspace_bytes(K: int, F: int, N: int, B: int = 1) -> int:
    return int(load_library().scap_swiglu_workspace_bytes(K, F, N, B))


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise ScapError(rc, where)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _code(t: torch.Tensor, what: str) -> int:
    try:
        return _TORCH_CODE[t.dtype]
    except KeyError:
        raise TypeError(f"{what}: dtype {t.dtype} is not float16, bfloat16 or int8") from None


_ACT = (torch.float16, torch.bfloat16)
_WGT = (torch.float16, torch.bfloat16, torch.int8)


class _Args:
    """Validation of one call's tensors.  The binding hands raw pointers to the kernels, so a tensor of the wrong
    dtype, layout or shape would be read or written out of bounds on the device: refuse it here."""

    def __init__(self):
        self.seen = []

    def want(self, t: Optional[torch.Tensor], what: str, shape=None, dtype=None, optional: bool = False) -> None:
        if t is None:
            if optional:
                return
            raise TypeError(f"{what}: a tensor is required")
        if not isinstance(t, torch.Tensor):
            raise TypeError(f"{what}: expected a torch.Tensor, got {type(t).__name__}")
        if dtype is not None and t.dtype not in (dtype if isinstance(dtype, tuple) else (dtype,)):
            raise TypeError(f"{what}: dtype {t.dtype}, expected {dtype}")
        if not t.is_contiguous():
            raise ValueError(f"{what}: must be contiguous (shape {tuple(t.shape)}, strides {t.stride()})")
        if shape is not None and tuple(t.shape) not in (shape if isinstance(shape, list) else [shape]):
            raise ValueError(f"{what}: shape {tuple(t.shape)}, expected {shape}")
        self.seen.append((what, t))   # where it lives is checked last, by on_one_gpu()

    def rows(self, t: Optional[torch.Tensor], what: str, B: int, width: int, dtype, optional: bool = True) -> None:
        """A [rows, width] buffer with at least B rows (or a [width] vector for one token)."""
        self.want(t, what, dtype=dtype, optional=optional)
        if t is None:
            return
        ok = (t.dim() == 2 and t.shape[1] == width and t.shape[0] >= B) or (B == 1 and tuple(t.shape) == (width,))
        if not ok:
            raise ValueError(f"{what}: shape {tuple(t.shape)}, expected [>= {B}, {width}]")

    def on_one_gpu(self, workspace=None) -> None:
        """Every tensor of the call, and the workspace, on one GPU."""
        seen = list(self.seen)
        if isinstance(workspace, Workspace):
            seen.append(("workspace", workspace.buf))
        first = None
        for what, t in seen:
            if not t.is_cuda:
                raise ValueError(f"{what}: must live on the GPU, is on {t.device}")
            if first is None:
                first = (what, t.device)
            elif t.device != first[1]:
                raise ValueError(f"{what}: on {t.device}, but {first[0]} is on {first[1]}")
        if workspace is not None and not isinstance(workspace, Workspace):
            raise TypeError("workspace: expected a Workspace")

    def weights(self, W: torch.Tensor, col_scale, what: str = "W") -> None:
        self.want(W, what, dtype=_WGT)
        if W.dim() != 2:
            raise ValueError(f"{what}: expected a [K, N] matrix, got shape {tuple(W.shape)}")
        if W.dtype == torch.int8:
            self.want(col_scale, f"{what} column scales", shape=(W.shape[1],), dtype=torch.float16)
        elif col_scale is not None:
            raise TypeError(f"{what}: column scales go with int8 weights only")

    def tokens(self, x: torch.Tensor, K: int, what: str = "x") -> int:
        self.want(x, what, dtype=_ACT)
        if x.dim() not in (1, 2) or x.shape[-1] != K:
            raise ValueError(f"{what}: shape {tuple(x.shape)}, expected [{K}] or [B, {K}]")
        return 1 if x.dim() == 1 else x.shape[0]


def _cfg(cfg):
    if cfg is None:
        return None
    if isinstance(cfg, LaunchCfg):
        return ctypes.byref(cfg)
    waves, rows, unroll, *rest = cfg
    return ctypes.byref(LaunchCfg(int(waves), int(rows), int(unroll), int(rest[0]) if rest else 0,
                                  int(rest[1]) if len(rest) > 1 else 0))


class Workspace:
    """Caller-owned scratch for one stream: a torch byte buffer passed once to scap_workspace_init."""

    def __init__(self, K: int, N: int, B: int = 1, device="cuda", stream=None, F: int = 0):
        """K x N layer and B tokens; with F > 0 a SwiGLU block K -> F -> N (scap_swiglu_workspace_bytes)."""
        nbytes = swiglu_workspace_bytes(K, F, N, B) if F else workspace_bytes(K, N, B)
        if nbytes == 0:
            raise ScapError(-2, "scap_workspace_bytes")
        self.buf = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.nbytes = nbytes
        self.shape = (K, N, B)
        _check(load_library().scap_workspace_init(_ptr(self.buf), nbytes, _stream(stream)), "scap_workspace_init")

    def fits(self, K: int, N: int, B: int) -> bool:
        return workspace_bytes(K, N, B) <= self.nbytes


def calibrate(X_calib: torch.Tensor, target_sparsity: float, est: int = MODE_MEDIAN, *, workspace: Workspace,
              stream=None) -> Tuple[float, float]:
    """(m, tau) of one layer from its calibration activations [n, K] (device tensor, fp16/bf16)."""
    lib = load_library()
    a = _Args()
    a.want(X_calib, "X_calib", dtype=_ACT)
    if X_calib.dim() != 2:
        raise ValueError(f"X_calib: expected [n, K], got shape {tuple(X_calib.shape)}")
    a.on_one_gpu(workspace)
    n, K = X_calib.shape
    m, tau = ctypes.c_float(0), ctypes.c_float(0)
    rc = lib.scap_calibrate(_ptr(X_calib), n, K, _code(X_calib, "X_calib"), float(target_sparsity), int(est),
                            ctypes.byref(m), ctypes.byref(tau), _ptr(workspace.buf), workspace.nbytes, _stream(stream))
    _check(rc, "scap_calibrate")
    return float(m.value), float(tau.value)


def fold_bias(W: torch.Tensor, m: float, bias: Optional[torch.Tensor] = None, *, col_scale=None,
              out: Optional[torch.Tensor] = None, workspace: Workspace, stream=None) -> torch.Tensor:
    lib = load_library()
    a = _Args()
    a.weights(W, col_scale)
    K, N = W.shape
    a.want(bias, "bias", shape=(N,), dtype=torch.float32, optional=True)
    a.want(out, "out", shape=(N,), dtype=torch.float32, optional=True)
    a.on_one_gpu(workspace)
    if out is None:
        out = torch.empty(N, dtype=torch.float32, device=W.device)
    rc = lib.scap_fold_bias(_ptr(W), _ptr(col_scale), K, N, _code(W, "W"), _ptr(bias), float(m), _ptr(out),
                            _ptr(workspace.buf), workspace.nbytes, _stream(stream))
    _check(rc, "scap_fold_bias")
    return out


def sparse_fc(W: torch.Tensor, x: torch.Tensor, m: float, tau: float, b_fused: Optional[torch.Tensor] = None, *,
              col_scale=None, y: Optional[torch.Tensor] = None, idx_out=None, nnz_out=None, union_nnz_out=None,
              workspace: Workspace, cfg=None, stream=None) -> torch.Tensor:
    """y[B,N] = ((x - m) masked by |x - m| > tau) @ W + b_fused.  x is [K] or [B, K]."""
    lib = load_library()
    a = _Args()
    a.weights(W, col_scale)
    K, N = W.shape
    B = a.tokens(x, K, W.device)
    a.want(b_fused, "b_fused", shape=(N,), dtype=torch.float32, optional=True)
    a.rows(y, "y", B, N, torch.float32)
    a.rows(idx_out, "idx_out", B, K, torch.int32)
    for t, what in ((nnz_out, "nnz_out"), (union_nnz_out, "union_nnz_out")):
        a.want(t, what, dtype=torch.int32, optional=True)
    if nnz_out is not None and nnz_out.numel() < B:
        raise ValueError(f"nnz_out: {nnz_out.numel()} entries for {B} tokens")
    if union_nnz_out is not None and union_nnz_out.numel() < 1:
        raise ValueError("union_nnz_out: needs one entry")
    a.on_one_gpu(workspace)
    if y is None:
        y = torch.empty((B, N), dtype=torch.float32, device=x.device)
    args = [_ptr(W), _ptr(col_scale), K, N, _code(W, "W"), _ptr(x), _code(x, "x"), B, float(m), float(tau),
            _ptr(b_fused), _ptr(y), _ptr(idx_out), _ptr(nnz_out), _ptr(union_nnz_out), _ptr(workspace.buf),
            workspace.nbytes, _stream(stream)]
    if cfg is None:
        rc = lib.scap_sparse_fc(*args)
    else:
        rc = lib.scap_sparse_fc_ex(*args, _cfg(cfg))
    _check(rc, "scap_sparse_fc")
    return y


STATIC_SCRATCH_BYTES = 24 * 1024 * 1024


def sparse_fc_static(W: torch.Tensor, x: torch.Tensor, m: float, tau: float, b_fused: Optional[torch.Tensor] = None, *,
                     col_scale=None, y: torch.Tensor, idx_out=None, nnz_out=None, union_nnz_out=None,
                     stream=None) -> torch.Tensor:
    """sparse_fc without a workspace and without any allocation (the output tensor is required): the scratch is a
    fixed array inside the library, one per GPU, shared by every call on that GPU."""
    lib = load_library()
    a = _Args()
    a.weights(W, col_scale)
    K, N = W.shape
    B = a.tokens(x, K)
    a.want(b_fused, "b_fused", shape=(N,), dtype=torch.float32, optional=True)
    a.rows(y, "y", B, N, torch.float32, optional=False)
    a.rows(idx_out, "idx_out", B, K, torch.int32)
    for t, what in ((nnz_out, "nnz_out"), (union_nnz_out, "union_nnz_out")):
        a.want(t, what, dtype=torch.int32, optional=True)
    if nnz_out is not None and nnz_out.numel() < B:
        raise ValueError(f"nnz_out: {nnz_out.numel()} entries for {B} tokens")
    if union_nnz_out is not None and union_nnz_out.numel() < 1:
        raise ValueError("union_nnz_out: needs one entry")
    a.on_one_gpu()
    rc = lib.scap_sparse_fc_static(_ptr(W), _ptr(col_scale), K, N, _code(W, "W"), _ptr(x), _code(x, "x"), B, float(m),
                                   float(tau), _ptr(b_fused), _ptr(y), _ptr(idx_out), _ptr(nnz_out),
                                   _ptr(union_nnz_out), _stream(stream))
    _check(rc, "scap_sparse_fc_static")
    return y


def dense_fc(W: torch.Tensor, x: torch.Tensor, bias: Optional[torch.Tensor] = None, *, col_scale=None,
             y: Optional[torch.Tensor] = None, workspace: Workspace, cfg=None, stream=None) -> torch.Tensor:
    lib = load_library()
    a = _Args()
    a.weights(W, col_scale)
    K, N = W.shape
    B = a.tokens(x, K, W.device)
    a.want(bias, "bias", shape=(N,), dtype=torch.float32, optional=True)
    a.rows(y, "y", B, N, torch.float32)
    a.on_one_gpu(workspace)
    if y is None:
        y = torch.empty((B, N), dtype=torch.float32, device=x.device)
    rc = lib.scap_dense_fc(_ptr(W), _ptr(col_scale), K, N, _code(W, "W"), _ptr(x), _code(x, "x"), B, _ptr(bias),
                           _ptr(y), _ptr(workspace.buf), workspace.nbytes, _stream(stream), _cfg(cfg))
    _check(rc, "scap_dense_fc")
    return y


def pack_gate_up(gate: torch.Tensor, up: torch.Tensor, stream=None) -> torch.Tensor:
    """[rows, 2F] (or [2F]) interleaving of two [rows, F] (or [F]) tensors in groups of 4 columns."""
    a = _Args()
    a.want(gate, "gate")
    a.want(up, "up", shape=tuple(gate.shape), dtype=gate.dtype)
    if gate.dim() not in (1, 2):
        raise ValueError(f"gate: expected [F] or [rows, F], got shape {tuple(gate.shape)}")
    a.on_one_gpu()
    rows = 1 if gate.dim() == 1 else gate.shape[0]
    F = gate.shape[-1]
    out = torch.empty(gate.shape[:-1] + (2 * F,), dtype=gate.dtype, device=gate.device)
    rc = load_library().scap_pack_gate_up(_ptr(gate), _ptr(up), rows, F, gate.element_size(), _ptr(out), _stream(stream))
    _check(rc, "scap_pack_gate_up")
    return out


def swiglu_block(W_gu: torch.Tensor, W_down: torch.Tensor, x: torch.Tensor, m_x: float, tau_x: float,
                 b_gu_fused: Optional[torch.Tensor], m_z: float, tau_z: float, b_down_fused: Optional[torch.Tensor], *,
                 gu_scale=None, down_scale=None, y: Optional[torch.Tensor] = None, z_out=None, idx_z_out=None,
                 nnz_z_out=None, workspace: Workspace, stream=None, residual: bool = False, cfg=None) -> torch.Tensor:
    """y[N] of the SwiGLU block: W_gu is the packed [K, 2F] gate|up matrix, W_down is [F, N].
    residual=True (one token): scap_swiglu_block_residual, the block's output is added to the given y.
    cfg: launch flags of the one-token form (scap_swiglu_block_ex), not together with residual."""
    lib = load_library()
    a = _Args()
    a.weights(W_gu, gu_scale, "W_gu")
    a.weights(W_down, down_scale, "W_down")
    K, F2 = W_gu.shape
    F, N = W_down.shape
    if F2 != 2 * F:
        raise ValueError(f"W_gu has {F2} columns, W_down has {F} rows")
    B = a.tokens(x, K, W_gu.device)
    dev = W_gu.device
    a.want(b_gu_fused, "b_gu_fused", shape=(2 * F,), dtype=torch.float32, optional=True)
    a.want(b_down_fused, "b_down_fused", shape=(N,), dtype=torch.float32, optional=True)
    a.rows(y, "y", B, N, torch.float32)
    a.rows(z_out, "z_out", B, F, torch.float32)
    a.rows(idx_z_out, "idx_z_out", B, F, torch.int32)
    a.want(nnz_z_out, "nnz_z_out", dtype=torch.int32, optional=True)
    if nnz_z_out is not None and nnz_z_out.numel() < B:
        raise ValueError(f"nnz_z_out: {nnz_z_out.numel()} entries for {B} tokens")
    a.on_one_gpu(workspace)
    if y is None:
        if residual:
            raise ValueError("residual=True adds to y: pass the tensor that holds the addend")
        y = torch.empty((B, N), dtype=torch.float32, device=x.device)
    if _code(W_gu, "W_gu") != _code(W_down, "W_down"):
        raise TypeError("W_gu and W_down must have one dtype")
    if cfg is not None and residual:
        raise ValueError("cfg and residual=True cannot be combined")
    entry = lib.scap_swiglu_block_residual if residual else (lib.scap_swiglu_block if cfg is None else lib.scap_swiglu_block_ex)
    extra = () if cfg is None else (_cfg(cfg),)
    rc = entry(_ptr(W_gu), _ptr(gu_scale), _ptr(W_down), _ptr(down_scale), K, F, N, _code(W_gu, "W_gu"),
               _ptr(x), _code(x, "x"), B, float(m_x), float(tau_x), _ptr(b_gu_fused), float(m_z),
               float(tau_z), _ptr(b_down_fused), _ptr(y), _ptr(z_out), _ptr(idx_z_out),
               _ptr(nnz_z_out), _ptr(workspace.buf), workspace.nbytes, _stream(stream), *extra)
    _check(rc, "scap_swiglu_block_residual" if residual else "scap_swiglu_block")
    return y


def read_probe(src: torch.Tensor, out: torch.Tensor, stream=None) -> None:
    a = _Args()
    a.want(src, "src")
    a.want(out, "out", dtype=(torch.int32, torch.uint32))
    if out.numel() < 2048:
        raise ValueError("out: needs 2048 entries (SCAP_PROBE_SLOTS)")
    a.on_one_gpu()
    rc = load_library().scap_read_probe(_ptr(src), src.numel() * src.element_size(), _ptr(out), _stream(stream))
    _check(rc, "scap_read_probe")
