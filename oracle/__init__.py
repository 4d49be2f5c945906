"""CPU oracle (test infrastructure only -- never imported by the product package).

`scap_oracle.c` is the definition-level implementation; this module compiles it with gcc
(`build()`), loads it through ctypes and exposes numpy-in / numpy-out wrappers.  Only the
tests, the smoke check and the benchmark's CPU-baseline leg may import it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "scap_oracle.c")
_LIB = os.path.join(_HERE, "libscap_oracle.so")

F16, BF16, I8 = 0, 1, 2
F32 = 3  # activations only: fp32 values (the gated product inside a SwiGLU block)
MODE_ZERO, MODE_MEAN, MODE_MEDIAN, MODE_HIST = 0, 1, 2, 3
EST = {"zero": MODE_ZERO, "mean": MODE_MEAN, "median": MODE_MEDIAN, "hist": MODE_HIST}

_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle: plain -O2, no fast-math, no FP contraction."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build(force=False)
    lib = ctypes.CDLL(_LIB)
    vp, i64, i32, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float
    lib.oracle_to_f32.restype = f32
    lib.oracle_to_f32.argtypes = [ctypes.c_uint16, i32]
    lib.oracle_centre_threshold.restype = i64
    lib.oracle_centre_threshold.argtypes = [vp, i32, i64, f32, f32, vp, vp]
    lib.oracle_sparse_fc.restype = i32
    lib.oracle_sparse_fc.argtypes = [vp, vp, i64, i64, i32, vp, i32, i64, f32, f32, vp, vp, vp, vp, vp, vp, i32]
    lib.oracle_dense_fc.restype = i32
    lib.oracle_dense_fc.argtypes = [vp, vp, i64, i64, i32, vp, i32, i64, vp, vp]
    lib.oracle_fold_bias.restype = i32
    lib.oracle_fold_bias.argtypes = [vp, vp, i64, i64, i32, vp, f32, vp]
    lib.oracle_calibrate.restype = i32
    lib.oracle_calibrate.argtypes = [vp, i64, i64, i32, f32, i32, vp, vp]
    lib.oracle_swiglu_block.restype = i32
    lib.oracle_swiglu_block.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, i32, vp, i32, f32, f32, vp, vp,
                                        f32, f32, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32]
    lib.oracle_ffn_sparsity.restype = ctypes.c_double
    lib.oracle_ffn_sparsity.argtypes = [ctypes.c_double, ctypes.c_double]
    _lib = lib
    return lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _w_array(W: np.ndarray, wdt: int) -> np.ndarray:
    want = np.int8 if wdt == I8 else np.uint16
    W = np.ascontiguousarray(W)
    if W.dtype != want:
        raise TypeError(f"weights for dtype code {wdt} must be {want}, got {W.dtype}")
    return W


def to_f32(bits: np.ndarray, dt: int) -> np.ndarray:
    lib = _load()
    flat = np.asarray(bits, dtype=np.uint16).ravel()
    return np.array([lib.oracle_to_f32(int(b), dt) for b in flat], dtype=np.float32).reshape(np.shape(bits))


def centre_threshold(x: np.ndarray, xdt: int, eta: float, tau: float) -> Tuple[np.ndarray, np.ndarray]:
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.uint16).ravel()
    d = np.empty(x.size, dtype=np.float32)
    keep = np.empty(x.size, dtype=np.uint8)
    lib.oracle_centre_threshold(_ptr(x), xdt, x.size, eta, tau, _ptr(d), _ptr(keep))
    return d, keep.astype(bool)


def sparse_fc(W: np.ndarray, x: np.ndarray, eta: float, tau: float, b_fused: Optional[np.ndarray],
              wdt: int, xdt: int, col_scale: Optional[np.ndarray] = None, nthreads: int = 1) -> dict:
    """Returns dict(y [B,N] f32, idx list of per-token int32 arrays, nnz [B], union_idx, union_nnz)."""
    lib = _load()
    W = _w_array(W, wdt)
    K, N = W.shape
    x = np.ascontiguousarray(x, dtype=np.float32 if xdt == F32 else np.uint16).reshape(-1, K)
    B = x.shape[0]
    if b_fused is not None:
        b_fused = np.ascontiguousarray(b_fused, dtype=np.float32)
        assert b_fused.shape == (N,)
    if col_scale is not None:
        col_scale = np.ascontiguousarray(col_scale, dtype=np.uint16)
    y = np.empty((B, N), dtype=np.float32)
    idx = np.full((B, K), -1, dtype=np.int32)
    nnz = np.zeros(B, dtype=np.int32)
    uidx = np.full(K, -1, dtype=np.int32)
    unnz = np.zeros(1, dtype=np.int32)
    rc = lib.oracle_sparse_fc(_ptr(W), _ptr(col_scale), K, N, wdt, _ptr(x), xdt, B, eta, tau, _ptr(b_fused),
                              _ptr(y), _ptr(idx), _ptr(nnz), _ptr(uidx), _ptr(unnz), nthreads)
    if rc != 0:
        raise ValueError(f"oracle_sparse_fc failed: {rc}")
    return {"y": y, "idx": [idx[b, :nnz[b]].copy() for b in range(B)], "nnz": nnz,
            "union_idx": uidx[:unnz[0]].copy(), "union_nnz": int(unnz[0])}


def swiglu_block(W_gate: np.ndarray, W_up: np.ndarray, W_down: np.ndarray, x: np.ndarray, eta_x: float,
                 tau_x: float, eta_z: float, tau_z: float, wdt: int, xdt: int, b_gate=None, b_up=None, b_down=None,
                 gate_scale=None, up_scale=None, down_scale=None, nthreads: int = 1) -> dict:
    """SwiGLU block of one token (Appendix B Alg. 2 with the centred FC of Alg. 3).
    Returns dict(g, u, z [F] f32, y [N] f32, idx_x, idx_z int32 arrays)."""
    lib = _load()
    W_gate, W_up, W_down = _w_array(W_gate, wdt), _w_array(W_up, wdt), _w_array(W_down, wdt)
    K, F = W_gate.shape
    assert W_up.shape == (K, F) and W_down.shape[0] == F
    N = W_down.shape[1]
    x = np.ascontiguousarray(x, dtype=np.uint16).reshape(K)

    def f32(a, n):
        if a is None:
            return None
        a = np.ascontiguousarray(a, dtype=np.float32)
        assert a.shape == (n,)
        return a

    def u16(a):
        return None if a is None else np.ascontiguousarray(a, dtype=np.uint16)

    b_gate, b_up, b_down = f32(b_gate, F), f32(b_up, F), f32(b_down, N)
    gate_scale, up_scale, down_scale = u16(gate_scale), u16(up_scale), u16(down_scale)
    g, u, z = (np.empty(F, dtype=np.float32) for _ in range(3))
    y = np.empty(N, dtype=np.float32)
    idx_x, idx_z = np.full(K, -1, dtype=np.int32), np.full(F, -1, dtype=np.int32)
    nnz_x, nnz_z = np.zeros(1, dtype=np.int32), np.zeros(1, dtype=np.int32)
    rc = lib.oracle_swiglu_block(_ptr(W_gate), _ptr(gate_scale), _ptr(W_up), _ptr(up_scale), _ptr(W_down),
                                 _ptr(down_scale), K, F, N, wdt, _ptr(x), xdt, eta_x, tau_x, _ptr(b_gate), _ptr(b_up),
                                 eta_z, tau_z, _ptr(b_down), _ptr(g), _ptr(u), _ptr(z), _ptr(y), _ptr(idx_x),
                                 _ptr(nnz_x), _ptr(idx_z), _ptr(nnz_z), nthreads)
    if rc != 0:
        raise ValueError(f"oracle_swiglu_block failed: {rc}")
    return {"g": g, "u": u, "z": z, "y": y, "idx_x": idx_x[:nnz_x[0]].copy(), "idx_z": idx_z[:nnz_z[0]].copy()}


def dense_fc(W: np.ndarray, x: np.ndarray, bias: Optional[np.ndarray], wdt: int, xdt: int,
             col_scale: Optional[np.ndarray] = None) -> np.ndarray:
    lib = _load()
    W = _w_array(W, wdt)
    K, N = W.shape
    x = np.ascontiguousarray(x, dtype=np.uint16).reshape(-1, K)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
    if col_scale is not None:
        col_scale = np.ascontiguousarray(col_scale, dtype=np.uint16)
    y = np.empty((x.shape[0], N), dtype=np.float32)
    rc = lib.oracle_dense_fc(_ptr(W), _ptr(col_scale), K, N, wdt, _ptr(x), xdt, x.shape[0], _ptr(bias), _ptr(y))
    if rc != 0:
        raise ValueError(f"oracle_dense_fc failed: {rc}")
    return y


def fold_bias(W: np.ndarray, eta: float, bias: Optional[np.ndarray], wdt: int,
              col_scale: Optional[np.ndarray] = None) -> np.ndarray:
    lib = _load()
    W = _w_array(W, wdt)
    K, N = W.shape
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
    if col_scale is not None:
        col_scale = np.ascontiguousarray(col_scale, dtype=np.uint16)
    out = np.empty(N, dtype=np.float32)
    rc = lib.oracle_fold_bias(_ptr(W), _ptr(col_scale), K, N, wdt, _ptr(bias), eta, _ptr(out))
    if rc != 0:
        raise ValueError(f"oracle_fold_bias failed: {rc}")
    return out


def calibrate(X: np.ndarray, xdt: int, s: float, est: int = MODE_MEDIAN) -> Tuple[float, float]:
    """Returns (eta, tau) as Python floats holding exact fp32 values."""
    lib = _load()
    X = np.ascontiguousarray(X, dtype=np.uint16)
    n, K = X.shape
    eta = np.zeros(1, dtype=np.float32)
    tau = np.zeros(1, dtype=np.float32)
    rc = lib.oracle_calibrate(_ptr(X), n, K, xdt, s, est, _ptr(eta), _ptr(tau))
    if rc != 0:
        raise ValueError(f"oracle_calibrate failed: {rc}")
    return float(eta[0]), float(tau[0])


def ffn_sparsity(s_x: float, s_gated: float) -> float:
    return float(_load().oracle_ffn_sparsity(s_x, s_gated))
