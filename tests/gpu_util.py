"""Helpers for the GPU parity tests: host bits -> device tensors, one call through the C ABI,
comparison against the CPU oracle at the stated bar."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2412_07174_amd as scap
import workloads as wl

# spec tolerance for y (16-bit storage, fp32 accumulation)
MAX_ABS = 1e-2
REL_L2 = 2e-3

_TORCH_DT = {wl.F16: torch.float16, wl.BF16: torch.bfloat16}


def to_dev(bits: np.ndarray, dt: int) -> torch.Tensor:
    if dt == wl.I8:
        return torch.from_numpy(np.ascontiguousarray(bits, dtype=np.int8)).cuda()
    t = torch.from_numpy(np.ascontiguousarray(bits, dtype=np.uint16).view(np.int16))
    return t.view(_TORCH_DT[dt]).cuda()


def f32_dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


class Layer:
    """Device copy of one layer plus a workspace."""

    def __init__(self, W_bits, wdt, col_scale_bits=None, B=16):
        self.W_host, self.wdt = W_bits, wdt
        self.K, self.N = W_bits.shape
        self.W = to_dev(W_bits, wdt)
        self.scale_host = col_scale_bits
        self.scale = None if col_scale_bits is None else to_dev(col_scale_bits, wl.F16)
        self.ws = scap.Workspace(self.K, self.N, B)


def gpu_sparse_fc(layer: Layer, x_bits, xdt, m, tau, bf, want_idx=True, cfg=None):
    x_bits = np.ascontiguousarray(x_bits, dtype=np.uint16).reshape(-1, layer.K)
    B = x_bits.shape[0]
    x = to_dev(x_bits, xdt)
    b = f32_dev(bf)
    idx = torch.full((B, layer.K), -7, dtype=torch.int32, device="cuda") if want_idx else None
    nnz = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    unz = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    y = torch.full((B, layer.N), float("nan"), dtype=torch.float32, device="cuda")
    scap.sparse_fc(layer.W, x, m, tau, b, col_scale=layer.scale, y=y, idx_out=idx, nnz_out=nnz, union_nnz_out=unz,
                   workspace=layer.ws, cfg=cfg)
    torch.cuda.synchronize()
    nn = nnz.cpu().numpy()
    out = {"y": y.cpu().numpy(), "nnz": nn, "union_nnz": int(unz.item())}
    if want_idx:
        ih = idx.cpu().numpy()
        out["idx"] = [ih[b, :nn[b]].copy() for b in range(B)]
    return out


def assert_y_close(got, want, what=""):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    fin = np.isfinite(want)
    assert np.array_equal(np.isnan(got), np.isnan(want)), f"{what}: NaN pattern differs"
    assert np.array_equal(got[~fin & ~np.isnan(want)], want[~fin & ~np.isnan(want)]), f"{what}: infinities differ"
    if fin.any():
        err = np.abs(got[fin] - want[fin]).max()
        den = np.linalg.norm(want[fin])
        rel = np.linalg.norm(got[fin] - want[fin]) / den if den > 0 else np.linalg.norm(got[fin] - want[fin])
        assert err <= MAX_ABS, f"{what}: max-abs {err}"
        assert rel <= REL_L2, f"{what}: rel-L2 {rel}"


def check_against_oracle(layer: Layer, x_bits, xdt, m, tau, bf, cfg=None, what=""):
    x_bits = np.ascontiguousarray(x_bits, dtype=np.uint16).reshape(-1, layer.K)
    want = oracle.sparse_fc(layer.W_host, x_bits, m, tau, bf, layer.wdt, xdt, col_scale=layer.scale_host)
    got = gpu_sparse_fc(layer, x_bits, xdt, m, tau, bf, cfg=cfg)
    assert np.array_equal(got["nnz"], want["nnz"]), f"{what}: nnz {got['nnz']} vs {want['nnz']}"
    for b in range(x_bits.shape[0]):
        assert np.array_equal(got["idx"][b], want["idx"][b]), f"{what}: kept-channel list of token {b} differs"
    assert got["union_nnz"] == want["union_nnz"], f"{what}: union {got['union_nnz']} vs {want['union_nnz']}"
    assert_y_close(got["y"], want["y"], what)
    return got, want
