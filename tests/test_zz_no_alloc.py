"""scap_sparse_fc_static -- the entry point for callers that cannot allocate (HIP graph capture, serving loops):
same kernels as scap_sparse_fc with the workspace held in a fixed array inside the library.  Its outputs must be
those of scap_sparse_fc bit for bit (and so within the oracle's bar), on consecutive calls that share the array,
the second smaller than the first."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2412_07174_amd as scap
import workloads as wl
from workloads import BF16, F16, I8

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import Layer, assert_y_close, f32_dev, to_dev


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def both_ways(layer, x_bits, xdt, m, tau, bf):
    """One call through scap_sparse_fc (own workspace) and one through scap_sparse_fc_static; returns both."""
    x_bits = np.ascontiguousarray(x_bits, dtype=np.uint16).reshape(-1, layer.K)
    B = x_bits.shape[0]
    x, b = to_dev(x_bits, xdt), f32_dev(bf)
    outs = []
    for static in (False, True):
        idx = torch.full((B, layer.K), -7, dtype=torch.int32, device="cuda")
        nnz = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        unz = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        y = torch.full((B, layer.N), float("nan"), dtype=torch.float32, device="cuda")
        if static:
            scap.sparse_fc_static(layer.W, x, m, tau, b, col_scale=layer.scale, y=y, idx_out=idx, nnz_out=nnz,
                                  union_nnz_out=unz)
        else:
            scap.sparse_fc(layer.W, x, m, tau, b, col_scale=layer.scale, y=y, idx_out=idx, nnz_out=nnz,
                           union_nnz_out=unz, workspace=layer.ws)
        torch.cuda.synchronize()
        nn = nnz.cpu().numpy()
        ih = idx.cpu().numpy()
        outs.append({"y": y.cpu().numpy(), "nnz": nn, "union": int(unz.item()),
                     "idx": [ih[t, :max(int(nn[t]), 0)].copy() for t in range(B)]})
    return outs


def same(a, b, what):
    assert np.array_equal(a["nnz"], b["nnz"]), f"{what}: counts {a['nnz']} vs {b['nnz']}"
    assert a["union"] == b["union"], f"{what}: union {a['union']} vs {b['union']}"
    for t in range(len(a["idx"])):
        assert np.array_equal(a["idx"][t], b["idx"][t]), f"{what}: kept list of token {t}"
    assert np.array_equal(a["y"].view(np.uint32), b["y"].view(np.uint32)), f"{what}: y differs in some bit"


def test_static_scratch_two_calls_in_a_row_second_smaller():
    big = Layer(wl.weights(4099, 1544, 971, BF16), BF16, B=4)
    small = Layer(wl.weights(333, 520, 972, F16), F16, B=4)
    cases = [(big, wl.laplace(1, 4099, 973, BF16), BF16, 0.1, 0.35, np.linspace(-1, 1, 1544).astype(np.float32)),
             (small, wl.laplace(1, 333, 974, F16), F16, 0.1, 0.2, None),
             (big, wl.laplace(3, 4099, 975, BF16), BF16, 0.1, 0.5, None),      # three tokens: larger partial sums
             (small, wl.laplace(2, 333, 976, F16), F16, 0.0, 0.0, None)]       # nothing pruned
    for n, (layer, X, xdt, m, tau, bf) in enumerate(cases):
        say(f"static scratch call {n}: K={layer.K} N={layer.N} B={X.shape[0]} tau={tau}")
        ws_way, static_way = both_ways(layer, X, xdt, m, tau, bf)
        same(ws_way, static_way, f"call {n}")
        want = oracle.sparse_fc(layer.W_host, X, m, tau, bf, layer.wdt, xdt)
        assert np.array_equal(static_way["nnz"], want["nnz"])
        for t in range(X.shape[0]):
            assert np.array_equal(static_way["idx"][t], want["idx"][t])
        assert static_way["union"] == want["union_nnz"]
        assert_y_close(static_way["y"], want["y"], f"call {n} against the oracle")


def test_static_scratch_headline_layer_then_int8():
    site = wl.sites(4)[1]          # 14336 -> 4096, bf16
    layer = Layer(site.make_weights(), site.wdt, B=1)
    _, tau = oracle.calibrate(site.calib(), site.xdt, 0.7, oracle.MODE_ZERO)
    X = site.draw(2, site.seed_test + 5)
    say("static scratch: 14336 x 4096 bf16, 70 %")
    a, b = both_ways(layer, X[0], site.xdt, 0.0, tau, None)
    same(a, b, "headline layer")
    Wq, sc = wl.quantize_i8(700, 2064, 977)
    q = Layer(Wq, I8, col_scale_bits=sc, B=1)
    say("static scratch: 700 x 2064 int8")
    a, b = both_ways(q, wl.laplace(1, 700, 978, BF16), BF16, 0.1, 0.3, None)
    same(a, b, "int8 after the large layer")
    a, b = both_ways(layer, X[1], site.xdt, 0.0, tau, None)
    same(a, b, "headline layer again")


def test_static_scratch_refuses_what_does_not_fit():
    K, N = 4096, 4096
    W = torch.zeros((K, N), dtype=torch.bfloat16, device="cuda")
    y = torch.full((16, N), 7.0, dtype=torch.float32, device="cuda")
    x = torch.zeros((16, K), dtype=torch.bfloat16, device="cuda")
    assert scap.workspace_bytes(K, N, 16) > scap.STATIC_SCRATCH_BYTES
    with pytest.raises(scap.ScapError) as e:
        scap.sparse_fc_static(W, x, 0.0, 0.1, None, y=y)
    assert e.value.status == -6
    torch.cuda.synchronize()
    assert bool((y == 7.0).all()), "a refused call must not write"
    # and the next call that fits still works
    y1 = torch.empty((1, N), dtype=torch.float32, device="cuda")
    scap.sparse_fc_static(W, x[0], 0.0, 0.1, None, y=y1)
    torch.cuda.synchronize()
    assert bool((y1 == 0).all())
