"""Pins of the oracle's SwiGLU block (Appendix B Alg. 2 with the centred FC of Alg. 3) against things other
than itself: library matrix products and activation routines, exact integer arithmetic, set definitions."""
import numpy as np
import pytest
import torch
from scipy import special

import oracle
import workloads as wl
from workloads import BF16, F16


def _dense_block(Wg, Wu, Wd, x, dt, bg=None, bu=None, bd=None):
    """Dense SwiGLU feed-forward in fp64 with library routines (matmul, logistic function)."""
    xd = wl.decode(x, dt).astype(np.float64)
    g = xd @ wl.decode(Wg, dt).astype(np.float64) + (0 if bg is None else bg)
    u = xd @ wl.decode(Wu, dt).astype(np.float64) + (0 if bu is None else bu)
    z = u * g * special.expit(g)
    return g, u, z, z @ wl.decode(Wd, dt).astype(np.float64) + (0 if bd is None else bd)


# ------------------------------------------------------------------ nothing pruned: the block is the dense SwiGLU
@pytest.mark.parametrize("dt", [F16, BF16])
@pytest.mark.parametrize("K,F,N", [(48, 40, 24), (200, 328, 136)])
def test_block_without_pruning_is_the_dense_swiglu(dt, K, F, N):
    Wg, Wu, Wd = wl.weights(K, F, 1, dt, std=0.1), wl.weights(K, F, 2, dt, std=0.1), wl.weights(F, N, 3, dt, std=0.1)
    x = wl.laplace(1, K, 4, dt, loc=0.0, scale=1.0)[0]
    g, u, z, y = _dense_block(Wg, Wu, Wd, x, dt)
    got = oracle.swiglu_block(Wg, Wu, Wd, x, 0.0, 0.0, 0.0, 0.0, dt, dt)
    for name, want in (("g", g), ("u", u), ("z", z), ("y", y)):
        assert np.allclose(got[name], want, rtol=0, atol=np.abs(want).max() * 2 ** -21), name
    # exact zeros aside, every channel of x and of the gated product is kept
    assert np.array_equal(got["idx_x"], np.nonzero(wl.decode(x, dt) != 0)[0])
    assert np.array_equal(got["idx_z"], np.nonzero(got["z"] != 0)[0])


# ------------------------------------------------------------------ Eq. 4-6 inside the block: centring alone changes nothing
def test_block_centred_without_pruning_is_still_dense():
    K, F, N = 96, 160, 72   # K != F != N: feeding x instead of the gated product to the last call cannot pass
    dt = BF16
    Wg, Wu, Wd = wl.weights(K, F, 5, dt, std=0.1), wl.weights(K, F, 6, dt, std=0.1), wl.weights(F, N, 7, dt, std=0.1)
    x = wl.laplace(1, K, 8, dt, loc=0.3, scale=1.0)[0]
    rng = np.random.default_rng(9)
    bg, bu, bd = (rng.standard_normal(n).astype(np.float32) * 0.1 for n in (F, F, N))
    g, u, z, y = _dense_block(Wg, Wu, Wd, x, dt, bg, bu, bd)
    eta_x, eta_z = 0.3, -0.05
    got = oracle.swiglu_block(Wg, Wu, Wd, x, eta_x, 0.0, eta_z, 0.0, dt, dt,
                              b_gate=oracle.fold_bias(Wg, eta_x, bg, dt), b_up=oracle.fold_bias(Wu, eta_x, bu, dt),
                              b_down=oracle.fold_bias(Wd, eta_z, bd, dt))
    assert np.linalg.norm(got["z"] - z) / np.linalg.norm(z) < 1e-6
    assert np.linalg.norm(got["y"] - y) / np.linalg.norm(y) < 1e-6


# ------------------------------------------------------------------ the activation is silu(t) = t * logistic(t)
def test_gate_goes_through_silu_and_multiplies_up():
    K = 64
    eye = wl.encode(np.eye(K), BF16)
    two = wl.encode(2.0 * np.eye(K), BF16)
    x = wl.encode(np.linspace(-12.0, 12.0, K), BF16)
    xv = wl.decode(x, BF16).astype(np.float64)
    got = oracle.swiglu_block(eye, two, eye, x, 0.0, 0.0, 0.0, 0.0, BF16, BF16)
    want = (2.0 * xv) * torch.nn.functional.silu(torch.from_numpy(xv)).numpy()   # gate path carries the silu
    assert np.allclose(got["z"], want, rtol=2 ** -22, atol=1e-30)
    assert np.allclose(got["y"], want, rtol=2 ** -22, atol=1e-30)
    # swapping the roles of gate and up is a different function: silu(2x) * x
    swapped = oracle.swiglu_block(two, eye, eye, x, 0.0, 0.0, 0.0, 0.0, BF16, BF16)["z"]
    want_swapped = xv * torch.nn.functional.silu(torch.from_numpy(2.0 * xv)).numpy()
    assert np.allclose(swapped, want_swapped, rtol=2 ** -22, atol=1e-30)
    assert not np.allclose(swapped, want, rtol=1e-3, atol=1e-6)


# ------------------------------------------------------------------ exact integer case, both pruners active
def test_block_exact_integers_with_both_pruners():
    """Gate pre-activations are 0 or at least 40 in magnitude: silu(0) = 0, silu(t) = t to the last fp64 bit for
    t >= 40, |silu(t)| < 1e-15 for t <= -40.  Everything else is small integers, so every value is exact."""
    dt = BF16
    x_int = np.array([3, -1, 0, 2, -3, 1, -2, 1])            # tau_x = 1 keeps |x| > 1: channels 0, 3, 4, 6
    K, F, N = 8, 6, 8
    kept = [i for i in range(K) if abs(int(x_int[i])) > 1]
    Wg = np.zeros((K, F), dtype=np.int64)
    for i in range(K):
        s = int(np.sign(x_int[i])) if x_int[i] != 0 else 1
        Wg[i, 0] = 20 * s        # g_0 = 20 * sum |x_i| over kept  = 200
        Wg[i, 1] = -20 * s       # g_1 = -200: silu ~ 0
        Wg[i, 2] = 0             # g_2 = 0
        Wg[i, 3] = 10 * s        # g_3 = 100
        Wg[i, 4] = 4 * s         # g_4 = 40
        Wg[i, 5] = 7 * s if i in (1, 2, 5, 7) else 0   # only pruned channels feed it: g_5 = 0
    rng = np.random.default_rng(17)
    Wu = rng.integers(-3, 4, size=(K, F))
    Wd = rng.integers(-4, 5, size=(F, N))
    g = [sum(int(x_int[i]) * int(Wg[i, f]) for i in kept) for f in range(F)]
    u = [sum(int(x_int[i]) * int(Wu[i, f]) for i in kept) for f in range(F)]
    assert g == [200, -200, 0, 100, 40, 0]
    z = [u[f] * g[f] if g[f] >= 40 else 0 for f in range(F)]   # integers (the g = -200 channel is ~1e-85, not 0)
    for tau_z in (0.0, 5.0, float(sorted(abs(v) for v in z)[-2]), 1e9):
        keep_z = [f for f in range(F) if abs(z[f]) > tau_z]
        y = [sum(z[f] * int(Wd[f, o]) for f in keep_z) for o in range(N)]
        got = oracle.swiglu_block(wl.encode(Wg, dt), wl.encode(Wu, dt), wl.encode(Wd, dt), wl.encode(x_int, dt),
                                  0.0, 1.0, 0.0, tau_z, dt, dt)
        assert got["idx_x"].tolist() == kept
        assert got["g"].tolist() == [float(v) for v in g]
        assert got["u"].tolist() == [float(v) for v in u]
        if tau_z > 0:
            assert got["idx_z"].tolist() == keep_z
            assert got["z"][[0, 2, 3, 4, 5]].tolist() == [float(z[f]) for f in (0, 2, 3, 4, 5)]
            assert abs(got["z"][1]) < 1e-30
            assert got["y"].tolist() == [float(v) for v in y]
        else:
            # tau = 0 keeps the 1e-85-sized product as well (strict compare against 0); it adds nothing visible
            assert set(keep_z) <= set(got["idx_z"].tolist())
            assert np.allclose(got["y"], y, rtol=0, atol=1e-20)


# ------------------------------------------------------------------ masks are set definitions; shared first mask
def test_block_masks_on_synthetic_layer_inputs():
    dt = BF16
    K, F, N = 256, 384, 256
    site = wl.Site("toy_up", K, F, dt, dt, "prenorm", 64, 71, 72, 73)
    Wg, Wu, Wd = wl.weights(K, F, 31, dt), wl.weights(K, F, 32, dt), wl.weights(F, N, 33, dt)
    x = site.draw(1, 74)[0]
    eta_x, tau_x = oracle.calibrate(site.draw(64, 75), dt, 0.5, oracle.MODE_MEDIAN)
    dense = oracle.swiglu_block(Wg, Wu, Wd, x, 0.0, 0.0, 0.0, 0.0, dt, dt)
    tau_z = float(np.sort(np.abs(dense["z"]))[int(0.6 * F)])
    eta_z = 0.01
    bgf, buf = oracle.fold_bias(Wg, eta_x, None, dt), oracle.fold_bias(Wu, eta_x, None, dt)
    got = oracle.swiglu_block(Wg, Wu, Wd, x, eta_x, tau_x, eta_z, tau_z, dt, dt, b_gate=bgf, b_up=buf)
    # first mask: the one sparse_fc reports on the concatenated [gate | up] weights (shared mask)
    cat = oracle.sparse_fc(np.concatenate([Wg, Wu], axis=1), x, eta_x, tau_x, np.concatenate([bgf, buf]), dt, dt)
    assert np.array_equal(got["idx_x"], cat["idx"][0])
    assert np.array_equal(got["g"], cat["y"][0, :F]) and np.array_equal(got["u"], cat["y"][0, F:])
    # second mask: the strict compare on the fp32 gated product
    dz = got["z"] - np.float32(eta_z)
    assert dz.dtype == np.float32
    assert np.array_equal(got["idx_z"], np.nonzero(np.abs(dz) > np.float32(tau_z))[0])
    assert 0.2 * F < got["idx_z"].size < 0.6 * F
    # last call = sparse_fc on the fp32 gated product
    again = oracle.sparse_fc(Wd, got["z"], eta_z, tau_z, None, dt, oracle.F32)
    assert np.array_equal(again["y"][0], got["y"]) and np.array_equal(again["idx"][0], got["idx_z"])
    # weights skipped by the three FCs of an equal-sized block: Appendix B's 2/3 s_x + 1/3 s_z
    s_x, s_z = 1 - got["idx_x"].size / K, 1 - got["idx_z"].size / F
    skipped = (2 * (K - got["idx_x"].size) * F + (F - got["idx_z"].size) * N) / (2 * K * F + F * N)
    assert abs(skipped - oracle.ffn_sparsity(s_x, s_z)) < 1e-12


def test_fp32_activation_input_matches_its_16bit_twin():
    """An fp32 vector whose values are exactly representable in bf16 gives the same result either way."""
    K, N = 128, 40
    W = wl.weights(K, N, 41, BF16)
    x = wl.laplace(1, K, 42, BF16, loc=0.2, scale=0.5)
    a = oracle.sparse_fc(W, x, 0.2, 0.3, None, BF16, BF16)
    b = oracle.sparse_fc(W, wl.decode(x, BF16).astype(np.float32), 0.2, 0.3, None, BF16, oracle.F32)
    assert np.array_equal(a["y"], b["y"]) and np.array_equal(a["idx"][0], b["idx"][0])
