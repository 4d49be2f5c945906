"""Pins for the CPU oracle: every check compares it with something other than itself --
a library routine (numpy / torch / scipy), exact integer arithmetic, a closed form, an
invariant the paper states, or numbers the paper prints."""
import itertools
import math
import os

import numpy as np
import pytest
import torch
from scipy import integrate, optimize, special

import oracle
import workloads as wl
from workloads import BF16, F16, I8

pytestmark = pytest.mark.filterwarnings("ignore")


# ------------------------------------------------------------------ storage conversion
def test_f16_widening_matches_numpy_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.to_f32(bits, F16)
    want = bits.view(np.float16).astype(np.float32)
    assert np.array_equal(got.view(np.uint32)[~np.isnan(want)], want.view(np.uint32)[~np.isnan(want)])
    assert np.isnan(got[np.isnan(want)]).all()


def test_bf16_widening_matches_torch_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.to_f32(bits, BF16)
    want = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).float().numpy()
    ok = ~np.isnan(want)
    assert np.array_equal(got.view(np.uint32)[ok], want.view(np.uint32)[ok])
    assert np.isnan(got[~ok]).all()


# ------------------------------------------------------------------ Eq. 1: tau = 0, eta = 0 is the dense GEMV
@pytest.mark.parametrize("dt", [F16, BF16])
@pytest.mark.parametrize("K,N,B", [(37, 24, 1), (256, 72, 3), (1000, 8, 2)])
def test_tau_zero_is_dense_gemv(dt, K, N, B):
    W = wl.weights(K, N, 11, dt)
    x = wl.laplace(B, K, 12, dt, loc=0.0, scale=1.0)
    bias = np.random.default_rng(13).standard_normal(N).astype(np.float32)
    want = wl.decode(x, dt).astype(np.float64) @ wl.decode(W, dt).astype(np.float64) + bias.astype(np.float64)
    got = oracle.sparse_fc(W, x, 0.0, 0.0, bias, dt, dt)
    assert np.allclose(got["y"], want, rtol=0, atol=np.abs(want).max() * 2 ** -23)
    dense = oracle.dense_fc(W, x, bias, dt, dt)
    assert np.allclose(dense, want, rtol=0, atol=np.abs(want).max() * 2 ** -23)
    # every nonzero entry is kept; exact zeros are pruned by the strict compare and add nothing
    for b in range(B):
        assert np.array_equal(got["idx"][b], np.nonzero(wl.decode(x[b], dt) != 0)[0])


# ------------------------------------------------------------------ Eq. 4-6: centring changes nothing before pruning
@pytest.mark.parametrize("eta", [0.1, -3.7, 12.5])
def test_mode_centring_identity(eta):
    K, N = 512, 64
    W = wl.weights(K, N, 21, BF16)
    x = wl.laplace(2, K, 22, BF16, loc=eta, scale=0.7)
    bias = np.random.default_rng(23).standard_normal(N).astype(np.float32)
    Wd, xd = wl.decode(W, BF16).astype(np.float64), wl.decode(x, BF16).astype(np.float64)
    want = xd @ Wd + bias
    bf = oracle.fold_bias(W, eta, bias, BF16)
    got = oracle.sparse_fc(W, x, eta, 0.0, bf, BF16, BF16)["y"]
    rel = np.linalg.norm(got - want) / np.linalg.norm(want)
    assert rel < 1e-6
    # and the fused bias itself is b + eta * column sums (library routine)
    eta32 = float(np.float32(eta))
    assert np.allclose(bf, bias + eta32 * Wd.sum(axis=0), rtol=0, atol=1e-6)


def test_fold_bias_without_bias_and_transposition():
    K, N = 48, 16
    W = wl.weights(K, N, 31, F16, std=1.0)
    Wd = wl.decode(W, F16).astype(np.float64)
    bf = oracle.fold_bias(W, 2.0, None, F16)
    assert bf.shape == (N,)
    assert np.allclose(bf, 2.0 * Wd.sum(axis=0), rtol=1e-6, atol=1e-6)
    assert not np.allclose(bf[:K][:N], (2.0 * Wd.sum(axis=1))[:N], atol=1e-3)


# ------------------------------------------------------------------ Eq. 2 / Alg. 3 on tiny exact cases
def _int_case(K, N, seed):
    rng = np.random.default_rng(seed)
    xi = rng.integers(-6, 7, size=K)
    Wi = rng.integers(-4, 5, size=(K, N))
    bi = rng.integers(-9, 10, size=N)
    return xi, Wi, bi


@pytest.mark.parametrize("dt", [F16, BF16])
def test_bruteforce_integer_cases_all_thresholds(dt):
    """Integers are exact in 16-bit storage and in every sum, so y must match integer arithmetic
    bit for bit, for every threshold that changes the mask and for zero and non-zero modes."""
    K, N = 8, 8
    for seed in range(6):
        xi, Wi, bi = _int_case(K, N, seed)
        x, W = wl.encode(xi.astype(np.float32), dt), wl.encode(Wi.astype(np.float32), dt)
        for eta in (0, 2, -3):
            bf_int = bi + eta * Wi.sum(axis=0)
            bf = oracle.fold_bias(W, float(eta), bi.astype(np.float32), dt)
            assert np.array_equal(bf, bf_int.astype(np.float32))
            for tau in range(0, 11):
                keep = [i for i in range(K) if abs(int(xi[i]) - eta) > tau]
                want = [int(bf_int[o]) + sum((int(xi[i]) - eta) * int(Wi[i, o]) for i in keep) for o in range(N)]
                got = oracle.sparse_fc(W, x, float(eta), float(tau), bf, dt, dt)
                assert got["idx"][0].tolist() == keep
                assert int(got["nnz"][0]) == len(keep)
                assert got["y"][0].tolist() == [float(v) for v in want]


def test_every_mask_of_eight_channels():
    """All 2^8 masks: channel i holds +-(i+2) when kept-to-be and +-1 when not; tau = 1."""
    K, N = 8, 8
    Wi = np.random.default_rng(5).integers(-3, 4, size=(K, N))
    W = wl.encode(Wi.astype(np.float32), BF16)
    for bits in itertools.product((0, 1), repeat=K):
        xi = np.array([(i + 2) * (-1) ** i if b else (-1) ** i for i, b in enumerate(bits)])
        x = wl.encode(xi.astype(np.float32), BF16)
        got = oracle.sparse_fc(W, x, 0.0, 1.0, None, BF16, BF16)
        keep = [i for i, b in enumerate(bits) if b]
        assert got["idx"][0].tolist() == keep
        want = [sum(int(xi[i]) * int(Wi[i, o]) for i in keep) for o in range(N)]
        assert got["y"][0].tolist() == [float(v) for v in want]


def test_threshold_is_strict():
    """Eq. 2 keeps |x| > tau: an entry whose importance equals tau is pruned."""
    x = wl.encode(np.array([0.5, -0.5, 0.50390625, -0.25, 1.0], dtype=np.float32), BF16)
    W = wl.encode(np.eye(5, 8, dtype=np.float32), BF16)
    got = oracle.sparse_fc(W, x, 0.0, 0.5, None, BF16, BF16)
    assert got["idx"][0].tolist() == [2, 4]
    d, keep = oracle.centre_threshold(x, BF16, 0.25, 0.25)
    assert keep.tolist() == [False, True, True, True, True]
    assert d.tolist() == [0.25, -0.75, 0.25390625, -0.5, 0.75]


def test_centred_value_multiplies_the_weights():
    """Alg. 3: the product uses x - eta, not x; with W = identity, y - b_fused is the masked d."""
    xs = np.array([3.0, 1.0, -2.0, 0.5, 7.0, 1.25, 1.0, 0.0], dtype=np.float32)
    x, W = wl.encode(xs, F16), wl.encode(np.eye(8, dtype=np.float32), F16)
    got = oracle.sparse_fc(W, x, 1.0, 0.5, None, F16, F16)
    assert got["y"][0].tolist() == [2.0, 0.0, -3.0, 0.0, 6.0, 0.0, 0.0, -1.0]
    assert got["idx"][0].tolist() == [0, 2, 4, 7]


def test_subtraction_is_single_precision():
    """d = fp32(x) - eta is rounded once to fp32: 1 - 2^-25 lies halfway between two fp32 values
    and ties-to-even gives exactly 1.0 (a wider subtraction would return 1 - 2^-25)."""
    x = wl.encode(np.array([1.0] * 8, dtype=np.float32), BF16)
    d, keep = oracle.centre_threshold(x, BF16, float(np.float32(2.0 ** -25)), float(np.float32(1 - 2.0 ** -24)))
    assert d.tolist() == [1.0] * 8 and keep.all()


def test_nonfinite_inputs():
    xs = np.array([np.nan, np.inf, -0.0, 0.0, 1.0, -1.0, 0.25, 2.0], dtype=np.float32)
    x = wl.encode(xs, BF16)
    W = wl.encode(np.eye(8, dtype=np.float32), BF16)
    got = oracle.sparse_fc(W, x, 0.0, 0.5, None, BF16, BF16)
    assert got["idx"][0].tolist() == [1, 4, 5, 7]              # NaN is pruned, the infinity is kept
    y = got["y"][0]
    assert y[1] == np.inf                                      # inf * 1
    assert np.isnan(y[[0, 2, 3, 4, 5, 6, 7]]).all()            # inf * 0 in every other column, as IEEE says
    xs[1] = -4.0
    got = oracle.sparse_fc(W, wl.encode(xs, BF16), 0.0, 0.5, None, BF16, BF16)
    assert got["y"][0].tolist() == [0.0, -4.0, 0.0, 0.0, 1.0, -1.0, 0.0, 2.0]   # the NaN never reaches y


def test_nothing_kept_returns_fused_bias():
    K, N = 64, 16
    W = wl.weights(K, N, 41, BF16)
    x = wl.laplace(1, K, 42, BF16)
    bf = np.random.default_rng(43).standard_normal(N).astype(np.float32)
    got = oracle.sparse_fc(W, x, 0.0, 1e9, bf, BF16, BF16)
    assert int(got["nnz"][0]) == 0 and got["idx"][0].size == 0
    assert np.array_equal(got["y"][0], bf)


def test_shared_mask_concatenated_weights():
    """Up and Gate read one input, hence one mask: the FC on [W_gate | W_up] is the two FCs side by side."""
    K, N = 300, 40
    Wg, Wu = wl.weights(K, N, 51, BF16), wl.weights(K, N, 52, BF16)
    x = wl.prenorm(1, K, 53, BF16, chan_seed=54)
    a = oracle.sparse_fc(Wg, x, 0.0, 0.8, None, BF16, BF16)
    b = oracle.sparse_fc(Wu, x, 0.0, 0.8, None, BF16, BF16)
    c = oracle.sparse_fc(np.concatenate([Wg, Wu], axis=1), x, 0.0, 0.8, None, BF16, BF16)
    assert np.array_equal(a["idx"][0], c["idx"][0]) and np.array_equal(b["idx"][0], c["idx"][0])
    assert np.array_equal(c["y"][0], np.concatenate([a["y"][0], b["y"][0]]))


def test_threaded_column_split_is_identical():
    K, N = 700, 104
    W = wl.weights(K, N, 61, F16)
    x = wl.laplace(2, K, 62, F16)
    a = oracle.sparse_fc(W, x, 0.1, 0.3, None, F16, F16, nthreads=1)
    b = oracle.sparse_fc(W, x, 0.1, 0.3, None, F16, F16, nthreads=5)
    assert np.array_equal(a["y"], b["y"])


def test_sparse_fc_equals_masked_dense_library_gemv():
    """Eq. 3 with a library matmul: zero the pruned entries of d, multiply, add the bias."""
    K, N = 2048, 48
    W = wl.weights(K, N, 71, BF16)
    x = wl.swiglu(3, K, 72, BF16)
    eta, tau = 0.015625, 0.2
    bf = np.random.default_rng(73).standard_normal(N).astype(np.float32)
    xf = wl.decode(x, BF16)
    d = (xf - np.float32(eta)).astype(np.float32)
    keep = np.abs(d) > np.float32(tau)
    want = (d * keep).astype(np.float64) @ wl.decode(W, BF16).astype(np.float64) + bf
    got = oracle.sparse_fc(W, x, eta, tau, bf, BF16, BF16)
    assert np.allclose(got["y"], want, rtol=0, atol=2e-7 * np.abs(want).max())
    for b in range(3):
        assert np.array_equal(got["idx"][b], np.nonzero(keep[b])[0])
    assert np.array_equal(got["union_idx"], np.nonzero(keep.any(axis=0))[0])
    assert got["union_nnz"] == int(keep.any(axis=0).sum())


def test_int8_weights_with_column_scales():
    K, N = 256, 32
    q, scale = wl.quantize_i8(K, N, 81)
    x = wl.swiglu(2, K, 82, BF16)
    sc = scale.view(np.float16).astype(np.float64)
    xf = wl.decode(x, BF16)
    keep = np.abs(xf) > np.float32(0.1)
    want = ((xf * keep).astype(np.float64) @ q.astype(np.float64)) * sc[None, :]
    got = oracle.sparse_fc(q, x, 0.0, 0.1, None, I8, BF16, col_scale=scale)
    assert np.allclose(got["y"], want, rtol=0, atol=2e-7 * np.abs(want).max())
    bf = oracle.fold_bias(q, 0.5, None, I8, col_scale=scale)
    assert np.allclose(bf, 0.5 * q.astype(np.float64).sum(axis=0) * sc, rtol=1e-6, atol=1e-7)


# ------------------------------------------------------------------ calibration: tau = Quantile(|X - eta|, s)
@pytest.mark.parametrize("s", [0.0, 0.3, 0.5, 0.7, 0.9, 0.999])
def test_quantile_is_the_inverted_cdf_order_statistic(s):
    X = wl.laplace(64, 257, 91, F16)
    eta, tau = oracle.calibrate(X, F16, s, oracle.MODE_ZERO)
    v = np.abs(wl.decode(X, F16)).ravel()
    assert eta == 0.0
    if s == 0.0:
        assert tau == 0.0
    else:
        assert tau == float(np.quantile(v, float(np.float32(s)), method="inverted_cdf"))
    # thresholding the calibration sample with tau prunes at least the target share
    pruned = float((v <= np.float32(tau)).mean())
    ties = float((v == np.float32(tau)).mean())
    assert s - 1e-7 <= pruned <= s + ties + 1.0 / v.size


def test_median_and_mean_estimators_match_numpy():
    for n, K in [(64, 257), (63, 257)]:      # even and odd pooled count
        X = wl.laplace(n, K, 92, BF16, loc=0.3, scale=0.4)
        v = wl.decode(X, BF16).ravel()
        eta_med, tau_med = oracle.calibrate(X, BF16, 0.5, oracle.MODE_MEDIAN)
        assert eta_med == float(np.float32(np.median(v.astype(np.float64))))
        eta_mean, _ = oracle.calibrate(X, BF16, 0.5, oracle.MODE_MEAN)
        assert abs(eta_mean - v.astype(np.float64).mean()) <= 1e-7
        imp = np.abs((v - np.float32(eta_med)).astype(np.float32))
        assert tau_med == float(np.quantile(imp, 0.5, method="inverted_cdf"))


def test_paper_example_quantile_03_gives_30_percent():
    """Text after Eq. 2: thresholding at Quantile(|X_calib|, 0.3) is expected to give 30 % sparsity."""
    X = wl.prenorm(256, 512, 93, BF16, chan_seed=94)
    _, tau = oracle.calibrate(X, BF16, 0.3, oracle.MODE_ZERO)
    fresh = wl.prenorm(256, 512, 95, BF16, chan_seed=94)
    d, keep = oracle.centre_threshold(fresh.ravel(), BF16, 0.0, tau)
    s_hat = 1.0 - keep.mean()
    m = fresh.size
    assert abs(s_hat - 0.3) <= 5 * math.sqrt(0.3 * 0.7 * 2 / m) + 0.004   # + bf16 tie mass at tau


def _laplace_sites():
    return wl.sites(1)[0]


def test_config1_closed_form_tau_and_mode():
    """|x - 0.1| ~ Exp(scale 0.5) for Laplace(0.1, 0.5): tau(s) = -0.5 ln(1 - s)."""
    site = wl.sites(1)[0]
    X = site.calib()
    for s in (0.5, 0.7, 0.9):
        eta, tau = oracle.calibrate(X, site.xdt, s, oracle.MODE_MEDIAN)
        assert abs(eta - 0.1) < 0.005
        assert abs(tau - (-0.5 * math.log(1 - s))) < 0.012 * (-0.5 * math.log(1 - s)) + 0.002
    eta, tau = oracle.calibrate(X, site.xdt, 0.5, oracle.MODE_MEDIAN)
    assert abs(tau - 0.34657) < 0.004
    # fresh vectors of the same law come out at the target sparsity
    T = site.test_vectors(64)
    _, keep = oracle.centre_threshold(T.ravel(), site.xdt, eta, tau)
    s_hat = 1 - keep.mean()
    assert abs(s_hat - 0.5) <= 5 * math.sqrt(0.25 * (1 / T.size + 1 / X.size)) + 0.002


def _tau_prenorm(s):
    f = lambda t: integrate.quad(lambda c: special.erf(t / (c * math.sqrt(2))), 0.5, 2.0)[0] / 1.5 - s
    return optimize.brentq(f, 1e-6, 20)


def _tau_swiglu(s):
    def cdf(t):
        g = lambda z: special.erf(t / (abs(z / (1 + math.exp(-z))) * math.sqrt(2) + 1e-300)) * math.exp(-z * z / 2)
        return integrate.quad(g, -12, 12, limit=400, points=[0.0])[0] / math.sqrt(2 * math.pi)
    return optimize.brentq(lambda t: cdf(t) - s, 1e-6, 20)


@pytest.mark.parametrize("s", [0.5, 0.7, 0.9])
def test_config2_tau_against_quadrature(s):
    """tau from the sample against the quantile of the generating law, by numerical integration:
    z*c, c~U(0.5,2):  E_c erf(tau/(c sqrt2)) = s;   SiLU(g)*u:  E_g erf(tau/(|SiLU(g)| sqrt2)) = s."""
    a, b = wl.sites(2)
    Xa = wl.prenorm(128, a.K, a.seed_calib, a.xdt, chan_seed=a.seed_w + 500)
    _, tau_a = oracle.calibrate(Xa, a.xdt, s, oracle.MODE_ZERO)
    c = np.sort(np.random.default_rng(a.seed_w + 500).uniform(0.5, 2.0, size=a.K))
    # the channel scales are a finite draw: use their empirical law for the reference quantile
    ref_a = optimize.brentq(lambda t: special.erf(t / (c * math.sqrt(2))).mean() - s, 1e-6, 20)
    assert abs(tau_a - ref_a) < 0.02 * ref_a
    assert abs(ref_a - _tau_prenorm(s)) < 0.03 * ref_a
    Xb = wl.swiglu(64, b.K, b.seed_calib, b.xdt)
    eta_b, tau_b = oracle.calibrate(Xb, b.xdt, s, oracle.MODE_MEDIAN)
    ref_b = _tau_swiglu(s)
    assert abs(tau_b - ref_b) < 0.02 * ref_b
    assert abs(eta_b) < 0.01


def test_mode_centring_raises_sparsity_closed_form():
    """Same tau with and without centring on Laplace(loc, 0.5): uncentred sparsity is
    P(|x| <= tau) = exp(-loc/b) sinh(tau/b) for tau < loc; centred it is 1 - exp(-tau/b)."""
    loc, b, tau = 1.0, 0.5, 0.34657
    X = wl.laplace(256, 1024, 101, F16, loc=loc, scale=b)
    _, keep_c = oracle.centre_threshold(X.ravel(), F16, loc, tau)
    _, keep_u = oracle.centre_threshold(X.ravel(), F16, 0.0, tau)
    s_c, s_u = 1 - keep_c.mean(), 1 - keep_u.mean()
    assert abs(s_c - (1 - math.exp(-tau / b))) < 0.006
    assert abs(s_u - math.exp(-loc / b) * math.sinh(tau / b)) < 0.006
    assert s_c - s_u > 0.35      # a gap of about 40 points, the size the mode-centring figure shows


def test_hist_mode_lands_near_the_closed_form_mode():
    X = wl.laplace(256, 1024, 102, F16, loc=1.0, scale=0.5)
    eta, tau = oracle.calibrate(X, F16, 0.5, oracle.MODE_HIST)
    assert abs(eta - 1.0) < 0.04
    assert abs(tau - 0.34657) < 0.03


@pytest.mark.parametrize("B", [1, 4, 16])
def test_union_density_iid(B):
    """Appendix C: rows needed by a batch are the union of the masks; for i.i.d. channels at
    per-token sparsity s the expected union density is 1 - s^B."""
    K = 14336
    calib = wl.swiglu(64, K, 111, BF16)
    x = wl.swiglu(B, K, 112, BF16)
    W = wl.encode(np.zeros((K, 8), dtype=np.float32), BF16)
    prev = 0
    for s in (0.9, 0.7, 0.5):
        _, tau = oracle.calibrate(calib, BF16, s, oracle.MODE_ZERO)
        got = oracle.sparse_fc(W, x, 0.0, tau, None, BF16, BF16)
        dens = got["union_nnz"] / K
        want = 1 - s ** B
        assert abs(dens - want) < 5 * math.sqrt(max(want * (1 - want), 1e-4) / K) + 0.01
        assert got["union_nnz"] >= max(int(n) for n in got["nnz"])
        assert got["union_nnz"] >= prev
        prev = got["union_nnz"]


def test_ffn_sparsity_rows_printed_in_the_paper(golden_dir):
    rows = np.loadtxt(os.path.join(golden_dir, "ffn_sparsity_rows.txt"))
    assert rows.shape == (25, 4)
    for up, gate, down, ffn in rows:
        assert up == gate
        assert abs(oracle.ffn_sparsity(up, down) - ffn) <= 0.1 + 1e-9   # inputs are themselves rounded to 0.1
