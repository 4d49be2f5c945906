"""GPU parity: every call goes through the C ABI of libscap.so and is compared with the CPU oracle on
the same seeded inputs -- kept-channel lists and counts bit-exact, y within max-abs 1e-2 and rel-L2 2e-3."""
import math
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
    from gpu_util import Layer, assert_y_close, check_against_oracle, f32_dev, gpu_sparse_fc, to_dev


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _calib(site, s, est="median"):
    return oracle.calibrate(site.calib(), site.xdt, s, oracle.EST[est])


# ------------------------------------------------------------------ small shapes: tiles, splits, ragged tails
SMALL = [
    # K, N: below one wave, ragged chunk, several splits, several column tiles, ragged last tile
    (1, 8), (63, 8), (64, 512), (65, 520), (200, 1032), (1000, 4096), (1024, 4104), (4099, 1544), (2048, 72),
]


@pytest.mark.parametrize("dt", [F16, BF16])
@pytest.mark.parametrize("K,N", SMALL)
def test_small_shapes(dt, K, N):
    W = wl.weights(K, N, 100 + K, dt)
    layer = Layer(W, dt, B=1)
    X = wl.laplace(3, K, 200 + K, dt, loc=0.2, scale=0.6)
    bf = np.random.default_rng(K).standard_normal(N).astype(np.float32)
    for tau in (0.0, 0.41, 1.4, 1e6):
        for b in range(X.shape[0]):
            say(f"small K={K} N={N} dt={dt} tau={tau} vec={b}")
            check_against_oracle(layer, X[b], dt, 0.2, tau, bf, what=f"K={K} N={N} tau={tau}")


@pytest.mark.parametrize("lanes", [64, 32])
@pytest.mark.parametrize("waves,unroll", [(4, 4), (4, 8), (4, 16), (8, 4), (8, 8), (8, 16), (16, 4), (16, 8), (16, 16)])
def test_every_launch_shape(waves, unroll, lanes):
    K, N = 3000, 1544
    W = wl.weights(K, N, 301, BF16)
    layer = Layer(W, BF16, B=1)
    x = wl.swiglu(1, K, 302, BF16)[0]
    bf = np.random.default_rng(303).standard_normal(N).astype(np.float32)
    for rows in (64, 192, 512, 1024, 3008):
        for tau in (0.05, 0.6):
            say(f"launch shape waves={waves} unroll={unroll} rows={rows} lanes={lanes} tau={tau}")
            check_against_oracle(layer, x, BF16, 0.0, tau, bf, cfg=(waves, rows, unroll, lanes),
                                 what=f"{waves}/{rows}/{unroll}/{lanes}")


# ------------------------------------------------------------------ the one-token kernel and the general kernel
ONE_TOKEN = [
    # K, N, dtype, rows per workgroup (0 = planner): one / two / four 512-channel chunks per wavefront, ragged
    # last chunk, an input whose length is not a multiple of 8, column tiles that are not a multiple of the 8
    # accelerator dies (so that a tile's workgroups sit on different dies), ragged last column tile
    (4099, 1544, BF16, 0), (4099, 1544, BF16, 1024), (4099, 1544, BF16, 2048), (777, 4096, F16, 0),
    (5000, 6144, BF16, 0), (2048, 11008, F16, 1024), (333, 8, BF16, 0), (6000, 2064, I8, 0), (3000, 5136, I8, 1536),
]


@pytest.mark.parametrize("K,N,dt,rows", ONE_TOKEN)
def test_one_token_kernel_shapes_and_both_hand_overs(K, N, dt, rows):
    """The one-token kernel against the oracle with each of its split-K hand-overs: fixed-point atomics (the
    default), and fp32 partial sums collected by the last arrival with ordinary loads (when all writers ran on the
    reader's own accelerator die) or with device-coherent loads -- those two bit-identical to each other --; and the
    general vector kernel; on repeated calls with changing inputs through one workspace."""
    if dt == I8:
        Wq, sc = wl.quantize_i8(K, N, 331 + K)
        layer = Layer(Wq, I8, col_scale_bits=sc, B=1)
        xdt = BF16
    else:
        layer = Layer(wl.weights(K, N, 331 + K, dt), dt, B=1)
        xdt = dt
    X = wl.laplace(6, K, 332 + K, xdt, loc=0.1, scale=0.5)
    bf = np.random.default_rng(K + N).standard_normal(N).astype(np.float32)
    for rep, tau in enumerate((0.0, 0.3, 0.35, 0.9, 2.5, 1e6)):
        x = X[rep]
        say(f"one-token K={K} N={N} dt={dt} rows={rows} tau={tau}")
        for unroll in (8, 16, 4):
            fx, _ = check_against_oracle(layer, x, xdt, 0.1, tau, bf, cfg=(8, rows, unroll, 64, 0),
                                         what=f"one-token K={K} N={N} rows={rows} unroll={unroll} tau={tau}")
            near, _ = check_against_oracle(layer, x, xdt, 0.1, tau, bf, cfg=(8, rows, unroll, 64, scap.CFG_PARTIAL_SUMS),
                                           what=f"one-token, partial sums K={K} N={N} rows={rows} unroll={unroll} tau={tau}")
            far = gpu_sparse_fc(layer, x, xdt, 0.1, tau, bf, cfg=(8, rows, unroll, 64, scap.CFG_DEVICE_SCOPE_LOADS))
            assert np.array_equal(near["y"].view(np.uint32), far["y"].view(np.uint32)), "partial-sum hand-overs differ"
            assert np.array_equal(near["idx"][0], far["idx"][0]) and np.array_equal(fx["idx"][0], far["idx"][0])
            again = gpu_sparse_fc(layer, x, xdt, 0.1, tau, bf, cfg=(8, rows, unroll, 64, 0))
            assert np.array_equal(fx["y"].view(np.uint32), again["y"].view(np.uint32)), "fixed-point hand-over not reproducible"
        check_against_oracle(layer, x, xdt, 0.1, tau, bf, cfg=(8, 0 if rows > 1024 else rows, 8, 64, scap.CFG_GENERAL_KERNEL),
                             what=f"general kernel K={K} N={N} tau={tau}")


@pytest.mark.parametrize("K,N,dt", [(4099, 1544, BF16), (777, 4096, F16), (64, 520, BF16), (6000, 2064, I8), (14336, 4096, BF16)])
def test_accumulate_into_y(K, N, dt):
    """The opt-in y += result mode of the one-token kernel (fp32 atomic adds, no split-K hand-over): y starts as a
    given addend, the result is the oracle's y plus that addend at the float tolerance (the order of the additions
    is not fixed), lists and counts are exact; dense mode likewise; calls that would need another kernel are refused."""
    if dt == I8:
        Wq, sc = wl.quantize_i8(K, N, 361 + K)
        layer = Layer(Wq, I8, col_scale_bits=sc, B=2)
        xdt = BF16
    else:
        layer = Layer(wl.weights(K, N, 361 + K, dt), dt, B=2)
        xdt = dt
    X = wl.laplace(4, K, 362 + K, xdt, loc=0.1, scale=0.5)
    bf = np.random.default_rng(K + N).standard_normal(N).astype(np.float32)
    addend = np.random.default_rng(7 * K + N).standard_normal(N).astype(np.float32)
    cfg = (0, 0, 0, 0, scap.CFG_ACCUMULATE)
    for rep, tau in enumerate((0.0, 0.3, 0.9, 1e6)):
        say(f"accumulate K={K} N={N} dt={dt} tau={tau}")
        want = oracle.sparse_fc(layer.W_host, X[rep], 0.1, tau, bf, dt, xdt, col_scale=layer.scale_host)
        y = f32_dev(addend).reshape(1, N).clone()
        idx = torch.full((1, K), -7, dtype=torch.int32, device="cuda")
        nnz = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        unz = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        scap.sparse_fc(layer.W, to_dev(X[rep], xdt), 0.1, tau, f32_dev(bf), col_scale=layer.scale, y=y, idx_out=idx,
                       nnz_out=nnz, union_nnz_out=unz, workspace=layer.ws, cfg=cfg)
        torch.cuda.synchronize()
        assert int(nnz.item()) == int(want["nnz"][0]) == int(unz.item())
        assert np.array_equal(idx.cpu().numpy()[0, :int(nnz.item())], want["idx"][0])
        assert_y_close(y.cpu().numpy()[0], want["y"][0] + addend, f"accumulate tau={tau}")
    say(f"accumulate K={K} N={N} dt={dt} dense, then an ordinary call on the same workspace")
    y = f32_dev(addend).reshape(1, N).clone()
    scap.dense_fc(layer.W, to_dev(X[0], xdt), f32_dev(bf), col_scale=layer.scale, y=y, workspace=layer.ws, cfg=cfg)
    torch.cuda.synchronize()
    assert_y_close(y.cpu().numpy()[0], oracle.dense_fc(layer.W_host, X[0], bf, dt, xdt, col_scale=layer.scale_host)[0] + addend, "accumulate dense")
    check_against_oracle(layer, X[1], xdt, 0.1, 0.3, bf, what="ordinary call after accumulate calls")
    with pytest.raises(scap.ScapError):
        scap.sparse_fc(layer.W, to_dev(X[:2], xdt), 0.1, 0.3, None, col_scale=layer.scale, workspace=layer.ws, cfg=cfg)
    with pytest.raises(scap.ScapError):
        scap.sparse_fc(layer.W, to_dev(X[0], xdt), 0.1, 0.3, None, col_scale=layer.scale, workspace=layer.ws,
                       cfg=(0, 0, 0, 0, scap.CFG_ACCUMULATE | scap.CFG_GENERAL_KERNEL))


FEW_TOKENS = [
    # K (a multiple of 8), N, dtype: one / two / four 512-channel chunks per wavefront, ragged last chunk, column
    # tiles that are not a multiple of the 8 accelerator dies, ragged last column tile, a single K split,
    # int8 weights with 8 and 16 bytes per lane
    (4096, 1544, BF16), (5000, 6144, BF16), (2048, 11008, F16), (776, 4096, F16), (336, 8, BF16), (64, 520, BF16),
    (6000, 2064, I8), (3000, 5136, I8), (14336, 4096, BF16),
]


@pytest.mark.parametrize("B", [2, 3, 4])
@pytest.mark.parametrize("K,N,dt", FEW_TOKENS)
def test_few_tokens_kernel_shapes_and_both_hand_overs(K, N, dt, B):
    """2 tokens on the two-token form of the one-token kernel, 3 and 4 tokens on its four-slot form (16-bit weights,
    input length a multiple of 8) or on whatever else the library picks for these shapes: against the oracle token by
    token -- y, every token's list and count, the union count --,
    with the kernel's default hand-over (repeatable bit for bit), and with ordinary and with device-coherent loads of
    the partial sums against each other bit for bit, and dense mode, on repeated calls with changing inputs through
    one workspace."""
    if dt == I8:
        Wq, sc = wl.quantize_i8(K, N, 351 + K)
        layer = Layer(Wq, I8, col_scale_bits=sc, B=4)
        xdt = BF16
    else:
        layer = Layer(wl.weights(K, N, 351 + K, dt), dt, B=4)
        xdt = dt
    X = wl.laplace(6 * B, K, 352 + K + B, xdt, loc=0.1, scale=0.5)
    bf = np.random.default_rng(K + N).standard_normal(N).astype(np.float32)
    for rep, tau in enumerate((0.0, 0.3, 0.35, 0.9, 2.5, 1e6)):
        x = X[rep * B:(rep + 1) * B]
        say(f"few tokens K={K} N={N} dt={dt} B={B} tau={tau}")
        what = f"few tokens K={K} N={N} B={B} tau={tau}"
        got, _ = check_against_oracle(layer, x, xdt, 0.1, tau, bf, what=what)  # the default hand-over of this kernel
        again = gpu_sparse_fc(layer, x, xdt, 0.1, tau, bf)
        assert np.array_equal(got["y"].view(np.uint32), again["y"].view(np.uint32)), "not reproducible"
        near, _ = check_against_oracle(layer, x, xdt, 0.1, tau, bf, cfg=(0, 0, 0, 0, scap.CFG_PARTIAL_SUMS), what=what)
        far = gpu_sparse_fc(layer, x, xdt, 0.1, tau, bf, cfg=(0, 0, 0, 0, scap.CFG_DEVICE_SCOPE_LOADS))
        assert np.array_equal(near["y"].view(np.uint32), far["y"].view(np.uint32)), "partial-sum hand-overs differ"
        for b in range(B):
            assert np.array_equal(near["idx"][b], far["idx"][b])
    say(f"few tokens K={K} N={N} dt={dt} B={B} dense")
    y = scap.dense_fc(layer.W, to_dev(X[:B], xdt), f32_dev(bf), col_scale=layer.scale, workspace=layer.ws)
    torch.cuda.synchronize()
    want = oracle.dense_fc(layer.W_host, X[:B], bf, dt, xdt, col_scale=layer.scale_host)
    assert_y_close(y.cpu().numpy(), want, "dense, few tokens")


def test_one_token_kernel_many_calls_in_a_row_both_hand_overs():
    """Back-to-back launches on one workspace with rotating weights and inputs (what the benchmark does): the
    ordinary-load hand-over must never see a partial sum of an earlier launch, and the fixed-point hand-over's
    words must be back at zero after every launch.  Every y of the partial-sum hand-over is compared bit for bit
    with the same call made with device-coherent loads; the fixed-point series is run twice and compared with
    itself bit for bit and with the partial-sum series at the float tolerance."""
    K, N = 14336, 4096
    Ws = [to_dev(wl.weights(K, N, 341 + i, BF16), BF16) for i in range(3)]
    X = to_dev(wl.swiglu(16, K, 345, BF16), BF16)
    ws = scap.Workspace(K, N, 1)
    calls = [(i % 3, i % 16, (0.05, 0.3, 0.8, 0.0)[i % 4]) for i in range(48)]
    ys = {}
    for key, flags in (("fx", 0), ("near", scap.CFG_PARTIAL_SUMS), ("far", scap.CFG_DEVICE_SCOPE_LOADS), ("fx again", 0)):
        out = torch.empty((len(calls), N), dtype=torch.float32, device="cuda")
        say(f"48 launches in a row, {key}")
        for n, (wi, xi, tau) in enumerate(calls):
            scap.sparse_fc(Ws[wi], X[xi], 0.0, tau, None, y=out[n:n + 1], workspace=ws, cfg=(8, 0, 8, 64, flags))
        torch.cuda.synchronize()
        ys[key] = out.cpu().numpy()
    assert np.array_equal(ys["near"].view(np.uint32), ys["far"].view(np.uint32))
    assert np.array_equal(ys["fx"].view(np.uint32), ys["fx again"].view(np.uint32))
    assert float(np.abs(ys["fx"] - ys["near"]).max()) < 1e-4
    ys[0] = ys["fx"]
    # and one of them against the oracle
    want = oracle.sparse_fc(wl.weights(K, N, 341 + 2, BF16), wl.swiglu(16, K, 345, BF16)[5], 0.0, 0.3, None, BF16, BF16)
    n = calls.index((2, 5, 0.3))
    assert_y_close(ys[0][n], want["y"][0], "launch in the middle of the series")


@pytest.mark.parametrize("dt", [F16, I8])
@pytest.mark.parametrize("lanes", [32])
def test_narrow_tiles_other_dtypes(dt, lanes):
    K, N = 1100, 2064 if dt == I8 else 1032
    if dt == I8:
        q, scale = wl.quantize_i8(K, N, 311)
        layer = Layer(q, I8, col_scale_bits=scale, B=1)
    else:
        layer = Layer(wl.weights(K, N, 311, dt), dt, B=1)
    x = wl.swiglu(1, K, 312, F16 if dt == F16 else BF16)[0]
    for rows in (128, 576):
        for tau in (0.0, 0.4):
            say(f"narrow tiles dt={dt} lanes={lanes} rows={rows} tau={tau}")
            check_against_oracle(layer, x, F16 if dt == F16 else BF16, 0.0, tau, None, cfg=(8, rows, 8, lanes),
                                 what=f"dt={dt} lanes={lanes}")


def test_invalid_launch_shape_is_rejected():
    layer = Layer(wl.weights(256, 512, 1, BF16), BF16, B=1)
    x = to_dev(wl.swiglu(1, 256, 2, BF16)[0], BF16)
    for cfg in [(3, 128, 8), (8, 100, 8), (8, 128, 5), (8, 128, 8, 48)]:
        with pytest.raises(scap.ScapError) as e:
            scap.sparse_fc(layer.W, x, 0.0, 0.1, None, workspace=layer.ws, cfg=cfg)
        assert e.value.status == -9


# ------------------------------------------------------------------ exact integer cases (bit-exact y)
@pytest.mark.parametrize("dt", [F16, BF16])
def test_integer_cases_are_bit_exact(dt):
    K, N = 96, 16
    rng = np.random.default_rng(7)
    xi, Wi, bi = rng.integers(-6, 7, size=K), rng.integers(-4, 5, size=(K, N)), rng.integers(-9, 10, size=N)
    layer = Layer(wl.encode(Wi.astype(np.float32), dt), dt, B=1)
    x = wl.encode(xi.astype(np.float32), dt)
    for eta in (0, 2, -3):
        bf_int = bi + eta * Wi.sum(axis=0)
        bfd = scap.fold_bias(layer.W, float(eta), f32_dev(bi.astype(np.float32)), workspace=layer.ws)
        assert bfd.cpu().numpy().tolist() == [float(v) for v in bf_int]
        for tau in range(0, 10):
            say(f"integer case dt={dt} eta={eta} tau={tau}")
            keep = [i for i in range(K) if abs(int(xi[i]) - eta) > tau]
            want = [int(bf_int[o]) + sum((int(xi[i]) - eta) * int(Wi[i, o]) for i in keep) for o in range(N)]
            got = gpu_sparse_fc(layer, x, dt, float(eta), float(tau), bf_int.astype(np.float32))
            assert got["idx"][0].tolist() == keep and int(got["nnz"][0]) == len(keep)
            assert got["y"][0].tolist() == [float(v) for v in want]


def test_ties_nonfinite_and_empty_mask():
    K, N = 256, 64
    W = wl.weights(K, N, 401, BF16)
    layer = Layer(W, BF16, B=1)
    xs = np.random.default_rng(402).choice(np.array([0.5, -0.5, 0.50390625, 0.25, 1.0, -2.0], dtype=np.float32), size=K)
    x = wl.encode(xs, BF16)
    say("ties at |d| == tau")
    got, want = check_against_oracle(layer, x, BF16, 0.0, 0.5, None, what="ties")
    assert int(want["nnz"][0]) == int((np.abs(xs) > 0.5).sum())
    xs2 = xs.copy()
    xs2[3], xs2[77] = np.nan, np.inf
    say("NaN and Inf inputs")
    check_against_oracle(layer, wl.encode(xs2, BF16), BF16, 0.0, 0.5, None, what="nonfinite")
    say("nothing kept")
    bf = np.random.default_rng(403).standard_normal(N).astype(np.float32)
    got = gpu_sparse_fc(layer, x, BF16, 0.0, 100.0, bf)
    assert int(got["nnz"][0]) == 0 and got["union_nnz"] == 0
    assert np.array_equal(got["y"][0], bf)


def test_two_tokens_ties_nonfinite_and_one_empty_mask():
    """The two-token kernel on the awkward inputs: ties at |d| == tau in one token, NaN and Inf in the other (its
    Inf row must not leak into the first token, whose value there is finite), then one token with nothing kept
    beside one with everything kept, then nothing kept at all."""
    K, N = 256, 64
    W = wl.weights(K, N, 411, BF16)
    layer = Layer(W, BF16, B=2)
    xs = np.random.default_rng(412).choice(np.array([0.5, -0.5, 0.50390625, 0.25, 1.0, -2.0], dtype=np.float32), size=K)
    xs2 = np.roll(xs, 5).copy()
    xs2[3], xs2[77] = np.nan, np.inf
    x = np.stack([wl.encode(xs, BF16), wl.encode(xs2, BF16)])
    say("two tokens: ties, NaN and Inf")
    got, want = check_against_oracle(layer, x, BF16, 0.0, 0.5, None, what="two tokens, ties and nonfinite")
    assert int(want["nnz"][0]) == int((np.abs(xs) > 0.5).sum())
    assert np.all(np.isfinite(got["y"][0])) and not np.all(np.isfinite(got["y"][1]))
    say("two tokens: one keeps nothing, one keeps everything")
    big = np.full(K, 3.0, dtype=np.float32)
    big[::2] = -3.0
    x = np.stack([wl.encode(np.zeros(K, dtype=np.float32), BF16), wl.encode(big, BF16)])
    bf = np.random.default_rng(413).standard_normal(N).astype(np.float32)
    got, want = check_against_oracle(layer, x, BF16, 0.0, 1.0, bf, what="two tokens, empty and full")
    assert list(got["nnz"]) == [0, K] and got["union_nnz"] == K
    assert np.array_equal(got["y"][0], bf)
    say("two tokens: nothing kept")
    got = gpu_sparse_fc(layer, x, BF16, 0.0, 100.0, bf)
    assert list(got["nnz"]) == [0, 0] and got["union_nnz"] == 0
    assert np.array_equal(got["y"][0], bf) and np.array_equal(got["y"][1], bf)


@pytest.mark.parametrize("B", [1, 2, 3, 4])
def test_fixed_point_hand_over_escapes(B):
    """Partial sums the fixed-point hand-over cannot carry -- 2^20 or more in magnitude, infinite, NaN -- travel as
    fp32 beside it: columns whose partial sums are all huge, columns where only some splits escape, and
    non-finite inputs, against the oracle at fp32 relative accuracy (one token: the one-token kernel; two to four: its
    two- and four-slot forms, the second token with sums that stay small); the words are back at zero afterwards (an
    ordinary call on the same workspace follows)."""
    K, N = 4096, 1544
    rng = np.random.default_rng(421)
    Wf = rng.standard_normal((K, N)).astype(np.float32)
    Wf[:, ::3] *= 1024.0     # every third column: partial sums around 2^21, most of them escape, not all
    Wf[:512, 1::3] *= 512.0  # the next ones: only splits that cover the first channels can escape
    W = wl.encode(Wf, BF16)
    layer = Layer(W, BF16, B=B)
    xs = (rng.standard_normal(K) * 300.0).astype(np.float32)
    for name, x in (("huge", xs), ("huge and non-finite", np.where(np.arange(K) == 77, np.inf, np.where(np.arange(K) == 3000, np.nan, xs)))):
        x = x.astype(np.float32)
        xb = wl.encode(np.stack([x, xs * 1e-3, xs * 0.5, -xs][:B]), BF16).reshape(B, K)
        for tau in (0.0, 150.0):
            say(f"escapes: B={B} {name} tau={tau}")
            want = oracle.sparse_fc(W, xb, 0.0, tau, None, BF16, BF16)
            got = gpu_sparse_fc(layer, xb, BF16, 0.0, tau, None)
            ref = gpu_sparse_fc(layer, xb, BF16, 0.0, tau, None, cfg=(0, 0, 0, 0, scap.CFG_PARTIAL_SUMS))
            for t in range(B):
                assert np.array_equal(got["idx"][t], want["idx"][t])
                wy, gy, ry = want["y"][t].astype(np.float64), got["y"][t].astype(np.float64), ref["y"][t].astype(np.float64)
                assert np.array_equal(np.isnan(gy), np.isnan(wy)) and np.array_equal(np.isinf(gy), np.isinf(wy))
                fin = np.isfinite(wy)
                if fin.any() and np.abs(wy[fin]).max() > 0:
                    if t == 0:
                        assert np.abs(wy[fin]).max() > 2.0 ** 22  # the case is what it claims to be
                    tol = 1e-5 * np.abs(wy[fin]) + 1e-6 * np.abs(wy[fin]).max()  # fp32 sums of terms up to 2^22
                    assert np.all(np.abs(gy[fin] - wy[fin]) <= tol), (np.abs(gy[fin] - wy[fin]) / tol).max()
                    assert np.all(np.abs(ry[fin] - wy[fin]) <= tol)
    say("an ordinary call afterwards")
    W2 = wl.weights(K, N, 422, BF16)
    layer2 = Layer(W2, BF16, B=B)
    layer2.ws = layer.ws
    check_against_oracle(layer2, wl.laplace(B, K, 423, BF16, loc=0.1, scale=0.5), BF16, 0.1, 0.3, None, what="after escapes")


def test_rerun_is_bit_identical_and_workspace_is_reusable():
    site = wl.sites(1)[0]
    W = site.make_weights()
    layer = Layer(W, site.wdt, B=1)
    X = site.test_vectors(4)
    ys = []
    for rep in range(3):
        for b in range(4):
            say(f"rerun rep={rep} vec={b}")
            ys.append(gpu_sparse_fc(layer, X[b], site.xdt, 0.1, 0.3466, None)["y"])
    for b in range(4):
        assert np.array_equal(ys[b], ys[4 + b]) and np.array_equal(ys[b], ys[8 + b])
    # a smaller layer through the same (larger) workspace
    W2 = wl.weights(320, 1032, 5, site.wdt)
    small = Layer(W2, site.wdt, B=1)
    small.ws = layer.ws
    check_against_oracle(small, wl.laplace(1, 320, 6, site.wdt)[0], site.xdt, 0.1, 0.3, None, what="shared workspace")


# ------------------------------------------------------------------ the benchmark configurations at full size
def test_config1_all_vectors():
    site = wl.sites(1)[0]
    layer = Layer(site.make_weights(), site.wdt, B=1)
    m, tau = _calib(site, 0.5)
    bf = oracle.fold_bias(layer.W_host, m, None, site.wdt)
    X = site.test_vectors(64)
    tot = 0
    for b in range(64):
        say(f"config1 vec={b}")
        got, _ = check_against_oracle(layer, X[b], site.xdt, m, tau, bf, what=f"cfg1 vec {b}")
        tot += int(got["nnz"][0])
    assert abs(1 - tot / (64 * site.K) - 0.5) < 0.02


@pytest.mark.parametrize("which", [0, 1])
def test_config2_llama_sites(which):
    site = wl.sites(2)[which]
    layer = Layer(site.make_weights(), site.wdt, B=1)
    X = site.test_vectors(3)
    calib = site.calib()
    for s in site.targets:
        m, tau = oracle.calibrate(calib, site.xdt, s, oracle.MODE_MEDIAN)
        bf = oracle.fold_bias(layer.W_host, m, None, site.wdt)
        for b in range(X.shape[0]):
            say(f"config2 {site.name} s={s} vec={b}")
            check_against_oracle(layer, X[b], site.xdt, m, tau, bf, what=f"{site.name} s={s}")


@pytest.mark.parametrize("which", [0, 1, 2, 3])
def test_config3_mistral_layers(which):
    site = wl.sites(3)[which]
    layer = Layer(site.make_weights(), site.wdt, B=1)
    m, tau = _calib(site, 0.5)
    bf = oracle.fold_bias(layer.W_host, m, None, site.wdt)
    X = site.test_vectors(2)
    for b in range(2):
        say(f"config3 {site.name} vec={b}")
        check_against_oracle(layer, X[b], site.xdt, m, tau, bf, what=site.name)


def test_headline_layer_three_sparsities_and_dense():
    site = wl.sites(4)[1]          # 14336 -> 4096, bf16
    W = site.make_weights()
    layer = Layer(W, site.wdt, B=1)
    X = site.test_vectors(2)
    calib = site.calib()
    for s in (0.5, 0.7, 0.9):
        _, tau = oracle.calibrate(calib, site.xdt, s, oracle.MODE_ZERO)
        for b in range(2):
            say(f"headline s={s} vec={b}")
            got, _ = check_against_oracle(layer, X[b], site.xdt, 0.0, tau, None, what=f"headline s={s}")
            assert abs(1 - got["nnz"][0] / site.K - s) < 0.03
    say("headline dense baseline")
    bias = np.random.default_rng(9).standard_normal(site.N).astype(np.float32)
    y = scap.dense_fc(layer.W, to_dev(X[0], site.xdt), f32_dev(bias), workspace=layer.ws)
    torch.cuda.synchronize()
    assert_y_close(y.cpu().numpy(), oracle.dense_fc(W, X[0], bias, site.wdt, site.xdt), "dense")


# ------------------------------------------------------------------ several tokens: own masks, union of rows
@pytest.mark.parametrize("path", ["auto", "vector", "matrix", "lists"])
@pytest.mark.parametrize("B", [2, 3, 4, 5, 8, 13, 16])
def test_batched_tokens_moderate(B, path):
    """auto: the library's choice; vector / matrix / lists: the batch forced onto the vector kernel, the
    single-launch matrix-core kernel, or the two-launch matrix-core form with its lists in the workspace."""
    K, N = 2500, 1032
    W = wl.weights(K, N, 501, BF16)
    layer = Layer(W, BF16, B=16)
    X = wl.swiglu(B, K, 502 + B, BF16)
    bf = np.random.default_rng(503).standard_normal(N).astype(np.float32)
    cfg = {"auto": None, "vector": (8, 0, 8 if B <= 4 else 4, 64), "matrix": (0, 0, 0, 16), "lists": (0, 0, 0, 1)}[path]
    for tau in (0.0, 0.15, 0.8, 50.0):
        say(f"batched B={B} path={path} tau={tau}")
        check_against_oracle(layer, X, BF16, 0.0, tau, bf, cfg=cfg, what=f"B={B} {path} tau={tau}")


@pytest.mark.parametrize("path", ["auto", "vector", "matrix", "lists"])
@pytest.mark.parametrize("B", [3, 8, 16])
def test_batched_tokens_huge_and_nonfinite_sums(B, path):
    """Several tokens, split K, with columns whose partial sums reach 2^21 and beyond, one token with an infinite
    and one with a NaN activation, one token whose sums stay small: against the oracle at fp32 relative accuracy,
    then an ordinary call on the same workspace."""
    K, N = 4099, 1544
    cfg = {"auto": None, "vector": (8, 0, 8 if B <= 4 else 4, 64), "matrix": (0, 0, 0, 16), "lists": (0, 0, 0, 1)}[path]
    rng = np.random.default_rng(541 + B)
    Wf = rng.standard_normal((K, N)).astype(np.float32)
    Wf[:, ::3] *= 1024.0
    Wf[:512, 1::3] *= 512.0
    Wh = wl.encode(Wf, BF16)
    huge = Layer(Wh, BF16, B=16)
    xs = (rng.standard_normal((B, K)) * 300.0).astype(np.float32)
    xs[2] *= 1e-3  # one token whose sums stay small
    xs[0, 77] = np.inf
    if B > 3:
        xs[3, 3000] = np.nan
    xb = wl.encode(xs, BF16)
    for tau in (0.0, 150.0):
        say(f"huge sums B={B} path={path} tau={tau}")
        want = oracle.sparse_fc(Wh, xb, 0.0, tau, None, BF16, BF16)
        got = gpu_sparse_fc(huge, xb, BF16, 0.0, tau, None, cfg=cfg)
        for b in range(B):
            assert np.array_equal(got["idx"][b], want["idx"][b])
            wy, gy = (v["y"][b].astype(np.float64) for v in (want, got))
            assert np.array_equal(np.isnan(gy), np.isnan(wy)) and np.array_equal(np.isinf(gy), np.isinf(wy)), f"token {b}"
            fin = np.isfinite(wy)
            if fin.any() and np.abs(wy[fin]).max() > 0:
                tol = 1e-5 * np.abs(wy[fin]) + 1e-6 * np.abs(wy[fin]).max()
                assert np.all(np.abs(gy[fin] - wy[fin]) <= tol), (b, (np.abs(gy[fin] - wy[fin]) / tol).max())
        assert np.abs(want["y"][1]).max() > 2.0 ** 22 and np.abs(want["y"][2]).max() < 2.0 ** 18  # what the case claims
    say("an ordinary call afterwards")
    layer = Layer(wl.weights(K, N, 540, BF16), BF16, B=16)
    layer.ws = huge.ws
    check_against_oracle(layer, wl.swiglu(B, K, 542 + B, BF16), BF16, 0.0, 0.2, rng.standard_normal(N).astype(np.float32), cfg=cfg, what="after huge sums")


@pytest.mark.parametrize("wdt", [F16, BF16, I8])
@pytest.mark.parametrize("B", [2, 3, 4])
def test_batched_tokens_half_width_tiles(B, wdt):
    """2-4 tokens on the vector kernel with half-width column tiles: forced, and as the default for a short
    input into a narrow layer (few full-width tiles)."""
    K, N = 1100, 2064 if wdt != I8 else 2080
    if wdt == I8:
        W, scale = wl.quantize_i8(K, N, 531)
    else:
        W, scale = wl.weights(K, N, 531, wdt), None
    xdt = BF16 if wdt == I8 else wdt
    layer = Layer(W, wdt, col_scale_bits=scale, B=4)
    X = wl.laplace(B, K, 532 + B, xdt, loc=0.1, scale=0.7)
    bf = np.random.default_rng(533).standard_normal(N).astype(np.float32)
    for cfg in ((8, 0, 8, 32), (8, 192, 8, 32), None):
        for m, tau in ((0.1, 0.0), (0.1, 0.6), (0.0, 2.5)):
            say(f"half-width tiles B={B} wdt={wdt} cfg={cfg} tau={tau}")
            check_against_oracle(layer, X, xdt, m, tau, bf, cfg=cfg, what=f"half-width B={B} wdt={wdt} cfg={cfg} tau={tau}")


@pytest.mark.parametrize("lanes", [16, 1])
def test_batched_matrix_core_edge_cases(lanes):
    """Ragged list lengths (not multiples of the 16-row MFMA block), infinities, one split and many splits."""
    K, N = 1000, 264
    W = wl.weights(K, N, 511, BF16)
    layer = Layer(W, BF16, B=16)
    X = wl.swiglu(6, K, 512, BF16)
    Xf = wl.decode(X, BF16)
    Xf[2, 17] = np.inf
    Xf[4, 900] = -np.inf
    Xf[1, 3] = np.nan
    X = wl.encode(Xf, BF16)
    for rows in (0, 64, 128, 832):
        for tau in (0.0, 0.3, 1.5, 2.5):
            say(f"matrix-core edge rows={rows} tau={tau}")
            check_against_oracle(layer, X, BF16, 0.01, tau, None, cfg=(0, rows, 0, lanes),
                                 what=f"mfma lanes={lanes} rows={rows} tau={tau}")


STAGED = [
    # K (multiple of 8: the staged-tile kernel), N, tokens, weight dtype, activation dtype
    (8, 128, 5, BF16, BF16), (16, 136, 16, BF16, BF16), (56, 264, 7, BF16, F16), (64, 128, 16, I8, BF16),
    (72, 272, 9, I8, F16), (120, 520, 5, BF16, BF16), (512, 1032, 16, BF16, F16), (2048, 264, 11, I8, BF16),
    (2568, 136, 16, BF16, BF16), (4104, 528, 6, I8, BF16), (6000, 128, 13, BF16, BF16),
    (8, 128, 5, F16, F16), (72, 272, 16, F16, BF16), (1000, 520, 7, F16, F16), (4104, 136, 16, F16, F16),
]


@pytest.mark.parametrize("K,N,B,wdt,xdt", STAGED)
def test_staged_tile_kernel_shapes(K, N, B, wdt, xdt):
    """More than 4 tokens with K a multiple of 8 run on the kernel that stages the raw input tile: shortest inputs,
    one chunk and many, ragged last split, both activation types with both weight types, centring on and off, from
    everything kept to almost nothing kept; and the dense call on the same kernel."""
    if wdt == I8:
        N = (N + 15) // 16 * 16
        W, scale = wl.quantize_i8(K, N, 7000 + K)
    else:
        W, scale = wl.weights(K, N, 7000 + K, wdt), None
    layer = Layer(W, wdt, col_scale_bits=scale, B=16)
    X = wl.laplace(B, K, 7100 + K, xdt, loc=0.1, scale=0.8)
    bias = np.random.default_rng(7200 + K).standard_normal(N).astype(np.float32)
    for m, tau, bf in ((0.0, 0.0, None), (0.13, 0.5, bias), (-0.4, 3.0, None), (0.0, 50.0, bias)):
        say(f"staged tile K={K} N={N} B={B} wdt={wdt} xdt={xdt} m={m} tau={tau}")
        check_against_oracle(layer, X, xdt, m, tau, bf, what=f"staged K={K} B={B} m={m} tau={tau}")
    y = scap.dense_fc(layer.W, to_dev(X, xdt), f32_dev(bias), col_scale=layer.scale, workspace=layer.ws)
    torch.cuda.synchronize()
    assert_y_close(y.cpu().numpy(), oracle.dense_fc(W, X, bias, wdt, xdt, col_scale=scale), "staged dense")


@pytest.mark.parametrize("wdt", [BF16, F16])
def test_staged_tile_kernel_lists_a_superset_of_the_union(wdt):
    """A wavefront whose first 64-channel chunk is kept entirely lists its other chunks without testing them.
    Here every fourth chunk holds large values and the three after it values that every token drops, with 1792
    channels per workgroup (4 chunks per wavefront): the lists are four times the union, and y, the per-token
    lists and the size of the union (column tile 0 counts it exactly when it is asked for) must not change."""
    K, N, B = 7168, 392, 16
    W = wl.weights(K, N, 541, wdt)
    layer = Layer(W, wdt, B=16)
    rng = np.random.default_rng(542)
    big = rng.choice([-1.0, 1.0], size=(B, K)) * rng.uniform(1.0, 2.0, size=(B, K))
    small = rng.uniform(-0.05, 0.05, size=(B, K))
    chunk = (np.arange(K) // 64) % 4
    Xf = np.where(chunk[None, :] == 0, big, small)
    Xf[3, 64 * 4 * 5 + 7] = 0.01     # one token drops a channel of a "large" chunk; the others keep it
    Xf[:, 64 * 4 * 9 + 11] = 0.02    # a channel of a "large" chunk dropped by every token (still at most 2 of 64)
    Xf[5, 64 * 13 + 3] = 1.5         # one token keeps a channel inside a "small" chunk
    X = wl.encode(Xf, wdt)
    bias = rng.standard_normal(N).astype(np.float32)
    for cfg in ((0, 1792, 0, 16), None):
        say(f"superset lists wdt={wdt} cfg={cfg}")
        got, want = check_against_oracle(layer, X, wdt, 0.0, 0.5, bias, cfg=cfg, what=f"superset cfg={cfg}")
        assert want["union_nnz"] == (K // 256) * 64 - 1 + 1
        # the rows that are read, and so the order of every sum, must not depend on which outputs were asked for
        plain = torch.full((B, N), float("nan"), dtype=torch.float32, device="cuda")
        scap.sparse_fc(layer.W, to_dev(X, wdt), 0.0, 0.5, f32_dev(bias), y=plain, workspace=layer.ws, cfg=cfg)
        torch.cuda.synchronize()
        assert np.array_equal(plain.cpu().numpy().view(np.uint32), got["y"].view(np.uint32)), "y depends on the outputs requested"


@pytest.mark.parametrize("B", [4, 16])
def test_batched_tokens_fp16_weights(B):
    K, N = 1500, 1032
    W = wl.weights(K, N, 521, F16)
    layer = Layer(W, F16, B=16)
    X = wl.laplace(B, K, 522, F16)
    for tau in (0.0, 0.4):
        say(f"batched fp16 B={B} tau={tau}")
        check_against_oracle(layer, X, F16, 0.1, tau, None, what=f"fp16 B={B} tau={tau}")


@pytest.mark.parametrize("which,B", [(0, 4), (0, 16), (1, 4), (1, 16)])
def test_config4_batched_full_size(which, B):
    """Both layers of the batched configuration at full size, 4 tokens (vector kernel / 16-slot staged tile) and 16
    tokens (staged-tile kernel: 112 narrow column tiles on 4096 -> 14336), at the three per-token targets."""
    site = wl.sites(4)[which]
    layer = Layer(site.make_weights(), site.wdt, B=16)
    calib = site.calib()
    X = site.draw(B, site.seed_test + 77)
    for s in (0.5, 0.7, 0.9):
        _, tau = oracle.calibrate(calib, site.xdt, s, oracle.MODE_ZERO)
        say(f"config4 {site.name} B={B} s={s}")
        got, want = check_against_oracle(layer, X, site.xdt, 0.0, tau, None, what=f"{site.name} B={B} s={s}")
        if site.kind == "swiglu":
            dens = want["union_nnz"] / site.K
            assert abs(dens - (1 - s ** B)) < 0.02


# ------------------------------------------------------------------ int8 weights with column scales
@pytest.mark.parametrize("K,N,B", [(700, 2064, 1), (4096, 1024, 1), (1500, 3088, 4)])
def test_int8_weights(K, N, B):
    q, scale = wl.quantize_i8(K, N, 601)
    layer = Layer(q, I8, col_scale_bits=scale, B=16)
    X = wl.swiglu(B, K, 602, BF16)
    for tau in (0.0, 0.3):
        say(f"int8 K={K} N={N} B={B} tau={tau}")
        check_against_oracle(layer, X, BF16, 0.0, tau, None, what=f"int8 {K}x{N}")
    bf_want = oracle.fold_bias(q, 0.25, None, I8, col_scale=scale)
    bf = scap.fold_bias(layer.W, 0.25, None, col_scale=layer.scale, workspace=layer.ws)
    torch.cuda.synchronize()
    assert np.allclose(bf.cpu().numpy(), bf_want, rtol=1e-5, atol=1e-5)


@pytest.mark.parametrize("path", ["auto", "vector", "matrix", "lists"])
@pytest.mark.parametrize("B", [2, 5, 8, 13, 16])
def test_int8_batched_tokens(B, path):
    """int8 weights with several tokens: the matrix-core kernel widens int8 to bf16 exactly (auto from 5 tokens)."""
    K, N = 2500, 1040          # 5 ragged 256-column tiles on the matrix cores, 2 tiles of 1024 on the vector kernel
    q, scale = wl.quantize_i8(K, N, 611)
    layer = Layer(q, I8, col_scale_bits=scale, B=16)
    X = wl.swiglu(B, K, 612 + B, BF16)
    bf = np.random.default_rng(613).standard_normal(N).astype(np.float32)
    cfg = {"auto": None, "vector": (8, 0, 8 if B <= 4 else 4, 64), "matrix": (0, 0, 0, 16), "lists": (0, 0, 0, 1)}[path]
    for tau in (0.0, 0.15, 0.8, 50.0):
        say(f"int8 batched B={B} path={path} tau={tau}")
        check_against_oracle(layer, X, BF16, 0.0, tau, bf, cfg=cfg, what=f"int8 B={B} {path} tau={tau}")
    # extreme codes: every weight -128 or 127
    q2 = np.where(np.random.default_rng(614).random((K, N)) < 0.5, -128, 127).astype(np.int8)
    layer2 = Layer(q2, I8, col_scale_bits=scale, B=16)
    check_against_oracle(layer2, X, BF16, 0.0, 0.3, None, cfg=cfg, what=f"int8 extremes B={B} {path}")


def test_config5_expert_down_projection():
    site = wl.sites(5)[1]          # expert 0, down 14336 -> 4096, int8
    q, scale = wl.quantize_i8(site.K, site.N, site.seed_w)
    layer = Layer(q, I8, col_scale_bits=scale, B=16)
    calib = wl.swiglu(128, site.K, site.seed_calib, BF16)
    m, tau = oracle.calibrate(calib, BF16, 0.7, oracle.MODE_MEDIAN)
    bf = oracle.fold_bias(q, m, None, I8, col_scale=scale)
    for B in (1, 8):
        X = wl.swiglu(B, site.K, site.seed_test + B, BF16)
        say(f"config5 expert down B={B}")
        check_against_oracle(layer, X, BF16, m, tau, bf, what=f"cfg5 B={B}")


# ------------------------------------------------------------------ fold_bias, dense, calibrate
@pytest.mark.parametrize("dt,K,N", [(F16, 1024, 4096), (BF16, 11008, 4096), (BF16, 333, 1544)])
def test_fold_bias(dt, K, N):
    W = wl.weights(K, N, 701, dt)
    layer = Layer(W, dt, B=1)
    bias = np.random.default_rng(702).standard_normal(N).astype(np.float32)
    for m, b in ((0.1, bias), (-3.7, None)):
        say(f"fold_bias dt={dt} K={K} N={N} m={m}")
        got = scap.fold_bias(layer.W, m, f32_dev(b), workspace=layer.ws)
        torch.cuda.synchronize()
        want = oracle.fold_bias(W, m, b, dt)
        assert np.abs(got.cpu().numpy() - want).max() <= 2e-5 * max(1.0, abs(m) * math.sqrt(K) * 0.02 * 50)


@pytest.mark.parametrize("dt,K,N,B", [(F16, 1024, 4096, 1), (BF16, 4096, 6144, 1), (BF16, 999, 1032, 5)])
def test_dense_fc(dt, K, N, B):
    W = wl.weights(K, N, 801, dt)
    layer = Layer(W, dt, B=16)
    X = wl.prenorm(B, K, 802, dt, chan_seed=803)
    bias = np.random.default_rng(804).standard_normal(N).astype(np.float32)
    say(f"dense dt={dt} K={K} N={N} B={B}")
    y = scap.dense_fc(layer.W, to_dev(X, dt), f32_dev(bias), workspace=layer.ws)
    torch.cuda.synchronize()
    assert_y_close(y.cpu().numpy(), oracle.dense_fc(W, X, bias, dt, dt), "dense")


@pytest.mark.parametrize("cfg,which", [(1, 0), (2, 0), (2, 1)])
def test_calibrate_matches_oracle_bit_for_bit(cfg, which):
    site = wl.sites(cfg)[which]
    X = site.calib()
    Xd = to_dev(X, site.xdt)
    ws = scap.Workspace(site.K, 0, X.shape[0])
    for est in ("zero", "median", "hist", "mean"):
        for s in (0.0, 0.5, 0.7, 0.9):
            say(f"calibrate {site.name} est={est} s={s}")
            m_g, t_g = scap.calibrate(Xd, s, oracle.EST[est], workspace=ws)
            m_o, t_o = oracle.calibrate(X, site.xdt, s, oracle.EST[est])
            if est == "mean":
                assert abs(m_g - m_o) <= abs(m_o) * 2 ** -22 + 1e-9
                assert abs(t_g - t_o) <= 1e-5
            else:
                assert m_g == m_o, f"{est}: m {m_g} vs {m_o}"
                assert t_g == t_o, f"{est}: tau {t_g} vs {t_o}"


def test_calibrate_odd_count_and_small_sample():
    X = wl.laplace(3, 333, 901, F16, loc=-0.4, scale=0.2)
    Xd = to_dev(X, F16)
    ws = scap.Workspace(333, 0, 3)
    for est in ("median", "zero"):
        for s in (0.001, 0.25, 0.999):
            say(f"calibrate odd est={est} s={s}")
            assert scap.calibrate(Xd, s, oracle.EST[est], workspace=ws) == oracle.calibrate(X, F16, s, oracle.EST[est])


def test_calibrate_paper_sized_sample():
    """The paper calibrates on 64 slices of 256 tokens = 16384 tokens per layer (Section 4): 67 million pooled
    values for a 4096-wide input.  Median and threshold must still equal the oracle's sort bit for bit."""
    n, K = 16384, 4096
    X = wl.prenorm(n, K, 951, BF16, 952)
    Xd = to_dev(X, BF16)
    ws = scap.Workspace(K, 0, n)
    say("calibrate 16384 x 4096 median s=0.5")
    got = scap.calibrate(Xd, 0.5, scap.MODE_MEDIAN, workspace=ws)
    want = oracle.calibrate(X, BF16, 0.5, oracle.MODE_MEDIAN)
    assert got == want, f"{got} vs {want}"
    # a second target on the same sample, uncentred, checked against numpy's order statistic
    say("calibrate 16384 x 4096 zero s=0.9")
    _, tau = scap.calibrate(Xd, 0.9, scap.MODE_ZERO, workspace=ws)
    v = np.abs(wl.decode(X, BF16).astype(np.float32)).ravel()
    k = int(np.ceil(np.float64(np.float32(0.9)) * v.size))
    assert tau == float(np.partition(v, k - 1)[k - 1])


def test_calibrate_paper_sized_sample_of_the_widest_input():
    """16384 tokens of the 14336-wide down-projection input: 235 million pooled values.  Sorting that many on the
    host takes minutes, so the order statistics are checked against numpy's selection (the routine the oracle's
    sort is pinned to) on the same fp32 values: the threshold uncentred and centred on the median."""
    n, K = 16384, 14336
    rng = np.random.default_rng(953)
    X = np.empty((n, K), dtype=np.uint16)
    for r0 in range(0, n, 2048):   # SiLU(g) * u drawn in slabs to bound host memory
        g = rng.standard_normal((2048, K), dtype=np.float32)
        u = rng.standard_normal((2048, K), dtype=np.float32)
        X[r0:r0 + 2048] = wl.encode(g / (1 + np.exp(-g)) * u + np.float32(0.05), BF16)
    Xd = to_dev(X, BF16)
    ws = scap.Workspace(K, 0, n)
    v = wl.decode(X, BF16).astype(np.float32).ravel()
    del X
    M = v.size
    say("calibrate 16384 x 14336 median s=0.7")
    m, tau = scap.calibrate(Xd, 0.7, scap.MODE_MEDIAN, workspace=ws)
    mid = np.partition(v, [M // 2 - 1, M // 2])[[M // 2 - 1, M // 2]]
    assert m == float(np.float32((np.float64(mid[0]) + np.float64(mid[1])) / 2))
    k = int(np.ceil(np.float64(np.float32(0.7)) * M))
    imp = np.abs(v - np.float32(m))     # one fp32 subtraction, as the pruner forms it
    assert tau == float(np.partition(imp, k - 1)[k - 1])
    say("calibrate 16384 x 14336 zero s=0.5")
    _, tau0 = scap.calibrate(Xd, 0.5, scap.MODE_ZERO, workspace=ws)
    k = int(np.ceil(np.float64(np.float32(0.5)) * M))
    np.abs(v, out=imp)
    assert tau0 == float(np.partition(imp, k - 1)[k - 1])


def test_calibrate_histogram_mode_on_hand_built_samples():
    """The histogram estimator against values worked out by hand from its definition (the samples and their
    derivations are in test_oracle_hist_pins.py): peaks that separate the definition from its near misses, a
    value equal to the upper end of the range, a window cut at the lower edge with a three-way tie."""
    import test_oracle_hist_pins as hp
    from fractions import Fraction
    cases = [(hp._case1(), 100.5 / 64),
             (hp._grid_sample({}, Fraction(0), hi_copies=60), 2045.5 / 64),
             (hp._grid_sample({}, Fraction(0), hi_copies=6, lo_copies=40, empty=range(1, 7)), 0.5 / 64)]
    for X, want in cases:
        ws = scap.Workspace(X.shape[1], 0, 1)
        say(f"calibrate hist hand-built M={X.size} want={want}")
        m, tau = scap.calibrate(to_dev(X, F16), 0.5, scap.MODE_HIST, workspace=ws)
        assert m == want
        assert (m, tau) == oracle.calibrate(X, F16, 0.5, oracle.MODE_HIST)
    Xc = np.full((3, 50), 2.5, dtype=np.float16).view(np.uint16)
    assert scap.calibrate(to_dev(Xc, F16), 0.3, scap.MODE_HIST, workspace=scap.Workspace(50, 0, 3)) == (2.5, 0.0)


@pytest.mark.parametrize("dt", [F16, BF16])
def test_calibrate_every_code_pattern(dt):
    """Every 16-bit code at least once (subnormals, both zeros, infinities, NaNs) plus a random bulk, a count
    that is not a multiple of the 8-code load; order statistics must still equal the oracle's sort."""
    rng = np.random.default_rng(961 + dt)
    bulk = wl.laplace(1, 50001, 962, dt, loc=0.3, scale=0.4)[0]
    X = np.concatenate([np.arange(65536, dtype=np.uint16), bulk, rng.integers(0, 65536, 4099).astype(np.uint16)])
    rng.shuffle(X)
    X = X.reshape(1, -1)
    Xd = to_dev(X, dt)
    ws = scap.Workspace(X.shape[1], 0, 1)
    for est in ("zero", "median", "hist"):
        for s in (0.01, 0.3, 0.5, 0.9):
            say(f"calibrate all codes dt={dt} est={est} s={s}")
            got = scap.calibrate(Xd, s, oracle.EST[est], workspace=ws)
            want = oracle.calibrate(X, dt, s, oracle.EST[est])
            assert got == want, f"{est} s={s}: {got} vs {want}"


def test_hip_graph_replays_match_eager_launches():
    """bench.py times launches replayed from a HIP graph: every replay must give what the eager launch gives.
    One-token kernel (also in its y += result mode), the two-token kernel, both matrix-core forms (single launch, union
    kernel + product kernel), the one-token and the 8-token SwiGLU block, replayed several times with eager work and synchronisation in between, on inputs that change
    between replays."""
    K, F, N = 1500, 2056, 1032
    W = to_dev(wl.weights(K, N, 971, BF16), BF16)
    Wg, Wu, Wd = (to_dev(wl.weights(K, F, 972, BF16), BF16), to_dev(wl.weights(K, F, 973, BF16), BF16),
                  to_dev(wl.weights(F, N, 974, BF16), BF16))
    W_gu = scap.pack_gate_up(Wg, Wu)
    ws = scap.Workspace(K, N, 8, F=F)
    X = to_dev(wl.laplace(8, K, 975, BF16, loc=0.0, scale=1.0), BF16)
    x1 = X[0].clone()
    xb = X.clone()
    y1 = torch.zeros((1, N), dtype=torch.float32, device="cuda")
    y8 = torch.zeros((8, N), dtype=torch.float32, device="cuda")
    y8l = torch.zeros((8, N), dtype=torch.float32, device="cuda")
    yb = torch.zeros((1, N), dtype=torch.float32, device="cuda")
    yb8 = torch.zeros((8, N), dtype=torch.float32, device="cuda")
    nnz = torch.zeros(8, dtype=torch.int32, device="cuda")
    two_launch = scap.LaunchCfg(0, 0, 0, 1)
    K2 = 1504  # a multiple of 8: two tokens run on the two-token kernel
    W2 = to_dev(wl.weights(K2, N, 976, BF16), BF16)
    ws2 = scap.Workspace(K2, N, 2)
    x2 = to_dev(wl.laplace(2, K2, 977, BF16, loc=0.0, scale=1.0), BF16)
    y2 = torch.zeros((2, N), dtype=torch.float32, device="cuda")
    nnz2 = torch.zeros(2, dtype=torch.int32, device="cuda")
    ya = torch.zeros((1, N), dtype=torch.float32, device="cuda")

    def work():
        scap.sparse_fc(W, x1, 0.0, 0.5, None, y=y1, workspace=ws)
        scap.sparse_fc(W2, x2, 0.0, 0.5, None, y=y2, nnz_out=nnz2, workspace=ws2)     # 2 tokens
        ya.fill_(1.0)
        scap.sparse_fc(W, x1, 0.0, 0.5, None, y=ya, workspace=ws, cfg=(0, 0, 0, 0, scap.CFG_ACCUMULATE))
        scap.sparse_fc(W, xb, 0.0, 0.5, None, y=y8, nnz_out=nnz, workspace=ws)        # 8 tokens: matrix cores
        scap.sparse_fc(W, xb, 0.0, 0.5, None, y=y8l, workspace=ws, cfg=two_launch)
        scap.swiglu_block(W_gu, Wd, x1, 0.0, 0.5, None, 0.0, 0.02, None, y=yb, workspace=ws)
        scap.swiglu_block(W_gu, Wd, xb, 0.0, 0.5, None, 0.0, 0.02, None, y=yb8, workspace=ws)

    work()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        work()
    for rep in range(4):
        say(f"graph replay {rep}")
        x1.copy_(X[(rep + 1) % 8])
        xb.copy_(torch.roll(X, rep + 1, dims=0))
        x2.copy_(torch.roll(x2, 1, dims=1))
        work()
        torch.cuda.synchronize()
        outs = (y1, y8, y8l, yb, yb8, nnz, y2, nnz2)
        want = tuple(t.clone() for t in outs)
        want_a = ya.clone()
        assert float((ya - 1.0 - y1).abs().max()) < 1e-4, "y += result differs from 1 + (y = result)"
        assert torch.equal(y8, y8l) or float((y8 - y8l).abs().max()) < 1e-4
        for t in outs:
            t.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(want, outs):
            assert torch.equal(a, b), f"replay {rep} differs from the eager launch"
        assert float((ya - want_a).abs().max()) < 1e-4  # atomic adds: the order of the additions is not fixed


@pytest.mark.parametrize("K,N,B", [(1 << 20, 8, 1), (1 << 20, 16, 3), (64, 1 << 19, 1), (72, 1 << 19, 16), (1 << 20, 136, 8)])
def test_maximum_sizes(K, N, B):
    """The largest layer dimensions the library accepts: 2^20 input channels, 2^19 output columns (the 16-token case
    has more 128-column tiles than the matrix-core path has counters and falls back to the vector kernel)."""
    W = wl.weights(K, N, 981, BF16)
    layer = Layer(W, BF16, B=16)
    X = wl.swiglu(B, K, 982, BF16)
    bf = np.random.default_rng(983).standard_normal(N).astype(np.float32)
    for tau in (0.0, 0.3):
        say(f"maximum sizes K={K} N={N} B={B} tau={tau}")
        check_against_oracle(layer, X, BF16, 0.0, tau, bf, what=f"max K={K} N={N} B={B} tau={tau}")
    assert scap.workspace_bytes((1 << 20) + 64, 8, 1) == 0 and scap.workspace_bytes(64, (1 << 19) + 8, 1) == 0


def test_two_streams_with_their_own_workspaces():
    """Calls that overlap in time are allowed when each stream has its own workspace: results equal the
    one-after-the-other results bit for bit."""
    K, N = 4096, 4096
    W = to_dev(wl.weights(K, N, 991, BF16), BF16)
    X = to_dev(wl.swiglu(32, K, 992, BF16), BF16)
    ws = [scap.Workspace(K, N, 8), scap.Workspace(K, N, 8)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    ref1 = [scap.sparse_fc(W, X[i], 0.0, 0.2, None, workspace=ws[0]).clone() for i in range(16)]
    ref8 = [scap.sparse_fc(W, X[i:i + 8], 0.0, 0.2, None, workspace=ws[0]).clone() for i in range(16)]
    torch.cuda.synchronize()
    out1 = [torch.empty((1, N), dtype=torch.float32, device="cuda") for _ in range(16)]
    out8 = [torch.empty((8, N), dtype=torch.float32, device="cuda") for _ in range(16)]
    for rep in range(3):
        say(f"two streams rep {rep}")
        for i in range(16):
            with torch.cuda.stream(streams[0]):
                scap.sparse_fc(W, X[i], 0.0, 0.2, None, y=out1[i], workspace=ws[0], stream=streams[0])
            with torch.cuda.stream(streams[1]):
                scap.sparse_fc(W, X[i:i + 8], 0.0, 0.2, None, y=out8[i], workspace=ws[1], stream=streams[1])
        torch.cuda.synchronize()
        for i in range(16):
            assert torch.equal(out1[i], ref1[i]) and torch.equal(out8[i], ref8[i]), f"rep {rep} call {i}"


def test_random_shapes_and_thresholds():
    """Seeded sweep over odd shapes: K from 1 to ~6000, N any multiple of the vector width up to ~7000, 1-16 tokens,
    every weight dtype, thresholds from 'keep all' to 'keep almost nothing', with and without bias and centring."""
    rng = np.random.default_rng(20241207)
    for case in range(90):
        wdt = (F16, BF16, I8)[case % 3]
        xdt = BF16 if wdt == I8 else wdt
        vec = 16 if wdt == I8 else 8
        K = int(rng.choice([1, 7, 63, 64, 65, 129, 500, 1023, 2049, 4097, 6001])) if case % 4 == 0 else int(rng.integers(1, 6000))
        N = vec * int(rng.integers(1, 7000 // vec))
        B = int(rng.choice([1, 1, 1, 2, 3, 4, 5, 7, 8, 11, 16]))
        m = float(rng.choice([0.0, 0.13, -0.4]))
        if wdt == I8:
            W, scale = wl.quantize_i8(K, N, 3000 + case)
        else:
            W, scale = wl.weights(K, N, 3000 + case, wdt), None
        layer = Layer(W, wdt, col_scale_bits=scale, B=16)
        X = wl.laplace(B, K, 4000 + case, xdt, loc=m, scale=0.7)
        d = np.abs(wl.decode(X, xdt).astype(np.float32) - np.float32(m))
        tau = float(np.quantile(d, rng.choice([0.0, 0.3, 0.5, 0.8, 0.97, 1.0])))
        bf = rng.standard_normal(N).astype(np.float32) if case % 2 else None
        say(f"random case {case}: wdt={wdt} K={K} N={N} B={B} m={m} tau={tau:.4g}")
        check_against_oracle(layer, X, xdt, m, tau, bf, what=f"random case {case} K={K} N={N} B={B}")
