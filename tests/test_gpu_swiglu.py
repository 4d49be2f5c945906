"""GPU parity of the fused SwiGLU block (Appendix B Alg. 2): scap_pack_gate_up and scap_swiglu_block through the
C ABI against the CPU oracle on the same seeded inputs.

The second pruner decides on a floating-point value (the gated product z) that the two sides sum in different
orders (and, on the matrix cores, with the centred inputs carried as bf16 head + tail), so a channel whose
|z - m_z| lies within a rounding-sized band of tau_z may legitimately fall either way: 1e-4 * max(1, |z|) on the
vector kernel (up to 4 tokens; int8 weights up to 2), 3e-4 * max(1, |z|) on the matrix cores, with z itself within
2e-5 * (1 + |z|) resp. 1e-4 * (1 + |z|) of the oracle's.
The tests require: every channel outside the band decided exactly as the oracle decides it; the kept list
ascending, duplicate-free and consistent with its count; z within rounding of the oracle's; and y within the
usual bar of the oracle's y for the decisions actually taken (the oracle's y plus/minus the band channels'
rows, evaluated here in fp64 from the oracle's own z)."""
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
    from gpu_util import assert_y_close, f32_dev, to_dev


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def pack_host(g, u):
    """The interleaving in groups of 4 columns, written with array reshapes."""
    g2, u2 = np.atleast_2d(g), np.atleast_2d(u)
    r, F = g2.shape
    out = np.stack([g2.reshape(r, F // 4, 4), u2.reshape(r, F // 4, 4)], axis=2).reshape(r, 2 * F)
    return out if np.ndim(g) == 2 else out[0]


def weights_of(dt, K, N, seed, std):
    if dt == I8:
        return wl.quantize_i8(K, N, seed, std=std)
    return wl.weights(K, N, seed, dt, std=std), None


def B_MATRIX(dt, B):
    """Does a fused block of B tokens over weights of type dt run on the matrix cores?"""
    return B >= (3 if dt == I8 else 5)


class Block:
    def __init__(self, K, F, N, dt, seed, std=0.05, B=1):
        self.K, self.F, self.N, self.dt = K, F, N, dt
        (self.Wg, self.sg), (self.Wu, self.su) = weights_of(dt, K, F, seed, std), weights_of(dt, K, F, seed + 1, std)
        self.Wd, self.sd = weights_of(dt, F, N, seed + 2, std)
        self.W_gu = scap.pack_gate_up(to_dev(self.Wg, dt), to_dev(self.Wu, dt))
        self.gu_scale = None if dt != I8 else scap.pack_gate_up(to_dev(self.sg, F16), to_dev(self.su, F16))
        self.W_down = to_dev(self.Wd, dt)
        self.down_scale = None if dt != I8 else to_dev(self.sd, F16)
        self.ws = scap.Workspace(K, N, B, F=F)
        torch.cuda.synchronize()
        assert np.array_equal(self.W_gu.cpu().view(torch.int8 if dt == I8 else torch.int16).numpy()
                              .view(np.int8 if dt == I8 else np.uint16), pack_host(self.Wg, self.Wu))

    def down_rows(self, rows):
        w = self.Wd[rows].astype(np.float64) if self.dt == I8 else wl.decode(self.Wd[rows], self.dt).astype(np.float64)
        if self.dt == I8:
            w = w * wl.decode(self.sd, F16).astype(np.float64)[None, :]
        return w

    def run(self, x_bits, xdt, m_x, tau_x, bg, bu, m_z, tau_z, bd, want_lists=True, want_z=True, addend=None, cfg=None):
        b_gu = None if bg is None else scap.pack_gate_up(f32_dev(bg), f32_dev(bu))
        z = torch.full((self.F,), float("nan"), dtype=torch.float32, device="cuda") if want_z else None
        idx = torch.full((self.F,), -7, dtype=torch.int32, device="cuda") if want_lists else None
        nnz = torch.full((1,), -7, dtype=torch.int32, device="cuda") if want_lists else None
        # addend given: the residual form, y starts as the addend and the block's output is added to it
        y = (torch.full((1, self.N), float("nan"), dtype=torch.float32, device="cuda") if addend is None
             else f32_dev(addend).reshape(1, self.N).clone())
        scap.swiglu_block(self.W_gu, self.W_down, to_dev(x_bits, xdt), m_x, tau_x, b_gu, m_z, tau_z, f32_dev(bd),
                          gu_scale=self.gu_scale, down_scale=self.down_scale, y=y, z_out=z, idx_z_out=idx,
                          nnz_z_out=nnz, workspace=self.ws, residual=addend is not None, cfg=cfg)
        torch.cuda.synchronize()
        out = {"y": y.cpu().numpy()[0]}
        if want_z:
            out["z"] = z.cpu().numpy()
        if want_lists:
            n = int(nnz.item())
            assert 0 <= n <= self.F
            out["idx_z"] = idx.cpu().numpy()[:n].copy()
        return out

    def run_batch(self, X_bits, xdt, m_x, tau_x, bg, bu, m_z, tau_z, bd, cfg=None):
        B = X_bits.shape[0]
        b_gu = None if bg is None else scap.pack_gate_up(f32_dev(bg), f32_dev(bu))
        z = torch.full((B, self.F), float("nan"), dtype=torch.float32, device="cuda")
        idx = torch.full((B, self.F), -7, dtype=torch.int32, device="cuda")
        nnz = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        y = torch.full((B, self.N), float("nan"), dtype=torch.float32, device="cuda")
        scap.swiglu_block(self.W_gu, self.W_down, to_dev(X_bits, xdt), m_x, tau_x, b_gu, m_z, tau_z, f32_dev(bd),
                          gu_scale=self.gu_scale, down_scale=self.down_scale, y=y, z_out=z, idx_z_out=idx,
                          nnz_z_out=nnz, workspace=self.ws, cfg=cfg)
        torch.cuda.synchronize()
        nn, ih, zh, yh = nnz.cpu().numpy(), idx.cpu().numpy(), z.cpu().numpy(), y.cpu().numpy()
        assert np.all((nn >= 0) & (nn <= self.F))
        return [{"y": yh[b], "z": zh[b], "idx_z": ih[b, :nn[b]].copy()} for b in range(B)]

    def check_batch(self, X_bits, xdt, m_x, tau_x, bg, bu, m_z, tau_z, bd, what, cfg=None):
        """Each token of a batch against the oracle's one-token block (tokens are independent: own masks)."""
        gots = self.run_batch(X_bits, xdt, m_x, tau_x, bg, bu, m_z, tau_z, bd, cfg=cfg)
        for b, got in enumerate(gots):
            want = oracle.swiglu_block(self.Wg, self.Wu, self.Wd, X_bits[b], m_x, tau_x, m_z, tau_z, self.dt, xdt,
                                       b_gate=bg, b_up=bu, b_down=bd, gate_scale=self.sg, up_scale=self.su,
                                       down_scale=self.sd, nthreads=8)
            # from 5 tokens (int8 weights: from 3) both launches run on the matrix cores
            self.compare(got, want, m_z, tau_z, f"{what} token {b}", matrix_cores=B_MATRIX(self.dt, len(gots)))
        return gots

    def check(self, x_bits, xdt, m_x, tau_x, bg, bu, m_z, tau_z, bd, what, addend=None, cfg=None):
        want = oracle.swiglu_block(self.Wg, self.Wu, self.Wd, x_bits, m_x, tau_x, m_z, tau_z, self.dt, xdt,
                                   b_gate=bg, b_up=bu, b_down=bd, gate_scale=self.sg, up_scale=self.su,
                                   down_scale=self.sd, nthreads=8)
        got = self.run(x_bits, xdt, m_x, tau_x, bg, bu, m_z, tau_z, bd, addend=addend, cfg=cfg)
        return got, want, self.compare(got, want, m_z, tau_z, what, addend=addend)

    def compare(self, got, want, m_z, tau_z, what, matrix_cores=False, addend=None):
        zo = want["z"].astype(np.float64)
        fin = np.isfinite(zo)
        # vector kernel (up to 4 tokens): fp32 sums in another order than the oracle's fp64 ones;
        # matrix cores: in addition the centred inputs are carried as bf16 head + tail, 2^-17 relative per product
        z_tol, band_tol = (1e-4, 3e-4) if matrix_cores else (2e-5, 1e-4)
        tol = z_tol + z_tol * np.abs(zo[fin])
        assert np.all(np.abs(got["z"][fin] - zo[fin]) <= tol), f"{what}: z off by {np.abs(got['z'][fin] - zo[fin]).max()}"
        # decisions: exact outside the band
        d = (want["z"] - np.float32(m_z)).astype(np.float32)
        margin = np.abs(np.abs(d.astype(np.float64)) - float(np.float32(tau_z)))
        band = margin <= band_tol * np.maximum(1.0, np.abs(zo))
        gi = got["idx_z"]
        assert np.all(np.diff(gi) > 0), f"{what}: kept list not strictly ascending"
        assert gi.size == 0 or (gi[0] >= 0 and gi[-1] < self.F)
        g_mask = np.zeros(self.F, dtype=bool)
        g_mask[gi] = True
        o_mask = np.zeros(self.F, dtype=bool)
        o_mask[want["idx_z"]] = True
        diff = g_mask != o_mask
        assert not np.any(diff & ~band), f"{what}: {np.count_nonzero(diff & ~band)} decisions differ outside the band"
        # y for the decisions taken
        y_want = want["y"].astype(np.float64)
        if addend is not None:
            y_want = y_want + addend.astype(np.float64)
        extra, missing = np.nonzero(diff & g_mask)[0], np.nonzero(diff & o_mask)[0]
        if extra.size:
            y_want = y_want + d[extra].astype(np.float64) @ self.down_rows(extra)
        if missing.size:
            y_want = y_want - d[missing].astype(np.float64) @ self.down_rows(missing)
        assert_y_close(got["y"], y_want, what)
        return int(np.count_nonzero(diff))


# ------------------------------------------------------------------ packing
@pytest.mark.parametrize("rows,F,dtype", [(1, 8, np.float32), (1, 4096, np.uint16), (3, 12, np.int8), (257, 1500, np.uint16),
                                          (64, 520, np.int8), (5, 36, np.float32)])
def test_pack_gate_up_layout(rows, F, dtype):
    rng = np.random.default_rng(rows * 1000 + F)
    if dtype == np.float32:
        g, u = rng.standard_normal((rows, F)).astype(dtype), rng.standard_normal((rows, F)).astype(dtype)
    else:
        info = np.iinfo(dtype)
        g = rng.integers(info.min, info.max, size=(rows, F), endpoint=True).astype(dtype)
        u = rng.integers(info.min, info.max, size=(rows, F), endpoint=True).astype(dtype)
    tdt = {np.float32: torch.float32, np.uint16: torch.int16, np.int8: torch.int8}[dtype]
    gd = torch.from_numpy(g.view(np.int16) if dtype == np.uint16 else g).cuda()
    ud = torch.from_numpy(u.view(np.int16) if dtype == np.uint16 else u).cuda()
    assert gd.dtype == tdt
    out = scap.pack_gate_up(gd, ud).cpu().numpy()
    want = pack_host(g, u)
    assert np.array_equal(out.view(dtype), want)
    # column p of the packed array: group p // 8, gate for p % 8 < 4
    for p in (0, 3, 4, 7, 8, 2 * F - 1):
        src = g if p % 8 < 4 else u
        assert np.array_equal(want[:, p], src[:, (p // 8) * 4 + p % 4])


# ------------------------------------------------------------------ small blocks: tiles, splits, ragged tails
SMALL = [
    # K, F, N
    (8, 8, 8), (64, 64, 16), (200, 328, 136), (130, 1032, 520), (1000, 1500, 264), (512, 4100, 1032), (3000, 776, 4104),
]


@pytest.mark.parametrize("dt", [F16, BF16])
@pytest.mark.parametrize("K,F,N", SMALL)
def test_small_blocks(dt, K, F, N):
    blk = Block(K, F, N, dt, seed=500 + K)
    X = wl.laplace(3, K, 600 + K, dt, loc=0.1, scale=0.8)
    rng = np.random.default_rng(K + F)
    bg, bu, bd = (rng.standard_normal(n).astype(np.float32) * 0.05 for n in (F, F, N))
    zs = np.abs(oracle.swiglu_block(blk.Wg, blk.Wu, blk.Wd, X[0], 0.1, 0.5, 0.0, 0.0, dt, dt, b_gate=bg, b_up=bu)["z"])
    flips = 0
    for tau_x, tau_z in ((0.0, 0.0), (0.5, float(np.median(zs))), (1.1, float(np.quantile(zs, 0.8))), (0.5, 1e9)):
        for b in range(X.shape[0]):
            say(f"block K={K} F={F} N={N} dt={dt} tau_x={tau_x} tau_z={tau_z:.4g} vec={b}")
            flips += blk.check(X[b], dt, 0.1, tau_x, bg, bu, 0.002, tau_z, bd, f"K={K} F={F} N={N} tau_z={tau_z}")[2]
    assert flips <= 6   # band decisions are rare


@pytest.mark.parametrize("K,F,N", [(64, 64, 16), (520, 1032, 2064), (1000, 2056, 528)])
def test_small_blocks_int8(K, F, N):
    blk = Block(K, F, N, I8, seed=700 + K)
    X = wl.laplace(2, K, 800 + K, BF16, loc=0.0, scale=0.8)
    zs = np.abs(oracle.swiglu_block(blk.Wg, blk.Wu, blk.Wd, X[0], 0.0, 0.4, 0.0, 0.0, I8, BF16, gate_scale=blk.sg,
                                    up_scale=blk.su, down_scale=blk.sd)["z"])
    for tau_x, tau_z in ((0.0, 0.0), (0.4, float(np.quantile(zs, 0.7)))):
        for b in range(X.shape[0]):
            say(f"block int8 K={K} F={F} N={N} tau_x={tau_x} tau_z={tau_z:.4g} vec={b}")
            blk.check(X[b], BF16, 0.0, tau_x, None, None, 0.0, tau_z, None, f"int8 K={K} F={F} N={N}")


@pytest.mark.parametrize("K,F,N,dt", [(256, 512, 128, BF16), (1000, 2056, 528, F16), (520, 1032, 2064, I8), (4096, 14336, 4096, BF16)])
def test_residual_block_adds_to_y(K, F, N, dt):
    """scap_swiglu_block_residual: y starts as a given addend and ends as addend + block output (fp32 atomic adds in the
    down launch, so compared at the float tolerance); z, the kept list and its count are exact as in the plain
    block; an ordinary block on the same workspace afterwards; more than one token is refused."""
    blk = Block(K, F, N, dt, seed=900 + K, std=0.02 if K >= 4096 else 0.05)
    xdt = BF16 if dt == I8 else dt
    X = wl.laplace(3, K, 901 + K, xdt, loc=0.0, scale=0.8)
    rng = np.random.default_rng(K + F + N)
    addend = rng.standard_normal(N).astype(np.float32)
    bd = rng.standard_normal(N).astype(np.float32) * 0.05
    sg = dict(gate_scale=blk.sg, up_scale=blk.su, down_scale=blk.sd)
    zs = np.abs(oracle.swiglu_block(blk.Wg, blk.Wu, blk.Wd, X[0], 0.0, 0.5, 0.0, 0.0, dt, xdt, nthreads=8, **sg)["z"])
    for b, (tau_x, tau_z) in enumerate(((0.0, 0.0), (0.5, float(np.median(zs))), (0.9, 1e9))):
        say(f"residual block K={K} F={F} N={N} dt={dt} tau_x={tau_x} tau_z={tau_z:.4g}")
        blk.check(X[b], xdt, 0.0, tau_x, None, None, 0.0, tau_z, bd, f"residual block K={K} tau_z={tau_z}", addend=addend)
    say("an ordinary block afterwards")
    blk.check(X[1], xdt, 0.0, 0.5, None, None, 0.0, float(np.median(zs)), bd, "block after residual blocks")
    blk2 = Block(64, 64, 16, BF16, seed=77, B=2)
    with pytest.raises(scap.ScapError):
        scap.swiglu_block(blk2.W_gu, blk2.W_down, to_dev(wl.laplace(2, 64, 78, BF16, loc=0.0, scale=1.0), BF16), 0.0, 0.1, None,
                          0.0, 0.1, None, y=torch.zeros((2, 16), dtype=torch.float32, device="cuda"), workspace=blk2.ws,
                          residual=True)


@pytest.mark.parametrize("K,F,N,dt", [(256, 512, 128, BF16), (1000, 2056, 528, F16), (520, 1032, 2064, I8), (4096, 14336, 4096, BF16)])
def test_one_token_block_hand_overs(K, F, N, dt):
    """The one-token block with each hand-over of its two launches: fixed-point atomics (the default; the gating
    epilogue of a slice run from registers), the same with every slice gated by the way through memory (what a slice
    takes when more than one wavefront finished its columns) -- bit-identical to the default in z, list and y --, and
    fp32 partial sums; each against the oracle."""
    blk = Block(K, F, N, dt, seed=950 + K, std=0.02 if K >= 4096 else 0.05)
    xdt = BF16 if dt == I8 else dt
    X = wl.laplace(2, K, 951 + K, xdt, loc=0.0, scale=0.8)
    rng = np.random.default_rng(K + F)
    bd = rng.standard_normal(N).astype(np.float32) * 0.05
    sg = dict(gate_scale=blk.sg, up_scale=blk.su, down_scale=blk.sd)
    zs = np.abs(oracle.swiglu_block(blk.Wg, blk.Wu, blk.Wd, X[0], 0.0, 0.5, 0.0, 0.0, dt, xdt, nthreads=8, **sg)["z"])
    for b, (tau_x, tau_z) in enumerate(((0.0, 0.0), (0.5, float(np.median(zs))))):
        say(f"block hand-overs K={K} F={F} N={N} dt={dt} tau_x={tau_x} tau_z={tau_z:.4g}")
        fx, _, _ = blk.check(X[b], xdt, 0.0, tau_x, None, None, 0.0, tau_z, bd, "block, fixed point")
        parked, _, _ = blk.check(X[b], xdt, 0.0, tau_x, None, None, 0.0, tau_z, bd, "block, parked slices",
                                 cfg=(0, 0, 0, 0, scap.CFG_PARK_SLICES))
        blk.check(X[b], xdt, 0.0, tau_x, None, None, 0.0, tau_z, bd, "block, partial sums", cfg=(0, 0, 0, 0, scap.CFG_PARTIAL_SUMS))
        assert np.array_equal(fx["z"].view(np.uint32), parked["z"].view(np.uint32))
        assert np.array_equal(fx["idx_z"], parked["idx_z"])
        assert np.array_equal(fx["y"].view(np.uint32), parked["y"].view(np.uint32))


# ------------------------------------------------------------------ several tokens: own masks, union of rows
@pytest.mark.parametrize("dt", [BF16, I8, F16])
@pytest.mark.parametrize("B", [2, 3, 4, 5, 8, 13, 16])
def test_batched_blocks(B, dt):
    K, F, N = 1000, 2056, 1040
    blk = Block(K, F, N, dt, seed=840 + B, B=B)
    xdt = F16 if dt == F16 else BF16
    X = wl.laplace(B, K, 850 + B, xdt, loc=0.1, scale=0.8)
    rng = np.random.default_rng(860 + B)
    bg, bu, bd = (rng.standard_normal(n).astype(np.float32) * 0.05 for n in (F, F, N))
    zs = np.abs(oracle.swiglu_block(blk.Wg, blk.Wu, blk.Wd, X[0], 0.1, 0.5, 0.0, 0.0, dt, xdt, b_gate=bg, b_up=bu,
                                    gate_scale=blk.sg, up_scale=blk.su, down_scale=blk.sd)["z"])
    for tau_x, tau_z in ((0.0, 0.0), (0.5, float(np.median(zs))), (1.1, float(np.quantile(zs, 0.9))), (0.5, 1e9)):
        say(f"batched block B={B} dt={dt} tau_x={tau_x} tau_z={tau_z:.4g}")
        a = blk.check_batch(X, xdt, 0.1, tau_x, bg, bu, 0.002, tau_z, bd, f"B={B} dt={dt} tau_z={tau_z}")
        if B <= 4:  # 2-4 tokens: launches that run on the two- / four-slot kernel by default, and the general kernels
            g = blk.check_batch(X, xdt, 0.1, tau_x, bg, bu, 0.002, tau_z, bd, f"general kernels B={B} dt={dt} tau_z={tau_z}",
                                cfg=(0, 0, 0, 0, scap.CFG_GENERAL_KERNEL))
            if dt != I8:  # the same gate|up kernel on both ways: the same z, the same lists
                for b in range(B):
                    assert np.array_equal(a[b]["z"].view(np.uint32), g[b]["z"].view(np.uint32))
                    assert np.array_equal(a[b]["idx_z"], g[b]["idx_z"])


@pytest.mark.parametrize("K,F,N,dt", [(1000, 2056, 1040, I8), (4096, 6144, 2080, I8), (520, 1032, 2064, I8), (256, 8, 16, I8),
                                      (1000, 2056, 1040, BF16), (4096, 14336, 4096, BF16), (777, 4104, 528, F16),
                                      (4096, 14336, 4096, I8)])
def test_two_token_block_on_the_two_token_kernel_and_on_the_general_kernels(K, F, N, dt):
    """Two tokens: by default each launch of the block runs on the two-token kernel where it applies (gate|up: int8
    weights with 2F > 4096; down: all weights), in the batched kernels' list format, so that the two
    forms mix; SCAP_CFG_GENERAL_KERNEL keeps both launches on the general kernels.  Both against the oracle token by
    token; z and the kept lists of the two must agree wherever the gate|up launch is the same kernel."""
    blk = Block(K, F, N, dt, seed=2600 + K, std=0.02 if K > 2000 else 0.05, B=2)
    xdt = F16 if dt == F16 else BF16
    X = wl.laplace(8, K, 2601 + K, xdt, loc=0.1, scale=0.8)
    rng = np.random.default_rng(2602 + K)
    bg, bu, bd = (rng.standard_normal(n).astype(np.float32) * 0.05 for n in (F, F, N))
    zs = np.abs(oracle.swiglu_block(blk.Wg, blk.Wu, blk.Wd, X[0], 0.1, 0.5, 0.0, 0.0, dt, xdt, b_gate=bg, b_up=bu,
                                    gate_scale=blk.sg, up_scale=blk.su, down_scale=blk.sd)["z"])
    full = K * F > 1 << 24
    cases = ((0.5, float(np.median(zs))),) if full else ((0.0, 0.0), (0.5, float(np.median(zs))), (1.1, float(np.quantile(zs, 0.9))), (0.5, 1e9), (1e9, 0.0))
    for rep, (tau_x, tau_z) in enumerate(cases):
        x = X[2 * (rep % 4):2 * (rep % 4) + 2]
        say(f"two-token block K={K} F={F} N={N} dt={dt} tau_x={tau_x} tau_z={tau_z:.4g}")
        a = blk.check_batch(x, xdt, 0.1, tau_x, bg, bu, 0.002, tau_z, bd, f"two-token kernel tau_z={tau_z}")
        g = blk.check_batch(x, xdt, 0.1, tau_x, bg, bu, 0.002, tau_z, bd, f"general kernels tau_z={tau_z}",
                            cfg=(0, 0, 0, 0, scap.CFG_GENERAL_KERNEL))
        again = blk.run_batch(x, xdt, 0.1, tau_x, bg, bu, 0.002, tau_z, bd)
        for b in range(2):
            assert np.array_equal(a[b]["y"].view(np.uint32), again[b]["y"].view(np.uint32)), "not reproducible"
            assert np.array_equal(a[b]["idx_z"], again[b]["idx_z"])
            if dt != I8:  # the same gate|up kernel on both ways: the same z, the same lists
                assert np.array_equal(a[b]["z"].view(np.uint32), g[b]["z"].view(np.uint32))
                assert np.array_equal(a[b]["idx_z"], g[b]["idx_z"])


# ------------------------------------------------------------------ degenerate cases
def test_nothing_kept_and_everything_kept():
    K, F, N = 300, 520, 264
    blk = Block(K, F, N, BF16, seed=900)
    x = wl.laplace(1, K, 901, BF16, loc=0.0, scale=1.0)[0]
    bd = np.random.default_rng(902).standard_normal(N).astype(np.float32)
    # second pruner drops everything: y is the fused bias exactly, the list is empty
    got = blk.run(x, BF16, 0.0, 0.3, None, None, 0.0, 1e30, bd)
    assert got["idx_z"].size == 0 and np.array_equal(got["y"], bd)
    # first pruner drops everything: gate = up = fused bias = 0, z = 0, nothing passes a strict compare with 0
    got = blk.run(x, BF16, 0.0, 1e30, None, None, 0.0, 0.0, bd)
    assert got["idx_z"].size == 0 and np.array_equal(got["y"], bd) and not got["z"].any()
    # a centred second pruner with an all-zero z keeps every channel at d = -m_z
    got, want, _ = blk.check(x, BF16, 0.0, 1e30, None, None, 0.25, 0.1, bd, "all-zero z, centred")
    assert got["idx_z"].size == F
    # outputs not asked for
    got = blk.run(x, BF16, 0.0, 0.3, None, None, 0.0, 0.01, bd, want_lists=False, want_z=False)
    ref = blk.run(x, BF16, 0.0, 0.3, None, None, 0.0, 0.01, bd)
    assert np.array_equal(got["y"], ref["y"])


def test_block_is_bit_reproducible_and_workspace_is_reusable():
    K, F, N = 1000, 2056, 1032
    blk = Block(K, F, N, BF16, seed=910)
    X = wl.laplace(2, K, 911, BF16, loc=0.0, scale=1.0)
    a0 = blk.run(X[0], BF16, 0.0, 0.4, None, None, 0.0, 0.02, None)
    b0 = blk.run(X[1], BF16, 0.0, 0.9, None, None, 0.0, 0.05, None)
    a1 = blk.run(X[0], BF16, 0.0, 0.4, None, None, 0.0, 0.02, None)
    b1 = blk.run(X[1], BF16, 0.0, 0.9, None, None, 0.0, 0.05, None)
    for p, q in ((a0, a1), (b0, b1)):
        assert np.array_equal(p["y"], q["y"]) and np.array_equal(p["z"], q["z"]) and np.array_equal(p["idx_z"], q["idx_z"])
    # the workspace of a block also serves plain calls on its layers
    y = scap.dense_fc(blk.W_down, to_dev(wl.laplace(1, F, 912, BF16)[0], BF16), None, workspace=blk.ws)
    torch.cuda.synchronize()
    assert np.isfinite(y.cpu().numpy()).all()


def test_block_argument_errors():
    K, F, N = 64, 64, 16
    blk = Block(K, F, N, BF16, seed=920)
    x = to_dev(wl.laplace(5, K, 921, BF16), BF16)
    with pytest.raises(scap.ScapError) as e:
        scap.swiglu_block(blk.W_gu, blk.W_down, x[0], 0.0, -1.0, None, 0.0, 0.1, None, workspace=blk.ws)
    assert e.value.status == -5
    with pytest.raises(scap.ScapError) as e:
        scap.swiglu_block(blk.W_gu, blk.W_down, x[0], 0.0, 0.1, None, 0.0, float("nan"), None, workspace=blk.ws)
    assert e.value.status == -5
    small = scap.Workspace(K, N, 1)
    small.nbytes = 4096
    with pytest.raises(scap.ScapError) as e:
        scap.swiglu_block(blk.W_gu, blk.W_down, x[0], 0.0, 0.1, None, 0.0, 0.1, None, workspace=small)
    assert e.value.status == -6
    idx = torch.empty(F, dtype=torch.int32, device="cuda")
    with pytest.raises(scap.ScapError) as e:
        scap.swiglu_block(blk.W_gu, blk.W_down, x[0], 0.0, 0.1, None, 0.0, 0.1, None, idx_z_out=idx, workspace=blk.ws)
    assert e.value.status == -1


# ------------------------------------------------------------------ full size: the Mistral-7B feed-forward block
@pytest.mark.parametrize("s_x,s_z", [(0.5, 0.5), (0.3, 0.7)])
def test_mistral_ffn_block_full_size(s_x, s_z):
    K, F, N = 4096, 14336, 4096
    site = wl.sites(3)[2]     # gate|up input of the Mistral layer
    assert site.K == K
    blk = Block(K, F, N, BF16, seed=3003, std=0.02)
    m_x, tau_x = oracle.calibrate(site.calib(), site.xdt, s_x, oracle.MODE_MEDIAN)
    X = site.test_vectors(3)
    # threshold of the gated product from the oracle's own z on calibration vectors
    zc = np.concatenate([oracle.swiglu_block(blk.Wg, blk.Wu, blk.Wd, v, m_x, tau_x, 0.0, 0.0, BF16, BF16, nthreads=8)["z"]
                         for v in site.draw(2, 77)])
    tau_z = float(np.sort(np.abs(zc))[int(np.ceil(s_z * zc.size)) - 1])
    bgf, buf = oracle.fold_bias(blk.Wg, m_x, None, BF16), oracle.fold_bias(blk.Wu, m_x, None, BF16)
    for b in range(X.shape[0]):
        say(f"mistral ffn block s_x={s_x} s_z={s_z} vec={b}")
        got, want, flips = blk.check(X[b], BF16, m_x, tau_x, bgf, buf, 0.0, tau_z, None, f"mistral block vec {b}")
        dens = got["idx_z"].size / F
        assert abs(dens - (1 - s_z)) < 0.05
        assert flips <= 3


@pytest.mark.parametrize("dt,B", [(BF16, 16), (I8, 8)])
def test_ffn_block_full_size_batched(dt, B):
    """The Mistral / expert feed-forward block at its real shape with a batch on the matrix cores; tokens sampled
    against the oracle (each token has its own masks, so any token checks the whole launch's plumbing)."""
    K, F, N = 4096, 14336, 4096
    site = wl.sites(3)[2]
    blk = Block(K, F, N, dt, seed=3103, std=0.02, B=B)
    m_x, tau_x = oracle.calibrate(site.calib(), site.xdt, 0.5, oracle.MODE_MEDIAN)
    X = site.draw(B, 3104)
    zc = oracle.swiglu_block(blk.Wg, blk.Wu, blk.Wd, X[0], m_x, tau_x, 0.0, 0.0, dt, BF16, gate_scale=blk.sg,
                             up_scale=blk.su, down_scale=blk.sd, nthreads=8)["z"]
    tau_z = float(np.sort(np.abs(zc))[int(np.ceil(0.6 * zc.size)) - 1])
    bgf = oracle.fold_bias(blk.Wg, m_x, None, dt, col_scale=blk.sg)
    buf = oracle.fold_bias(blk.Wu, m_x, None, dt, col_scale=blk.su)
    say(f"full-size batched block dt={dt} B={B}")
    gots = blk.run_batch(X, BF16, m_x, tau_x, bgf, buf, 0.0, tau_z, None)
    for b in sorted({0, B // 2, B - 1}):
        want = oracle.swiglu_block(blk.Wg, blk.Wu, blk.Wd, X[b], m_x, tau_x, 0.0, tau_z, dt, BF16, b_gate=bgf, b_up=buf,
                                   gate_scale=blk.sg, up_scale=blk.su, down_scale=blk.sd, nthreads=8)
        flips = blk.compare(gots[b], want, 0.0, tau_z, f"full-size batched block token {b}",
                            matrix_cores=B_MATRIX(dt, B))
        assert flips <= 3
        assert abs(gots[b]["idx_z"].size / F - 0.4) < 0.06


def test_blocks_on_two_streams_with_their_own_workspaces():
    """Independent blocks (experts of a mixture) may overlap in time when each stream has its own workspace:
    results equal the one-after-the-other results bit for bit."""
    K, F, N = 1024, 2048, 1024
    blks = [Block(K, F, N, I8, seed=8100, B=8), Block(K, F, N, BF16, seed=8200, B=8)]
    X = to_dev(wl.laplace(16, K, 8300, BF16, loc=0.0, scale=1.0), BF16)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]

    def call(blk, x, y, stream=None):
        scap.swiglu_block(blk.W_gu, blk.W_down, x, 0.0, 0.4, None, 0.0, 0.05, None, gu_scale=blk.gu_scale,
                          down_scale=blk.down_scale, y=y, workspace=blk.ws, stream=stream)

    cases = [(blks[0], X[i], (1, N)) for i in range(8)] + [(blks[0], X[i:i + 5], (5, N)) for i in range(4)]
    cases2 = [(blks[1], X[i:i + 8], (8, N)) for i in range(8)] + [(blks[1], X[i], (1, N)) for i in range(4)]
    refs = []
    for group in (cases, cases2):
        for blk, x, shape in group:
            y = torch.empty(shape, dtype=torch.float32, device="cuda")
            call(blk, x, y)
            refs.append(y)
    torch.cuda.synchronize()
    for rep in range(3):
        say(f"blocks on two streams rep {rep}")
        outs = [torch.full(r.shape, float("nan"), dtype=torch.float32, device="cuda") for r in refs]
        torch.cuda.synchronize()
        for i in range(len(cases)):
            for s, group, base in ((0, cases, 0), (1, cases2, len(cases))):
                blk, x, _ = group[i]
                with torch.cuda.stream(streams[s]):
                    call(blk, x, outs[base + i], stream=streams[s])
        torch.cuda.synchronize()
        for i, (o, r) in enumerate(zip(outs, refs)):
            assert torch.equal(o, r), f"rep {rep} call {i}"


def test_random_blocks():
    """Seeded sweep over odd block shapes, 1-16 tokens, every weight dtype."""
    rng = np.random.default_rng(20241208)
    for case in range(24):
        dt = (F16, BF16, I8)[case % 3]
        xdt = BF16 if dt == I8 else dt
        K = int(rng.integers(8, 3000))
        F = (8 if dt == I8 else 4) * int(rng.integers(1, 600))
        N = (16 if dt == I8 else 8) * int(rng.integers(1, 300))
        B = int(rng.choice([1, 1, 2, 3, 4, 6, 16]))
        blk = Block(K, F, N, dt, seed=5000 + case, B=B)
        X = wl.laplace(B, K, 6000 + case, xdt, loc=0.05, scale=0.9)
        zs = np.abs(oracle.swiglu_block(blk.Wg, blk.Wu, blk.Wd, X[0], 0.05, 0.3, 0.0, 0.0, dt, xdt, gate_scale=blk.sg,
                                        up_scale=blk.su, down_scale=blk.sd)["z"])
        tau_x = float(rng.choice([0.0, 0.3, 0.9]))
        tau_z = float(np.quantile(zs, rng.choice([0.0, 0.4, 0.9])))
        say(f"random block {case}: dt={dt} K={K} F={F} N={N} B={B} tau_x={tau_x} tau_z={tau_z:.4g}")
        blk.check_batch(X, xdt, 0.05, tau_x, None, None, 0.001, tau_z, None, f"random block {case}")


def test_mixture_of_experts_layer_grouped_by_expert():
    """Config-5 style layer at small size: 8 int8 experts, top-2 routing from seeded logits (harness level, the same
    on both sides), tokens grouped per expert on the GPU side (each group one fused block call with its own batch
    size), one token at a time on the oracle side; outputs combined with the gate weights."""
    K, F, N, E, B = 256, 512, 256, 8, 8
    experts = [Block(K, F, N, I8, seed=7000 + 10 * e, B=B) for e in range(E)]
    X = wl.laplace(B, K, 7100, BF16, loc=0.0, scale=0.8)
    order, gate = wl.top2_route(wl.router_logits(B, E, 7101))
    m_x, tau_x, m_z = 0.0, 0.35, 0.0
    zs = np.abs(oracle.swiglu_block(experts[0].Wg, experts[0].Wu, experts[0].Wd, X[0], m_x, tau_x, 0.0, 0.0, I8, BF16,
                                    gate_scale=experts[0].sg, up_scale=experts[0].su, down_scale=experts[0].sd)["z"])
    tau_z = float(np.quantile(zs, 0.7))
    want = np.zeros((B, N))
    for t in range(B):
        for slot in range(2):
            e = int(order[t, slot])
            blk = experts[e]
            y = oracle.swiglu_block(blk.Wg, blk.Wu, blk.Wd, X[t], m_x, tau_x, m_z, tau_z, I8, BF16, gate_scale=blk.sg,
                                    up_scale=blk.su, down_scale=blk.sd)["y"]
            want[t] += gate[t, slot] * y.astype(np.float64)
    got = np.zeros((B, N))
    sizes = []
    for e in range(E):
        tok, slot = np.nonzero(order == e)
        if tok.size == 0:
            continue
        sizes.append(int(tok.size))
        say(f"expert {e}: tokens {tok.tolist()}")
        outs = experts[e].run_batch(X[tok], BF16, m_x, tau_x, None, None, m_z, tau_z, None)
        for j, t in enumerate(tok):
            got[t] += gate[t, slot[j]] * outs[j]["y"].astype(np.float64)
    assert sum(sizes) == 2 * B and max(sizes) >= 2
    # a band decision on z moves y by about tau_z * |w| ~ 1e-3, inside the bar; compare the combined outputs
    assert_y_close(got, want, "mixture of experts")
