#!/usr/bin/env python3
"""Benchmark of the decode-time sparse FC (SCAP Alg. 3) on one MI355X.

A step is one pass of the whole hot path -- centre, threshold, compact, gathered GEMV, reduction --
for one token through one layer: a single `scap_sparse_fc` launch.  The headline workload is the
Mistral-7B down projection (14336 -> 4096, bf16, batch 1) at 50 % target sparsity on SiLU(g)*u
inputs; the same run also reports 70 % / 90 %, the dense GEMV on the same kernels, a streaming-read
ceiling, and the CPU oracle on the host cores.

Timing protocol: weights rotate through R distinct device copies (R * bytes >= 1 GiB) so that neither
L2 nor the memory-side cache serves them; the 64 seeded test vectors cycle, so masks differ from
launch to launch; the K timed launches are captured once into a HIP graph and replayed, which keeps
the Python/ctypes call overhead out of the timed region (use --eager to time direct calls).

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth

# HBM bytes per launch from rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE, scaled by a copy kernel of known size),
# keyed by workload.  These are RECORDED values, copied from the profile summaries named beside them (each of
# which gives the command that produced it); they are not measured in the run that prints them, since hardware
# counters need the profiler.  Absent = not profiled.
MEASURED_TRAFFIC = {
    "mistral7b_down_14336x4096_bf16_b1_s50":
        (60225237, "recorded: profiles/gemv1_kernel_bf16_mistral_down_hbm_traffic.txt"),
    "mistral7b_down_14336x4096_bf16_b16_s90":
        (104241478, "recorded: profiles/gemm_inline_raw_kernel_bf16_mistral_down_b16_s90_hbm_traffic.txt"),
}


def algorithmic_bytes(nnz_rows: float, K: int, N: int, B: int, wbytes: int) -> float:
    """Weight rows actually read + input + fused bias + output (index lists and split-K partials are
    overhead, not algorithmic traffic)."""
    return nnz_rows * N * wbytes + B * K * 2 + N * 4 + B * N * 4


def graph_timed(torch, fn, n, repeats=1):
    """us per call of fn(i), i = 0..n-1, captured once into a HIP graph and replayed (best of `repeats`)."""
    for i in range(10):
        fn(i)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(n):
            fn(i)
    g.replay()
    torch.cuda.synchronize()
    best = float("inf")
    for _ in range(repeats):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) / n * 1e3)
    return best


def bench_site(torch, scap, wl, dev, rows, cfg_no, site, batches, targets, est, steps, library_gemm=False):
    """One layer of a benchmark configuration: dense and sparse launches for every batch size and target, appended
    to `rows` as dicts (us per launch, GB/s on the bytes actually needed).  Weights are random on the device
    (their values do not matter for timing) and rotate over >= 1 GiB of copies; inputs come from the seeded
    generators, thresholds from scap_calibrate."""
    def dev16(bits, dt):
        t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
        return t.view(torch.float16 if dt == wl.F16 else torch.bfloat16).to(dev)

    K, N = site.K, site.N
    wbytes = 1 if site.wdt == wl.I8 else 2
    if site.wdt == wl.I8:
        W0 = torch.randint(-127, 128, (K, N), dtype=torch.int8, device=dev)
        scale = (torch.rand(N, device=dev) * 1e-3 + 1e-4).to(torch.float16)
    else:
        W0 = (torch.randn(K, N, device=dev) * 0.02).to(torch.float16 if site.wdt == wl.F16 else torch.bfloat16)
        scale = None
    R = max(2, -(-(1 << 30) // (K * N * wbytes)))
    Ws = [W0] + [W0.clone() for _ in range(R - 1)]
    X = dev16(site.draw(64, site.seed_test), site.xdt)
    calib = dev16(site.draw(128, site.seed_calib), site.xdt)
    ws = scap.Workspace(K, N, max(batches))
    unz = torch.zeros(1, dtype=torch.int32, device=dev)
    taus = {s: scap.calibrate(calib, s, est, workspace=ws) for s in targets}
    for B in batches:
        y = torch.empty((B, N), dtype=torch.float32, device=dev)

        def xs(i):
            o = (i * B) % (64 - B + 1)
            return X[o] if B == 1 else X[o:o + B]

        t_dense = graph_timed(torch, lambda i: scap.dense_fc(Ws[i % R], xs(i), None, col_scale=scale, y=y, workspace=ws), steps)
        rows.append({"cfg": cfg_no, "layer": site.name, "K": K, "N": N, "w": wl.DTYPE_NAME[site.wdt], "B": B,
                     "target": None, "density": 1.0, "us": round(t_dense, 2),
                     "GBps": round(algorithmic_bytes(K, K, N, B, wbytes) / t_dense / 1e3, 1)})
        if library_gemm and site.wdt != wl.I8:
            # the vendor library's dense GEMM on the same operands, for the crossover against a dense batch
            yl = torch.empty((B, N), dtype=W0.dtype, device=dev)
            t_lib = graph_timed(torch, lambda i: torch.matmul(xs(i).reshape(B, K), Ws[i % R], out=yl), steps)
            rows[-1]["library_dense_gemm_us"] = round(t_lib, 2)
        for s in targets:
            m, tau = taus[s]
            dens = 0.0
            for i in range(8):
                scap.sparse_fc(Ws[0], xs(i), m, tau, None, col_scale=scale, y=y, union_nnz_out=unz, workspace=ws)
                dens += unz.item() / K / 8
            t = graph_timed(torch, lambda i: scap.sparse_fc(Ws[i % R], xs(i), m, tau, None, col_scale=scale, y=y, workspace=ws), steps)
            rows.append({"cfg": cfg_no, "layer": site.name, "K": K, "N": N, "w": wl.DTYPE_NAME[site.wdt], "B": B,
                         "target": s, "density": round(dens, 4), "us": round(t, 2),
                         "GBps": round(algorithmic_bytes(dens * K, K, N, B, wbytes) / t / 1e3, 1),
                         "frac_of_8TBps": round(algorithmic_bytes(dens * K, K, N, B, wbytes) / t / 1e3 / HBM_PEAK_GBS, 4),
                         "vs_dense": round(t_dense / t, 3)})
    del Ws, W0
    torch.cuda.empty_cache()


def suite_summary(torch, scap, wl, dev, steps=200):
    """A few points of the other benchmark configurations for the default run's JSON line: the Mistral layer's FC
    set (config 3) dense and at 50 %, 16-token batches on both feed-forward layers (config 4), and the int8 expert
    down projection at 70 % with 1 and 8 tokens (config 5)."""
    rows = []
    for st in wl.sites(3):
        bench_site(torch, scap, wl, dev, rows, 3, st, (1,), (0.5,), scap.MODE_MEDIAN, steps)
    for st in wl.sites(4):
        bench_site(torch, scap, wl, dev, rows, 4, st, (16,), (0.5, 0.7, 0.9), scap.MODE_ZERO, steps, library_gemm=True)
    bench_site(torch, scap, wl, dev, rows, 5, wl.sites(5)[1], (1, 8), (0.7,), scap.MODE_MEDIAN, steps)
    layer3 = [r for r in rows if r["cfg"] == 3]
    out = {"mistral_layer_fc_set_dense_us": round(sum(r["us"] for r in layer3 if r["target"] is None), 2),
           "mistral_layer_fc_set_s50_us": round(sum(r["us"] for r in layer3 if r["target"] == 0.5), 2),
           "launches_per_point": steps, "points": []}
    for r in rows:
        out["points"].append({k: r[k] for k in ("cfg", "layer", "w", "B", "target", "density", "us", "GBps") if k in r}
                             | ({"library_dense_gemm_us": r["library_dense_gemm_us"]} if "library_dense_gemm_us" in r else {}))
    return out


def run_suite(args, torch, scap, wl, dev):
    """Every benchmark configuration, one line per (layer, batch, target sparsity): us per launch and GB/s
    on the bytes actually needed.  Prints ONE JSON line."""
    steps = max(100, args.steps // 10)
    steps_box = [steps]

    def dev16(bits, dt):
        t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
        return t.view(torch.float16 if dt == wl.F16 else torch.bfloat16).to(dev)

    def timed(fn):
        return graph_timed(torch, fn, steps_box[0])

    rows = []

    def run_site(cfg_no, site, batches, targets, est):
        bench_site(torch, scap, wl, dev, rows, cfg_no, site, batches, targets, est, steps, library_gemm=(cfg_no == 4))

    def want(part):
        return not args.only or args.only == part

    if want("layers"):
        run_site(1, wl.sites(1)[0], (1,), (0.5,), scap.MODE_MEDIAN)
        for st in wl.sites(2):
            run_site(2, st, (1,), (0.5, 0.7, 0.9), scap.MODE_MEDIAN)
        for st in wl.sites(3):
            run_site(3, st, (1,), (0.5,), scap.MODE_MEDIAN)
        for st in wl.sites(4):
            run_site(4, st, (1, 4, 16), (0.5, 0.7, 0.9), scap.MODE_ZERO)
        c5 = wl.sites(5)
        run_site(5, c5[0], (1,), (0.4,), scap.MODE_MEDIAN)
        run_site(5, c5[1], (1, 8), (0.7,), scap.MODE_MEDIAN)

    # Feed-forward blocks (Alg. 2): the fused two-launch block against the same work as separate calls
    # (sparse_fc on [gate | up], torch silu * up and cast to 16 bits, sparse_fc on down) and the dense block.
    blocks = []

    def run_block(name, K, F, N, targets):
        dt = torch.bfloat16
        Wg = (torch.randn(K, F, device=dev) * 0.02).to(dt)
        Wu = (torch.randn(K, F, device=dev) * 0.02).to(dt)
        Wd0 = (torch.randn(F, N, device=dev) * 0.02).to(dt)
        R = max(2, -(-(1 << 30) // (3 * K * F * 2)))
        Wcat = [torch.cat([Wg, Wu], dim=1).contiguous() for _ in range(R)]
        Wgu = [scap.pack_gate_up(Wg, Wu) for _ in range(R)]
        Wd = [Wd0.clone() for _ in range(R)]
        del Wg, Wu
        site = wl.Site(name, K, 2 * F, wl.BF16, wl.BF16, "prenorm", 128, 4001, 4002, 4003)
        X = dev16(site.draw(64, site.seed_test), wl.BF16)
        calib = dev16(site.draw(128, site.seed_calib), wl.BF16)
        ws = scap.Workspace(K, N, 1, F=F)
        ycat = torch.empty((1, 2 * F), dtype=torch.float32, device=dev)
        y = torch.empty((1, N), dtype=torch.float32, device=dev)
        nz = torch.zeros(1, dtype=torch.int32, device=dev)
        nx = torch.zeros(1, dtype=torch.int32, device=dev)

        def dense_block(i):
            scap.dense_fc(Wcat[i % R], X[i % 64], None, y=ycat, workspace=ws)
            z = (torch.nn.functional.silu(ycat[:, :F]) * ycat[:, F:]).to(dt)
            scap.dense_fc(Wd[i % R], z, None, y=y, workspace=ws)

        t_dense = timed(dense_block)
        blocks.append({"block": name, "K": K, "F": F, "N": N, "variant": "dense, 2 calls + torch silu*up", "target": None,
                       "us": round(t_dense, 2)})
        for s in targets:
            m_x, tau_x = scap.calibrate(calib, s, scap.MODE_MEDIAN, workspace=ws)
            bgu = scap.fold_bias(Wgu[0], m_x, None, workspace=ws)
            bcat = scap.fold_bias(Wcat[0], m_x, None, workspace=ws)
            zc = torch.empty((32, F), dtype=dt, device=dev)
            for j in range(32):
                scap.sparse_fc(Wcat[0], calib[j], m_x, tau_x, bcat, y=ycat, workspace=ws)
                zc[j] = (torch.nn.functional.silu(ycat[0, :F]) * ycat[0, F:]).to(dt)
            _, tau_z = scap.calibrate(zc, s, scap.MODE_ZERO, workspace=ws)

            def unfused(i):
                scap.sparse_fc(Wcat[i % R], X[i % 64], m_x, tau_x, bcat, y=ycat, workspace=ws)
                z = (torch.nn.functional.silu(ycat[:, :F]) * ycat[:, F:]).to(dt)
                scap.sparse_fc(Wd[i % R], z, 0.0, tau_z, None, y=y, workspace=ws)

            def fused(i):
                scap.swiglu_block(Wgu[i % R], Wd[i % R], X[i % 64], m_x, tau_x, bgu, 0.0, tau_z, None, y=y, workspace=ws)

            dx = dz = 0.0
            for i in range(8):
                scap.sparse_fc(Wcat[0], X[i], m_x, tau_x, bcat, y=ycat, nnz_out=nx, workspace=ws)
                scap.swiglu_block(Wgu[0], Wd[0], X[i], m_x, tau_x, bgu, 0.0, tau_z, None, y=y, nnz_z_out=nz, workspace=ws)
                dx += nx.item() / K / 8
                dz += nz.item() / F / 8
            def fused_residual(i):  # y += block output (another operation: the residual addition taken into the block)
                scap.swiglu_block(Wgu[i % R], Wd[i % R], X[i % 64], m_x, tau_x, bgu, 0.0, tau_z, None, y=y, workspace=ws,
                                  residual=True)

            t_u, t_f = timed(unfused), timed(fused)
            y.zero_()
            t_r = timed(fused_residual)
            nbytes = dx * K * 2 * F * 2 + dz * F * N * 2 + K * 2 + 2 * F * 4 + N * 4
            for variant, t in (("sparse, 2 calls + torch silu*up", t_u), ("sparse, fused block", t_f),
                               ("sparse, fused block adding to y (fp32 atomic adds)", t_r)):
                blocks.append({"block": name, "K": K, "F": F, "N": N, "variant": variant, "target": s,
                               "density_x": round(dx, 4), "density_z": round(dz, 4), "us": round(t, 2),
                               "GBps": round(nbytes / t / 1e3, 1), "vs_dense": round(t_dense / t, 3)})
        del Wcat, Wgu, Wd
        torch.cuda.empty_cache()

    if want("blocks"):
        run_block("mistral7b_ffn", 4096, 14336, 4096, (0.5, 0.7, 0.9))
        run_block("llama2_7b_ffn", 4096, 11008, 4096, (0.5,))

    # Latency of the fused block against FFN sparsity (Appendix B: the latency-scaling figure and the rule
    # FFN sparsity = 2/3 s_x + 1/3 s_gated for three equal-sized FCs): a grid of input and gated-product targets,
    # each point timed on its own, then one straight line through all of them.
    grids = []

    def run_block_grid(name, K, F, N, wname):
        dt = torch.bfloat16
        i8 = wname == "i8"
        levels = (0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8)
        if i8:
            Wgu0 = torch.randint(-127, 128, (K, 2 * F), dtype=torch.int8, device=dev)
            Wd0 = torch.randint(-127, 128, (F, N), dtype=torch.int8, device=dev)
            sgu = (torch.rand(2 * F, device=dev) * 2e-4 + 1e-4).to(torch.float16)
            sdn = (torch.rand(N, device=dev) * 2e-4 + 1e-4).to(torch.float16)
        else:
            Wgu0 = (torch.randn(K, 2 * F, device=dev) * 0.02).to(dt)
            Wd0 = (torch.randn(F, N, device=dev) * 0.02).to(dt)
            sgu = sdn = None
        wb = 1 if i8 else 2
        R = max(2, -(-(1 << 30) // (3 * K * F * wb)))
        Wgu = [Wgu0] + [Wgu0.clone() for _ in range(R - 1)]
        Wd = [Wd0] + [Wd0.clone() for _ in range(R - 1)]
        site = wl.Site(name, K, 2 * F, wl.BF16, wl.BF16, "prenorm", 128, 4101, 4102, 4103)
        X = dev16(site.draw(64, site.seed_test), wl.BF16)
        calib = dev16(site.draw(32, site.seed_calib), wl.BF16)
        ws = scap.Workspace(K, N, 1, F=F)
        y = torch.empty((1, N), dtype=torch.float32, device=dev)
        zf = torch.empty((1, F), dtype=torch.float32, device=dev)
        nz = torch.zeros(1, dtype=torch.int32, device=dev)
        nx = torch.zeros(1, dtype=torch.int32, device=dev)
        ygu = torch.empty((1, 2 * F), dtype=torch.float32, device=dev)
        n = max(50, steps // 2)
        t_dense = graph_timed(torch, lambda i: scap.swiglu_block(Wgu[i % R], Wd[i % R], X[i % 64], 0.0, 0.0, None, 0.0, 0.0,
                                                                 None, gu_scale=sgu, down_scale=sdn, y=y, workspace=ws), n)
        pts = []
        for sx in levels:
            m_x, tau_x = scap.calibrate(calib, sx, scap.MODE_MEDIAN, workspace=ws)
            bgu = scap.fold_bias(Wgu[0], m_x, None, col_scale=sgu, workspace=ws)
            zc = torch.empty((32, F), dtype=dt, device=dev)
            for j in range(32):   # the gated product the block itself forms at this input sparsity
                scap.swiglu_block(Wgu[0], Wd[0], calib[j], m_x, tau_x, bgu, 0.0, 0.0, None, gu_scale=sgu, down_scale=sdn,
                                  y=y, z_out=zf, workspace=ws)
                zc[j] = zf[0].to(dt)
            for sz in levels:
                _, tau_z = scap.calibrate(zc, sz, scap.MODE_ZERO, workspace=ws)
                dx = dz = 0.0
                for i in range(4):
                    scap.sparse_fc(Wgu[0], X[i], m_x, tau_x, bgu, col_scale=sgu, y=ygu, nnz_out=nx, workspace=ws)
                    scap.swiglu_block(Wgu[0], Wd[0], X[i], m_x, tau_x, bgu, 0.0, tau_z, None, gu_scale=sgu, down_scale=sdn,
                                      y=y, nnz_z_out=nz, workspace=ws)
                    dx += nx.item() / K / 4
                    dz += nz.item() / F / 4
                t = graph_timed(torch, lambda i: scap.swiglu_block(Wgu[i % R], Wd[i % R], X[i % 64], m_x, tau_x, bgu, 0.0, tau_z,
                                                                   None, gu_scale=sgu, down_scale=sdn, y=y, workspace=ws), n)
                ffn = (2 * (1 - dx) + (1 - dz)) / 3
                pts.append({"s_x": sx, "s_gated": sz, "sparsity_x": round(1 - dx, 4), "sparsity_gated": round(1 - dz, 4),
                            "ffn_sparsity": round(ffn, 4), "us": round(t, 2)})
        xs_ = np.array([0.0] + [p["ffn_sparsity"] for p in pts])
        ts_ = np.array([t_dense] + [p["us"] for p in pts])
        A = np.stack([np.ones_like(xs_), xs_], axis=1)
        coef, *_ = np.linalg.lstsq(A, ts_, rcond=None)
        r2 = 1.0 - float(((A @ coef - ts_) ** 2).sum()) / float(((ts_ - ts_.mean()) ** 2).sum())
        grids.append({"block": name, "w": wname, "K": K, "F": F, "N": N, "nothing_pruned_us": round(t_dense, 2),
                      "fit_us_at_ffn_sparsity_0": round(float(coef[0]), 2), "fit_us_per_unit_ffn_sparsity": round(float(coef[1]), 2),
                      "fit_us_at_ffn_sparsity_1": round(float(coef[0] + coef[1]), 2), "r2": round(r2, 5),
                      "max_abs_residual_us": round(float(np.abs(A @ coef - ts_).max()), 2), "launches_per_point": n,
                      "points": pts})
        del Wgu, Wd, Wgu0, Wd0
        torch.cuda.empty_cache()

    if want("grid"):
        run_block_grid("mistral7b_ffn", 4096, 14336, 4096, "bf16")
        run_block_grid("mistral7b_ffn", 4096, 14336, 4096, "i8")

    # Mixture-of-experts feed-forward (config 5): 8 int8 experts, top-2 routing from seeded logits, the tokens
    # of a step grouped per expert; an expert's group goes through the fused block or through separate calls.
    # Routing is done beforehand on the host (it is not part of the library); gathering the group's tokens and
    # the gate-weighted scatter-add are torch ops inside the timed region.  Experts are independent, so the last
    # variant spreads their blocks over 4 streams (one workspace each): one block's prologue and hand-over
    # phases, when HBM idles, overlap another block's weight stream.
    moe_rows = []

    def run_moe():
        K, F, N, E = 4096, 14336, 4096, 8
        dt = torch.bfloat16
        Wgu, sgu, Wdn, sdn = [], [], [], []
        for e in range(E):
            Wgu.append(torch.randint(-127, 128, (K, 2 * F), dtype=torch.int8, device=dev))
            sgu.append((torch.rand(2 * F, device=dev) * 2e-4 + 1e-4).to(torch.float16))
            Wdn.append(torch.randint(-127, 128, (F, N), dtype=torch.int8, device=dev))
            sdn.append((torch.rand(N, device=dev) * 2e-4 + 1e-4).to(torch.float16))
        site = wl.Site("moe_in", K, 2 * F, wl.I8, wl.BF16, "prenorm", 128, 5001, 5002, 5003)
        X = dev16(site.draw(256, site.seed_test), wl.BF16)
        calib = dev16(site.draw(128, site.seed_calib), wl.BF16)
        ws = scap.Workspace(K, N, 8, F=F)
        wsb = scap.Workspace(K, N, 8, F=F)
        n_side = 4
        side = [torch.cuda.Stream() for _ in range(n_side)]
        side_ws = [scap.Workspace(K, N, 8, F=F) for _ in range(n_side)]
        m_x, tau_x = scap.calibrate(calib, 0.4, scap.MODE_MEDIAN, workspace=ws)
        bgu = [scap.fold_bias(Wgu[e], m_x, None, col_scale=sgu[e], workspace=ws) for e in range(E)]
        ygu = torch.empty((8, 2 * F), dtype=torch.float32, device=dev)

        def gate(yv):  # packed columns: groups of 4 gate, 4 up
            v = yv.view(yv.shape[0], F // 4, 2, 4)
            return (torch.nn.functional.silu(v[:, :, 0, :]) * v[:, :, 1, :]).reshape(yv.shape[0], F).to(dt)

        zc = torch.empty((32, F), dtype=dt, device=dev)
        for j in range(32):
            scap.sparse_fc(Wgu[0], calib[j], m_x, tau_x, bgu[0], col_scale=sgu[0], y=ygu[:1], workspace=ws)
            zc[j] = gate(ygu[:1])[0]
        _, tau_z = scap.calibrate(zc, 0.7, scap.MODE_ZERO, workspace=ws)

        for B in (1, 8):
            nsteps = max(50, steps // 2)
            order, gatew = wl.top2_route(wl.router_logits(B * nsteps, E, 5004 + B))
            # Routing as a serving stack does it: the step's (token, expert) pairs are sorted by expert once, the
            # inputs of all experts are gathered in one go, every expert works on its contiguous slice, and the
            # gate-weighted outputs are scattered back and added in one go.
            plans = []
            for i in range(nsteps):
                groups, src_all, dst_all, gw_all, off = [], [], [], [], 0
                for e in range(E):
                    tok, slot = np.nonzero(order[i * B:(i + 1) * B] == e)
                    if tok.size:
                        groups.append((e, off, int(tok.size)))
                        src_all.append(tok + (i * B) % (256 - B))
                        dst_all.append(tok)
                        gw_all.append(gatew[i * B + tok, slot].astype(np.float32))
                        off += int(tok.size)
                plans.append((groups, torch.from_numpy(np.concatenate(src_all)).to(dev),
                              torch.from_numpy(np.concatenate(dst_all)).to(dev),
                              torch.from_numpy(np.concatenate(gw_all)).to(dev)))
            out = torch.zeros((B, N), dtype=torch.float32, device=dev)
            ybuf = torch.empty((2 * B, N), dtype=torch.float32, device=dev)  # top-2: two rows per token

            def expert(e, xg, y, sparse, fused, wsx):
                n = xg.shape[0]
                if sparse and fused:
                    scap.swiglu_block(Wgu[e], Wdn[e], xg, m_x, tau_x, bgu[e], 0.0, tau_z, None, gu_scale=sgu[e],
                                      down_scale=sdn[e], y=y, workspace=wsx)
                elif sparse:
                    scap.sparse_fc(Wgu[e], xg, m_x, tau_x, bgu[e], col_scale=sgu[e], y=ygu[:n], workspace=wsx)
                    scap.sparse_fc(Wdn[e], gate(ygu[:n]), 0.0, tau_z, None, col_scale=sdn[e], y=y, workspace=wsx)
                else:
                    scap.dense_fc(Wgu[e], xg, None, col_scale=sgu[e], y=ygu[:n], workspace=wsx)
                    scap.dense_fc(Wdn[e], gate(ygu[:n]), None, col_scale=sdn[e], y=y, workspace=wsx)

            def step(i, sparse, fused):
                groups, src, dst, gw = plans[i % nsteps]
                xg = X.index_select(0, src)
                for e, off, n in groups:
                    expert(e, xg[off:off + n], ybuf[off:off + n], sparse, fused, wsb if fused else ws)
                out.zero_()
                out.index_add_(0, dst, ybuf[:src.numel()] * gw[:, None])

            def step_streams(i):
                main = torch.cuda.current_stream()
                groups, src, dst, gw = plans[i % nsteps]
                xg = X.index_select(0, src)
                used = []
                for j, (e, off, n) in enumerate(groups):
                    k = j % n_side
                    if k not in used:
                        side[k].wait_stream(main)
                        used.append(k)
                    with torch.cuda.stream(side[k]):
                        expert(e, xg[off:off + n], ybuf[off:off + n], True, True, side_ws[k])
                for k in used:
                    main.wait_stream(side[k])
                out.zero_()
                out.index_add_(0, dst, ybuf[:src.numel()] * gw[:, None])

            saved = steps_box[0]
            steps_box[0] = nsteps
            t_dense = timed(lambda i: step(i, False, False))
            t_sep = timed(lambda i: step(i, True, False))
            t_fused = timed(lambda i: step(i, True, True))
            t_streams = timed(step_streams)
            steps_box[0] = saved
            active = float(np.mean([len(p[0]) for p in plans]))
            moe_rows.append({"tokens": B, "experts": E, "top_k": 2, "active_experts_per_step": round(active, 2),
                             "target_x": 0.4, "target_z": 0.7, "dense_us": round(t_dense, 1),
                             "sparse_separate_calls_us": round(t_sep, 1), "sparse_fused_blocks_us": round(t_fused, 1),
                             "sparse_fused_blocks_4_streams_us": round(t_streams, 1),
                             "vs_dense": round(t_dense / t_fused, 3)})

    if want("moe"):
        run_moe()
    torch.cuda.empty_cache()

    # Offline calibration at the paper's sample size (64 slices x 256 tokens per layer): wall time of the
    # synchronous call (one counting pass on the GPU, statistics on the host), median estimator + threshold.
    calib_rows = []
    for K in ((4096, 14336) if want("calibration") else ()):
        n = 16384
        Xc = torch.randn(n, K, device=dev).to(torch.bfloat16)
        wsc = scap.Workspace(K, 0, n)
        scap.calibrate(Xc, 0.5, scap.MODE_MEDIAN, workspace=wsc)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        reps = 5
        for _ in range(reps):
            scap.calibrate(Xc, 0.5, scap.MODE_MEDIAN, workspace=wsc)
        dt_ms = (time.perf_counter() - t0) / reps * 1e3
        calib_rows.append({"n_tokens": n, "K": K, "estimator": "median", "ms": round(dt_ms, 3),
                           "sample_GB": round(n * K * 2 / 1e9, 3),
                           "sample_GBps": round(n * K * 2 / dt_ms / 1e6, 1)})
        del Xc
        torch.cuda.empty_cache()

    layer3 = [r for r in rows if r["cfg"] == 3]
    summary = {"mistral_layer_fc_set_dense_us": round(sum(r["us"] for r in layer3 if r["target"] is None), 2),
               "mistral_layer_fc_set_s50_us": round(sum(r["us"] for r in layer3 if r["target"] == 0.5), 2)}
    print(json.dumps({"suite": rows, "blocks": blocks, "block_latency_vs_ffn_sparsity": grids, "moe": moe_rows, "calibration": calib_rows, "summary": summary, "steps_per_point": steps, "launch": "hipgraph",
                      "note": "GB/s = (rows read x N x sizeof(w) + x + bias + y) / time; density = union of the "
                              "batch's masks / K"}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--eager", action="store_true", help="time direct calls instead of a HIP graph replay")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-sweep", action="store_true", help="only the headline point")
    ap.add_argument("--no-summary", action="store_true",
                    help="skip the few points of the other configurations that the default run appends")
    ap.add_argument("--cfg", type=str, default="", help="launch shape waves,rows,unroll (tuning)")
    ap.add_argument("--only", type=str, default="",
                    help="with --suite: only the named part: layers, blocks, grid (fused-block latency against FFN "
                         "sparsity), moe or calibration")
    ap.add_argument("--suite", action="store_true",
                    help="time every benchmark configuration (layers of configs 1-5, batches, sparsities) instead "
                         "of the headline run")
    ap.add_argument("--batch", type=int, default=1,
                    help="tokens per call on the headline layer (default 1 = the headline workload; other values "
                         "time that batch alone, without the sweep and the CPU leg)")
    ap.add_argument("--target", type=float, default=0.5, help="target sparsity of the timed point: 0.5, 0.7 or 0.9")
    ap.add_argument("--counter-pass", action="store_true",
                    help="for rocprofv3 --pmc runs: a few eager launches of a copy of known size, the headline "
                         "sparse FC and the dense FC, then exit (no timing, no JSON)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch

    import paper_2412_07174_amd as scap
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    cfg = tuple(int(v) for v in args.cfg.split(",")) if args.cfg else None
    if args.suite:
        return run_suite(args, torch, scap, wl, dev)

    site = wl.sites(4)[1]  # mistral_down: 14336 -> 4096, bf16, SiLU(g)*u inputs
    K, N = site.K, site.N
    W_host = site.make_weights()
    X_host = site.test_vectors(64)
    calib_host = site.calib()

    def dev16(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(dev)

    W0 = dev16(W_host)
    wbytes_total = W0.numel() * 2
    R = max(2, -(-(1 << 30) // wbytes_total))
    Ws = [W0] + [W0.clone() for _ in range(R - 1)]
    X = dev16(X_host)
    calib = dev16(calib_host)
    B = args.batch
    if B < 1 or B > 16 or args.target not in site.targets:
        print(f"bench.py: --batch 1..16, --target one of {site.targets}", file=sys.stderr)
        return 2
    if B > 1 or args.target != 0.5:
        args.no_sweep = args.no_cpu = args.no_summary = True
    ws = scap.Workspace(K, N, B)
    ws_cal = scap.Workspace(K, 0, calib.shape[0])
    y = torch.empty((B, N), dtype=torch.float32, device=dev)
    nnz_buf = torch.zeros(64, dtype=torch.int32, device=dev)

    def xin(i):  # input of launch i: one test vector, or B consecutive ones
        if B == 1:
            return X[i % 64]
        j = (i * B) % (64 - B + 1)
        return X[j:j + B]

    # offline part through the library: (m, tau) per target, fused bias
    layer = {}
    for s in site.targets:
        m, tau = scap.calibrate(calib, s, scap.MODE_MEDIAN, workspace=ws_cal)
        bf = scap.fold_bias(W0, m, None, workspace=ws)
        layer[s] = (m, tau, bf)
    torch.cuda.synchronize()

    def measured_nnz(s):
        m, tau, bf = layer[s]
        for i in range(64):  # rows read per launch: the token's kept channels, or the union of the batch's
            if B == 1:
                scap.sparse_fc(Ws[0], xin(i), m, tau, bf, y=y, nnz_out=nnz_buf[i:i + 1], workspace=ws, cfg=cfg)
            else:
                scap.sparse_fc(Ws[0], xin(i), m, tau, bf, y=y, union_nnz_out=nnz_buf[i:i + 1], workspace=ws, cfg=cfg)
        torch.cuda.synchronize()
        return nnz_buf.cpu().numpy().astype(np.float64)

    def launcher(s, use_cfg="default"):
        c = cfg if use_cfg == "default" else use_cfg
        if s is None:
            return lambda i: scap.dense_fc(Ws[i % R], xin(i), None, y=y, workspace=ws, cfg=c)
        m, tau, bf = layer[s]
        return lambda i: scap.sparse_fc(Ws[i % R], xin(i), m, tau, bf, y=y, workspace=ws, cfg=c)

    if args.counter_pass:
        # reference for scaling the byte counters: torch copies W (reads and writes wbytes_total each)
        dst = torch.empty_like(W0)
        for i in range(10):
            dst.copy_(Ws[i % R])
        torch.cuda.synchronize()
        fn_s, fn_d = launcher(args.target), launcher(None)
        for i in range(50):
            fn_s(i)
        torch.cuda.synchronize()
        for i in range(20):
            fn_d(i)
        torch.cuda.synchronize()
        print(json.dumps({"counter_pass": True, "copy_bytes_each_way": wbytes_total,
                          "sparse_launches": 50, "dense_launches": 20}))
        return 0

    def time_steps(fn, steps, warmup):
        """Returns (wall ms per step, event ms per step) over exactly `steps` launches."""
        for i in range(warmup):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if args.eager:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            e0.record()
            for i in range(steps):
                fn(warmup + i)
            e1.record()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
        else:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):  # the binding launches on torch's current (capture) stream
                for i in range(steps):
                    fn(warmup + i)
            g.replay()  # untimed replay: uploads the graph
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            e0.record()
            g.replay()
            e1.record()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
        return (t1 - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps

    # ---- headline: 50 % target sparsity (or the point asked for)
    s_head = args.target
    nnz_head = measured_nnz(s_head)
    wall_ms, ev_ms = time_steps(launcher(s_head), args.steps, args.warmup)
    mean_nnz = float(nnz_head.mean())
    abytes = algorithmic_bytes(mean_nnz, K, N, B, 2)
    gbs = abytes / (ev_ms * 1e-3) / 1e9

    sweep = []
    read_ceiling = None
    if not args.no_sweep:
        sub_steps = max(200, args.steps // 4)
        for s in (None, 0.5, 0.7, 0.9):
            nn = float(K) if s is None else float(measured_nnz(s).mean())
            w_ms, e_ms = time_steps(launcher(s), sub_steps, 50)
            ab = algorithmic_bytes(nn, K, N, 1, 2)
            sweep.append({"target_sparsity": s, "density": round(nn / K, 4), "us": round(e_ms * 1e3, 3),
                          "GBps": round(ab / (e_ms * 1e-3) / 1e9, 1),
                          "frac_of_8TBps": round(ab / (e_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)})
            if B == 1 and not args.cfg:
                # the opt-in y += result mode (fp32 atomic adds instead of the split-K hand-over; the order of the
                # additions is not fixed): another operation than the headline's y = result, reported beside it
                y_keep = y.clone()
                w_ms, a_ms = time_steps(launcher(s, (0, 0, 0, 0, scap.CFG_ACCUMULATE)), sub_steps, 50)
                y.copy_(y_keep)
                sweep[-1]["accumulate_mode_us"] = round(a_ms * 1e3, 3)
                sweep[-1]["accumulate_mode_frac_of_8TBps"] = round(ab / (a_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
        # one launch on its own: event pair around a single eager launch of the headline call, GPU idle before
        fn = launcher(s_head)
        lat = []
        for i in range(60):
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn(i)
            e1.record()
            torch.cuda.synchronize()
            lat.append(e0.elapsed_time(e1) * 1e3)
        single_launch_us = round(float(np.median(lat[10:])), 2)
        # streaming-read ceiling of this machine: read the R weight copies once per launch
        chk = torch.zeros(2048, dtype=torch.int32, device=dev)
        w_ms, e_ms = time_steps(lambda i: scap.read_probe(Ws[i % R], chk), sub_steps, 50)
        read_ceiling = round(wbytes_total / (e_ms * 1e-3) / 1e9, 1)
        # latency vs density: t = t0 + rho * t1
        rho = np.array([r["density"] for r in sweep])
        tt = np.array([r["us"] for r in sweep])
        A = np.stack([np.ones_like(rho), rho], axis=1)
        coef, res, *_ = np.linalg.lstsq(A, tt, rcond=None)
        ss_tot = float(((tt - tt.mean()) ** 2).sum())
        r2 = 1.0 - float(((A @ coef - tt) ** 2).sum()) / ss_tot if ss_tot > 0 else 1.0
        fit = {"t0_us": round(float(coef[0]), 3), "t1_us": round(float(coef[1]), 3), "r2": round(r2, 5),
               "t0_over_dense": round(float(coef[0]) / sweep[0]["us"], 4)}
        # The machine's floor for one dependent launch, to read the fixed part against: the back-to-back period
        # of a kernel that does next to nothing (the 1-workgroup fill of a 4 KB workspace header), and of the
        # headline call with a threshold that keeps no channel (every phase of the kernel except the row stream).
        import ctypes
        lib = scap.load_library()
        tiny = torch.zeros(4096, dtype=torch.uint8, device=dev)

        def tiny_launch(i):
            lib.scap_workspace_init(ctypes.c_void_p(tiny.data_ptr()), 4096,
                                    ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))

        m, _, bf = layer[s_head]
        floor = {"empty_kernel_period_us": round(graph_timed(torch, tiny_launch, sub_steps), 3),
                 "nothing_kept_us": round(graph_timed(
                     torch, lambda i: scap.sparse_fc(Ws[i % R], xin(i), m, 3.0e38, bf, y=y, workspace=ws, cfg=cfg), sub_steps), 3)}
    else:
        fit = None
        single_launch_us = None
        floor = None

    # ---- CPU oracle on the host cores (baseline, not the target)
    cpu = None
    if not args.no_cpu:
        import oracle
        m, tau, bf = layer[s_head]
        bf_host = bf.cpu().numpy()
        cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
        cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
        n1, t0 = 0, time.perf_counter()
        while n1 < 64 and time.perf_counter() - t0 < 6.0:
            oracle.sparse_fc(W_host, X_host[n1], m, tau, bf_host, site.wdt, site.xdt, nthreads=1)
            n1 += 1
        us_1 = (time.perf_counter() - t0) / n1 * 1e6
        nm, t0 = 0, time.perf_counter()
        while nm < 256 and time.perf_counter() - t0 < 10.0:
            oracle.sparse_fc(W_host, X_host[nm % 64], m, tau, bf_host, site.wdt, site.xdt, nthreads=cores)
            nm += 1
        us_m = (time.perf_counter() - t0) / nm * 1e6
        model = "unknown"
        try:
            with open("/proc/cpuinfo") as f:
                for line in f:
                    if line.startswith("model name"):
                        model = line.split(":", 1)[1].strip()
                        break
        except OSError:
            pass
        cpu = {"value": round(us_m, 1), "unit": "us/token", "cores": cores, "kind": "oracle",
               "cpu_model": model, "nproc": os.cpu_count(),
               "sample": f"{nm} tokens of the headline workload, output columns split over {cores} threads; "
                         f"single thread: {round(us_1, 1)} us/token over {n1} tokens",
               "single_thread_us": round(us_1, 1)}

    workload = f"mistral7b_down_14336x4096_bf16_b{B}_s{int(round(s_head * 100))}"
    kernel = ("scap::gemv1_kernel<bf16>" if B == 1 else "scap::gemv_kernel<bf16>" if B == 2 else
              "scap::gemm_inline_raw_kernel<bf16> (matrix cores)")
    summary = None if args.no_summary else suite_summary(torch, scap, wl, dev)
    out = {
        "metric": "sparse_fc_us_per_token" if B == 1 else "sparse_fc_us_per_call",
        "value": round(wall_ms * 1e3, 3),
        "unit": "us/token" if B == 1 else f"us/call of {B} tokens",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16 storage, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": workload, "K": K, "N": N, "batch": B, "target_sparsity": s_head,
                   "measured_density": round(mean_nnz / K, 4), "weight_copies_rotated": R,
                   "launch": "eager" if args.eager else "hipgraph", "launch_cfg": args.cfg or "default"},
        "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": MEASURED_TRAFFIC.get(workload, (None, None))[0],
                     "traffic_source": MEASURED_TRAFFIC.get(workload, (None, None))[1],
                     "kernel": kernel, "us_per_launch": round(ev_ms * 1e3, 3),
                     "algorithmic_bytes_per_launch": int(abytes)},
        "cpu_baseline": cpu,
        "sweep": sweep,
        "read_ceiling_GBps": read_ceiling,
        "single_eager_launch_us": single_launch_us,
        "latency_vs_density_fit": fit,
        "launch_floor": floor,
        "suite_summary": summary,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
