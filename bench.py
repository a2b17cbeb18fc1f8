#!/usr/bin/env python3
"""Benchmark of the OMC hot path on one MI355X.

A "step" is one training iteration over the whole variable set: for every quantized weight
matrix decompress -> SGD update -> recompress (fused in one kernel), for every fp32 variable the
update alone, then the per-variable (s, b) finalize -- i.e. one omc_step_update_recompress call.
The workload is the Conformer-encoder-shaped set of about 115 M weight-matrix parameters
(17 blocks, d_model 512, FFN 2048, depthwise kernel 32, plus a front end), every weight matrix in
the 8-bit S1E4M3 code with the per-variable transformation, biases and norm vectors in fp32,
values N(0, 1/sqrt(fan_in)), gradients N(0, 1e-3), all seeded and synthetic and resident in HBM
before the timed region.

Prints one JSON line.  `value` is compressed-parameter GB/s (packed bytes of the quantized
variables stepped per second); `roofline` prices the dominant kernel's algorithmic HBM bytes
(6 B per 8-bit element: code in, gradient in, code out) against 8 TB/s; `cpu_baseline` is the CPU
oracle timed on a bounded sample of the same variable set on this machine's host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def build_workload(torch, omc, synth, blocks, d_model, ffn, seed=0):
    """Config-2 variable set, compressed on the GPU by the library itself."""
    import numpy as np
    specs = synth.conformer_varset(d_model, blocks, ffn, 32, frontend=True)
    mask = np.array([s.is_matrix for s in specs])
    gf = omc.fmt(4, 3)
    lay = synth.make_layout(specs, mask, lambda n: omc.omc_packed_bytes(gf, n))
    vals = synth.init_values(lay, seed)
    vals_d = torch.from_numpy(vals).cuda()
    arena = torch.zeros(lay.arena_bytes, dtype=torch.uint8, device="cuda")
    sb = torch.zeros((len(specs), 2), dtype=torch.float32, device="cuda")
    sb[:, 0] = 1.0
    table = [dict(data_offset=int(lay.data_offset[i]), aux_offset=int(lay.aux_offset[i]), n=s.n, fmt=gf,
                  quantized=bool(mask[i])) for i, s in enumerate(specs)]
    plan = omc.omc_plan_build(omc.make_var_table(table))
    ws = torch.empty(max(plan.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
    omc.omc_compress_set(vals_d, plan, arena, sb, ws)
    torch.cuda.synchronize()
    return dict(specs=specs, mask=mask, lay=lay, vals=vals, vals_d=vals_d, arena=arena, sb=sb, plan=plan, table=table)


def cpu_baseline(wl, synth, sample_blocks, iters, threads, gpu_after=None):
    """The oracle as it stands on a bounded sample: the variables of the first `sample_blocks`
    Conformer blocks, `iters` iterations.  Also returns the oracle's state for a parity check."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    from oracle import omc_oracle as orc
    specs, lay, mask = wl["specs"], wl["lay"], wl["mask"]
    of = orc.Format(4, 3)
    pick = [i for i, s in enumerate(specs)
            if s.name.startswith("block") and int(s.name.split("/")[0][5:]) < sample_blocks]
    sub_specs = [specs[i] for i in pick]
    sub_mask = mask[pick]
    sub_lay = synth.make_layout(sub_specs, sub_mask, lambda n: orc.packed_bytes(n, of.bits))
    arena = np.zeros(sub_lay.arena_bytes, np.uint8)
    sbt = np.zeros((len(pick), 2), np.float32)
    sbt[:, 0] = 1.0

    def init(j):
        i = pick[j]
        s = specs[i]
        a = int(lay.aux_offset[i])
        x = wl["vals"][a:a + s.n]
        d = int(sub_lay.data_offset[j])
        if sub_mask[j]:
            p, sb = orc.compress(x, of)
            arena[d:d + p.size] = p
            sbt[j] = sb
        else:
            arena[d:d + 4 * s.n] = x.view(np.uint8)

    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(init, range(len(pick))))
    table = orc.make_var_table(dict(data_offset=int(sub_lay.data_offset[j]), aux_offset=int(sub_lay.aux_offset[j]),
                                    n=specs[i].n, fmt=of, quantized=bool(sub_mask[j]))
                               for j, i in enumerate(pick))
    grads = []
    for gset in wl["grads_host"]:
        g = np.zeros(sub_lay.aux_elems, np.float32)
        for j, i in enumerate(pick):
            a, b = int(lay.aux_offset[i]), int(sub_lay.aux_offset[j])
            g[b:b + specs[i].n] = gset[a:a + specs[i].n]
        grads.append(g)
    n_elems = sum(specs[i].n for i in pick)
    packed_bytes = sum(orc.packed_bytes(specs[i].n, 8) for j, i in enumerate(pick) if sub_mask[j])
    first = None
    t0 = time.perf_counter()
    for t in range(iters):
        orc.step_varset(arena, table, sbt, grads[t % len(grads)], None, None,
                        orc.Opt(kind=0, lr=0.01, t=t + 1), threads=threads)
        if t == 0:
            first = (arena.copy(), sbt.copy())
    dt = (time.perf_counter() - t0) / iters
    return dict(pick=pick, sub_lay=sub_lay, sub_mask=sub_mask, first=first, sec_per_iter=dt,
                n_elems=n_elems, packed_bytes=packed_bytes)


LEG_WARMUP_S = 0.15


def warm(torch, fn, seconds=None):
    """Untimed calls for `seconds` of wall time: after host-side set-up the GPU runs at reduced clocks for
    the first tens of milliseconds, and a handful of warm-up calls measures that ramp instead of the kernel."""
    seconds = LEG_WARMUP_S if seconds is None else seconds
    t0 = time.perf_counter()
    k = 0
    while True:
        for _ in range(10):
            fn(k)
            k += 1
        torch.cuda.synchronize()
        if time.perf_counter() - t0 >= seconds:
            return k


def copy_ceiling(torch, n=1 << 28, iters=20):
    """GB/s of the runtime's own device-to-device copy of 1 GiB (2 GiB moved): the practical ceiling for a
    kernel that writes as much as it reads, measured in the same run."""
    src = torch.empty(n, device="cuda").normal_()
    dst = torch.empty_like(src)
    warm(torch, lambda k: dst.copy_(src))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    return 8.0 * n / (ms * 1e-3) / 1e9


def gemm_leg(torch, omc, synth, iters=20):
    """Forward-path dequant-fused GEMM (BASELINE config 5): bf16 activations [8192 x 1024] times S1E4M3
    weights [1024 x 4096], and [8192 x 4096] times [4096 x 1024]; fp32 accumulate and output."""
    import numpy as np
    gf = omc.fmt(4, 3)
    out = []
    for (M, N, K) in ((8192, 4096, 1024), (8192, 1024, 4096)):
        A = torch.from_numpy(synth.to_bf16_bits(synth.normal_f32(M * K, 1.0, 11)).view(np.int16)).cuda()
        W = torch.from_numpy(synth.normal_f32(K * N, 1.0 / np.sqrt(K), 12)).cuda()
        codes = torch.zeros(omc.omc_packed_bytes(gf, K * N), dtype=torch.uint8, device="cuda")
        sb = torch.zeros(2, device="cuda")
        wsc = torch.empty(omc.omc_compress_workspace_bytes(K * N), dtype=torch.uint8, device="cuda")
        omc.omc_compress(W, K * N, gf, True, codes, sb, wsc)
        C = torch.empty((M, N), dtype=torch.float32, device="cuda")
        ws = torch.empty(omc.omc_dequant_gemm_workspace_bytes(M), dtype=torch.uint8, device="cuda")
        warm(torch, lambda k: omc.omc_dequant_gemm(A, codes, gf, sb, C, M, N, K, ws))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            omc.omc_dequant_gemm(A, codes, gf, sb, C, M, N, K, ws)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        tf = 2.0 * M * N * K / (ms * 1e-3) / 1e12
        rec = {"M": M, "N": N, "K": K, "ms": ms, "TFLOPs": tf, "frac_of_bf16_mfma_peak": tf / 2500.0,
               "hbm_bytes": 2 * M * K + K * N + 4 * M * N}
        # the same product with the weights in the paper's 11-bit format (Table 1: S1E3M7), generic decode
        gf11 = omc.fmt(3, 7)
        codes11 = torch.zeros(omc.omc_packed_bytes(gf11, K * N), dtype=torch.uint8, device="cuda")
        sb11 = torch.zeros(2, device="cuda")
        omc.omc_compress(W, K * N, gf11, True, codes11, sb11, wsc)
        warm(torch, lambda k: omc.omc_dequant_gemm(A, codes11, gf11, sb11, C, M, N, K, ws))
        e0.record()
        for _ in range(iters):
            omc.omc_dequant_gemm(A, codes11, gf11, sb11, C, M, N, K, ws)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        rec["S1E3M7_ms"] = ms
        rec["S1E3M7_TFLOPs"] = 2.0 * M * N * K / (ms * 1e-3) / 1e12
        del codes11
        # the same layer's input gradient: dX[M, K] = dY[M, N] @ Wbar^T
        del C
        dY = torch.from_numpy(synth.to_bf16_bits(synth.normal_f32(M * N, 1.0, 13)).view(np.int16)).cuda()
        dX = torch.empty((M, K), dtype=torch.float32, device="cuda")
        warm(torch, lambda k: omc.omc_dequant_gemm_dx(dY, codes, gf, sb, dX, M, N, K, ws))
        e0.record()
        for _ in range(iters):
            omc.omc_dequant_gemm_dx(dY, codes, gf, sb, dX, M, N, K, ws)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        rec["dx_ms"] = ms
        rec["dx_TFLOPs"] = 2.0 * M * N * K / (ms * 1e-3) / 1e12
        # and its weight gradient dW[K, N] = X^T @ dY, consumed by the SGD update + recompression in the epilogue
        del dX
        wsd = torch.empty(omc.omc_dw_update_workspace_bytes(gf, M, N, K), dtype=torch.uint8, device="cuda")
        o = omc.opt(omc.OMC_SGD, 0.01)
        warm(torch, lambda k: omc.omc_dw_update_recompress(A, dY, codes, gf, sb, True, None, None, o, None, M, N, K, wsd))
        e0.record()
        for _ in range(iters):
            omc.omc_dw_update_recompress(A, dY, codes, gf, sb, True, None, None, o, None, M, N, K, wsd)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        rec["dw_update_ms"] = ms
        rec["dw_update_TFLOPs"] = 2.0 * M * N * K / (ms * 1e-3) / 1e12
        rec["dw_workspace_bytes"] = wsd.numel()   # fit partials + parked accumulators of the contraction splits
        out.append(rec)
    return out


def set_conversion_leg(torch, omc, wl, n_q, n_f, iters=20):
    """Whole-set conversions (start / end of a round): fp32 -> packed arena and back, one call each."""
    lay, plan = wl["lay"], wl["plan"]
    arena = torch.empty_like(wl["arena"])
    sb = torch.empty_like(wl["sb"])
    out = torch.empty(lay.aux_elems, device="cuda")
    ws = torch.empty(max(plan.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
    res = {}
    for name, fn, nbytes in (
            ("compress_set", lambda: omc.omc_compress_set(wl["vals_d"], plan, arena, sb, ws), 5.0 * n_q + 8.0 * n_f),
            ("decompress_set", lambda: omc.omc_decompress_set(arena, plan, sb, out), 5.0 * n_q + 8.0 * n_f)):
        warm(torch, lambda k: fn())
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        res[name] = {"ms": ms, "algorithmic_GBps": nbytes / (ms * 1e-3) / 1e9,
                     "frac_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    res["transport_bytes"] = plan.transport_bytes
    res["transport_over_fp32"] = plan.transport_bytes / (4.0 * (n_q + n_f))
    return res


def aggregate_leg(torch, omc, synth, blocks, R=8, iters=20):
    """Server side of a round: mean of R clients' copies of the set, each client with its own 90 %
    subset of the weight matrices in S1E4M3 and the rest in fp32."""
    import numpy as np
    specs = synth.conformer_varset(512, blocks, 2048, 32, frontend=True)
    gf = omc.fmt(4, 3)
    arenas, sbs, plans = [], [], []
    alg = 0.0
    vals_d = None
    for r in range(R):
        mask = synth.ppq_mask(specs, 0.9, 100 + r)
        lay = synth.make_layout(specs, mask, lambda n: omc.omc_packed_bytes(gf, n))
        table = [dict(data_offset=int(lay.data_offset[i]), aux_offset=int(lay.aux_offset[i]), n=s.n, fmt=gf,
                      quantized=bool(mask[i])) for i, s in enumerate(specs)]
        plan = omc.omc_plan_build(omc.make_var_table(table))
        if vals_d is None:
            vals_d = torch.from_numpy(synth.init_values(lay, 0)).cuda()
        client = vals_d + 1e-3 * torch.randn_like(vals_d)
        arena = torch.zeros(lay.arena_bytes, dtype=torch.uint8, device="cuda")
        sb = torch.zeros((len(specs), 2), device="cuda")
        ws = torch.empty(max(plan.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
        omc.omc_compress_set(client, plan, arena, sb, ws)
        arenas.append(arena); sbs.append(sb); plans.append(plan)
        alg += sum((1.0 if q else 4.0) * s.n for s, q in zip(specs, mask))
    n_total = sum(s.n for s in specs)
    alg += 4.0 * n_total
    agg = omc.omc_aggregate_plan_build(plans)
    out = torch.empty(vals_d.numel(), device="cuda")
    warm(torch, lambda k: omc.omc_aggregate_mean(agg, arenas, sbs, out))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        omc.omc_aggregate_mean(agg, arenas, sbs, out)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    return {"clients": R, "params": n_total, "ms": ms, "algorithmic_bytes": alg,
            "algorithmic_GBps": alg / (ms * 1e-3) / 1e9, "frac_hbm_peak": alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "fp32_clients_bytes": 4.0 * n_total * (R + 1)}


def formats_leg(torch, omc, synth, blocks, steps=20):
    """The fused decompress + SGD + recompress kernel on the same variable set for every storage
    format of the paper's tables (Tables 1-3: 19-, 13-, 11- and 6-bit), per-variable transformation on
    and, for the 11-bit format, off (the ablation's switch)."""
    import numpy as np
    specs = synth.conformer_varset(512, blocks, 2048, 32, frontend=True)
    mask = np.array([s.is_matrix for s in specs])
    n_q = int(sum(s.n for s, q in zip(specs, mask) if q))
    res = []
    vals_d = None
    for (E, M, pvt) in ((4, 14, True), (4, 8, True), (3, 9, True), (2, 10, True), (5, 7, True), (3, 7, True),
                        (3, 7, False), (2, 3, True)):
        gf = omc.fmt(E, M)
        B = 1 + E + M
        lay = synth.make_layout(specs, mask, lambda n: omc.omc_packed_bytes(gf, n))
        table = [dict(data_offset=int(lay.data_offset[i]), aux_offset=int(lay.aux_offset[i]), n=s.n, fmt=gf,
                      quantized=bool(mask[i]), use_pvt=pvt) for i, s in enumerate(specs)]
        plan = omc.omc_plan_build(omc.make_var_table(table))
        if vals_d is None:
            vals_d = torch.from_numpy(synth.init_values(lay, 0)).cuda()
            grads = [torch.from_numpy(synth.gradients(lay, 1e-3, 1000 + k)).cuda() for k in range(2)]
        arena = torch.zeros(lay.arena_bytes, dtype=torch.uint8, device="cuda")
        sb = torch.zeros((len(specs), 2), device="cuda")
        ws = torch.empty(max(plan.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
        omc.omc_compress_set(vals_d, plan, arena, sb, ws)
        o = omc.opt(omc.OMC_SGD, 0.01)
        nl = plan.launches
        ev = omc.HipEvents(2 * nl * steps)
        warm(torch, lambda k: omc.omc_step_update_recompress(arena, plan, sb, grads[k % 2], None, None, o, ws))
        for k in range(steps):
            omc.omc_step_update_recompress_events(arena, plan, sb, grads[k % 2], None, None, o, ws, ev, first=k * 2 * nl)
        torch.cuda.synchronize()
        ms = sum(ev.elapsed_ms(k * 2 * nl, k * 2 * nl + 1) for k in range(steps)) / steps
        alg = (2.0 * B / 8.0 + 4.0) * n_q
        res.append({"format": f"S1E{E}M{M}", "bits": B, "pvt": pvt, "kernel_ms": ms,
                    "algorithmic_GBps": alg / (ms * 1e-3) / 1e9, "frac_hbm_peak": alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS})
        del arena, sb, ws, plan
    return res


def other_configs_leg(torch, omc, synth, steps=10):
    """The other step configurations of the baseline at full size (they are parity-test cases first; timed here
    for reference): config 3 = the benchmark set with half of the matrices quantized in three formats (8, 11,
    16 bit) and Adam; config 4 = a 604 M-parameter set (24 blocks, d_model 1024, ffn 4096) in S1E3M7 with momentum."""
    import numpy as np
    res = []
    for name, dims, frac, choices, kind, lr in (
            ("config3: 17 blocks d=512, 50% of matrices quantized (S1E4M3 / S1E3M7 / S1E5M10), Adam",
             (512, 17, 2048, 32, True), 0.5, [(4, 3), (3, 7), (5, 10)], omc.OMC_ADAM, 1e-3),
            ("config4: 24 blocks d=1024 ffn=4096, all matrices S1E3M7, momentum 0.9",
             (1024, 24, 4096, 32, False), None, [(3, 7)], omc.OMC_MOMENTUM, 0.01)):
        specs = synth.conformer_varset(dims[0], dims[1], dims[2], dims[3], frontend=dims[4])
        mask = synth.ppq_mask(specs, frac, 3) if frac is not None else np.array([s.is_matrix for s in specs])
        fm = [choices[i % len(choices)] for i in range(len(specs))]
        gfs = [omc.fmt(*fm[i]) if mask[i] else None for i in range(len(specs))]
        sizes = iter([omc.omc_packed_bytes(gfs[i], specs[i].n) for i in range(len(specs)) if mask[i]])
        lay = synth.make_layout(specs, mask, lambda n: next(sizes))
        table = [dict(data_offset=int(lay.data_offset[i]), aux_offset=int(lay.aux_offset[i]), n=s.n, fmt=gfs[i],
                      quantized=bool(mask[i])) for i, s in enumerate(specs)]
        plan = omc.omc_plan_build(omc.make_var_table(table))
        gen = torch.Generator(device="cuda").manual_seed(5)
        vals = torch.empty(lay.aux_elems, device="cuda")
        for i, s in enumerate(specs):
            a = int(lay.aux_offset[i])
            vals[a:a + s.n].normal_(0.0, 1.0 / np.sqrt(s.fan_in) if s.is_matrix else 0.02, generator=gen)
        grads = [torch.empty(lay.aux_elems, device="cuda").normal_(0.0, 1e-3, generator=gen) for _ in range(2)]
        arena = torch.zeros(lay.arena_bytes, dtype=torch.uint8, device="cuda")
        sb = torch.zeros((len(specs), 2), device="cuda")
        ws = torch.empty(max(plan.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
        omc.omc_compress_set(vals, plan, arena, sb, ws)
        del vals
        m = torch.zeros(lay.aux_elems, device="cuda")
        v = torch.zeros(lay.aux_elems, device="cuda") if kind == omc.OMC_ADAM else None
        state = 8.0 if kind == omc.OMC_MOMENTUM else 16.0
        alg = sum((2.0 * (1 + sum(fm[i])) / 8.0 + 4.0 + state) * s.n if mask[i] else (12.0 + state) * s.n
                  for i, s in enumerate(specs))
        packed = sum(omc.omc_packed_bytes(gfs[i], s.n) for i, s in enumerate(specs) if mask[i])
        t = warm(torch, lambda k: omc.omc_step_update_recompress(arena, plan, sb, grads[k % 2], m, v, omc.opt(kind, lr, t=k + 1), ws))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for k in range(steps):
            omc.omc_step_update_recompress(arena, plan, sb, grads[k % 2], m, v, omc.opt(kind, lr, t=t + k + 1), ws)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        nl = plan.launches
        ev = omc.HipEvents(2 * nl * steps)
        for k in range(steps):
            omc.omc_step_update_recompress_events(arena, plan, sb, grads[k % 2], m, v, omc.opt(kind, lr, t=t + steps + k + 1), ws, ev,
                                                  first=k * 2 * nl)
        torch.cuda.synchronize()
        kms = [sum(ev.elapsed_ms(k * 2 * nl + 2 * j, k * 2 * nl + 2 * j + 1) for k in range(steps)) / steps for j in range(nl)]
        res.append({"workload": name, "params": int(sum(s.n for s in specs)), "launches_per_step": plan.launches,
                    "ms_per_step": ms, "kernel_ms": kms, "algorithmic_GBps": alg / (ms * 1e-3) / 1e9,
                    "frac_hbm_peak": alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                    "compressed_param_GBps": packed / (ms * 1e-3) / 1e9})
        del arena, sb, ws, m, v, grads, plan
        torch.cuda.empty_cache()
    return res


def main():
    global LEG_WARMUP_S
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--blocks", type=int, default=17, help="Conformer blocks (17 = the benchmark workload)")
    ap.add_argument("--cpu-sample-blocks", type=int, default=4)
    ap.add_argument("--cpu-iters", type=int, default=6)
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle leg (for profiler runs)")
    ap.add_argument("--leg-warmup-s", type=float, default=LEG_WARMUP_S, help="untimed wall time before each extra leg's measurement (profiler runs shorten it)")
    ap.add_argument("--step-only", action="store_true", help="skip the extra legs (set conversions, aggregation, formats, "
                                                             "other configurations, matrix-core kernels); for profiler runs")
    ap.add_argument("--eager", action="store_true", help="(default) one library call per step")
    ap.add_argument("--clock-warmup-s", type=float, default=0.5,
                    help="seconds of untimed steps before any measurement, so that the GPU clocks have ramped up")
    ap.add_argument("--graph", action="store_true",
                    help="time HIP graph replays of two captured steps instead (checked against eager launches first); "
                         "measured: no faster than eager launches on this machine")
    ap.add_argument("--gemm-only", action="store_true", help="only the forward GEMM leg (for profiler runs)")
    ap.add_argument("--aggregate-only", action="store_true", help="only the server aggregation leg")
    ap.add_argument("--configs-only", action="store_true", help="only the leg over the baseline's other step configurations")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device-to-device copy of known size (1 GiB read + 1 GiB written "
                         "per launch) to calibrate profiler byte counters and show the copy ceiling")
    args = ap.parse_args()
    LEG_WARMUP_S = args.leg_warmup_s
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU; --gpus must be 1 "
                 "(no collectives or sharding exist in this library)")

    import numpy as np
    import torch
    from paper_2205_03494_amd import omc, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        n = 1 << 28                                   # 2^28 floats = 1 GiB
        src = torch.randn(n, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 20
        print(json.dumps({"copy_kernel": "torch Tensor.copy_ fp32", "bytes_read": 4 * n, "bytes_written": 4 * n,
                          "ms": ms, "GBps": 8 * n / (ms * 1e-3) / 1e9}))
        return
    if args.gemm_only:
        print(json.dumps({"gemm": gemm_leg(torch, omc, synth)}))
        return
    if args.configs_only:
        print(json.dumps({"other_step_configs": other_configs_leg(torch, omc, synth)}))
        return
    if args.aggregate_only:
        print(json.dumps({"server_aggregation": aggregate_leg(torch, omc, synth, args.blocks)}))
        return
    wl = build_workload(torch, omc, synth, args.blocks, 512, 2048)
    specs, mask, lay, plan = wl["specs"], wl["mask"], wl["lay"], wl["plan"]
    # a ring of two pre-generated gradient sets, resident in HBM
    wl["grads_host"] = [synth.gradients(lay, 1e-3, 1000 + k) for k in range(2)]
    grads = [torch.from_numpy(g).cuda() for g in wl["grads_host"]]
    ws = torch.empty(max(plan.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
    o = omc.opt(omc.OMC_SGD, 0.01)
    arena, sb = wl["arena"], wl["sb"]
    arena0, sb0 = arena.clone(), sb.clone()

    n_q = int(sum(s.n for s, q in zip(specs, mask) if q))
    n_f = int(sum(s.n for s, q in zip(specs, mask) if not q))
    packed_bytes = int(sum(omc.omc_packed_bytes(omc.fmt(4, 3), s.n) for s, q in zip(specs, mask) if q))
    alg_bytes_q = 6.0 * n_q            # per element: 1 B code in + 4 B gradient in + 1 B code out
    alg_bytes_step = alg_bytes_q + 12.0 * n_f + 8.0 * int(mask.sum())

    def step(k):
        omc.omc_step_update_recompress(arena, plan, sb, grads[k % 2], None, None, o, ws)

    # ---- parity spot check + CPU baseline (oracle) on a bounded sample ------------------------
    cpu = None
    parity = None
    if not args.no_cpu:
        threads = min(16, os.cpu_count() or 1)
        cpu = cpu_baseline(wl, synth, min(args.cpu_sample_blocks, args.blocks), args.cpu_iters, threads)
        step(0)
        torch.cuda.synchronize()
        ga, gs = arena.cpu().numpy(), sb.cpu().numpy()
        oa, osb = cpu["first"]
        parity = True
        for j, i in enumerate(cpu["pick"]):
            d, e = int(lay.data_offset[i]), int(cpu["sub_lay"].data_offset[j])
            nb = omc.omc_packed_bytes(omc.fmt(4, 3), specs[i].n) if mask[i] else 4 * specs[i].n
            parity &= bool(np.array_equal(ga[d:d + nb], oa[e:e + nb]))
            if mask[i]:
                parity &= bool(np.array_equal(gs[i], osb[j]))
        arena.copy_(arena0)
        sb.copy_(sb0)

    # ---- the step as a HIP graph: two steps (one per gradient buffer) captured once, replayed ----------
    # The library only enqueues kernels on the caller's stream, so a caller can capture it; replaying
    # removes the launch gaps between the fused kernel and the finalize.  Checked here against eager
    # launches on the same state, over several replays, before it is used for the timed region.
    graph = None
    if args.graph:
        cap = torch.cuda.Stream()
        cap.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=cap):
            omc.omc_step_update_recompress(arena, plan, sb, grads[0], None, None, o, ws, stream=cap)
            omc.omc_step_update_recompress(arena, plan, sb, grads[1], None, None, o, ws, stream=cap)
        torch.cuda.synchronize()
        arena.copy_(arena0)
        sb.copy_(sb0)
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        ga, gs = arena.clone(), sb.clone()
        arena.copy_(arena0)
        sb.copy_(sb0)
        for k in range(6):
            step(k)
        torch.cuda.synchronize()
        assert torch.equal(ga, arena) and torch.equal(gs.view(torch.int32), sb.view(torch.int32)), \
            "graph replay and eager launches disagree"
        arena.copy_(arena0)
        sb.copy_(sb0)

    def run_steps(n, first=0):
        k = first
        if graph is not None:
            if k % 2 == 1 and n > 0:
                step(k); k += 1; n -= 1
            for _ in range(n // 2):
                graph.replay()
            k += 2 * (n // 2)
            if n % 2:
                step(k)
        else:
            for j in range(n):
                step(k + j)

    # ---- bring the GPU to its steady clocks: after idling (host-side set-up, the oracle leg) the first tens of
    # milliseconds of kernels run at reduced clocks (measured: the same kernel 232 us -> 109 us), which
    # W = 5 warm-up steps of 0.1 ms do not cover.  Untimed; the state is restored afterwards.
    t_warm = time.perf_counter()
    k = 0
    while time.perf_counter() - t_warm < args.clock_warmup_s:
        for _ in range(50):
            step(k)
            k += 1
        torch.cuda.synchronize()
    arena.copy_(arena0)
    sb.copy_(sb0)

    # ---- per-kernel durations: the steps with an event pair around every launch ------
    nl = plan.launches
    ev = omc.HipEvents(2 * nl * args.steps)
    for k in range(args.steps):
        omc.omc_step_update_recompress_events(arena, plan, sb, grads[k % 2], None, None, o, ws, ev,
                                              first=k * 2 * nl)
    torch.cuda.synchronize()
    kern_ms = [0.0] * nl
    for k in range(args.steps):
        for j in range(nl):
            kern_ms[j] += ev.elapsed_ms(k * 2 * nl + 2 * j, k * 2 * nl + 2 * j + 1)
    kern_ms = [x / args.steps for x in kern_ms]
    arena.copy_(arena0)
    sb.copy_(sb0)
    # ---- the same kernel when the packed codes do not come back from the memory-side cache: between two
    # steps of a training loop lies a forward and a backward pass, which leaves nothing of the codes in the
    # 256 MB Infinity Cache, while back-to-back steps find all 115 MB of them there.  A 512 MiB device copy
    # between the steps (1 GiB of traffic) stands in for that pass; only the step kernel is timed.
    cold_ms = None
    if not args.step_only:
        nc = min(args.steps, 30)
        fl_src = torch.empty(1 << 27, device="cuda")
        fl_dst = torch.empty_like(fl_src)
        cold_ms = {}
        for name, flags in (("default", 0), ("OMC_OPT_STREAM_CODES", omc.OMC_OPT_STREAM_CODES)):
            oc = omc.opt(omc.OMC_SGD, 0.01, flags=flags)
            ev2 = omc.HipEvents(2 * nl * nc)
            for k in range(nc):
                fl_dst.copy_(fl_src)
                omc.omc_step_update_recompress_events(arena, plan, sb, grads[k % 2], None, None, oc, ws, ev2, first=k * 2 * nl)
            torch.cuda.synchronize()
            cold_ms[name] = sum(ev2.elapsed_ms(k * 2 * nl, k * 2 * nl + 1) for k in range(nc)) / nc
            arena.copy_(arena0)
            sb.copy_(sb0)
        del fl_src, fl_dst
    # ---- timed region: whole steps ---------------------------------------------------------------
    run_steps(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(args.steps, first=args.warmup)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / args.steps

    dom_ms = kern_ms[0]                                     # launch 0: the 8-bit fused step kernel
    achieved = alg_bytes_q / (dom_ms * 1e-3) / 1e9
    # HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on this same command and
    # scaled by a plain copy's reading (summary and commands: profiles/step_kernel_sgd8_conformer115m.md)
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "step_kernel_sgd8_traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as fh:
            tj = json.load(fh)
        if tj.get("n_quantized_params") == n_q:
            traffic = tj["fetch_bytes_per_launch"] + tj["write_bytes_per_launch"]

    out = {
        "metric": "compressed-param GB/s per decompress+update+recompress step; % HBM peak",
        "value": packed_bytes / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"conformer-encoder-shaped set, {args.blocks} blocks d_model=512 ffn=2048 conv_k=32 "
                               f"+ front end, {n_q} weight-matrix params in S1E4M3 (8-bit) with per-variable "
                               f"transformation, {n_f} fp32 bias/norm params, SGD lr=0.01, grads N(0,1e-3)",
                   "n_quantized_params": n_q, "n_fp32_params": n_f, "n_variables": len(specs),
                   "packed_bytes": packed_bytes, "algorithmic_bytes_per_step": alg_bytes_step,
                   "step_GBps_algorithmic": alg_bytes_step / (ms_per_step * 1e-3) / 1e9,
                   "Gparam_per_s": (n_q + n_f) / (ms_per_step * 1e-3) / 1e9,
                   "launch": "one library call per step" if graph is None else
                             "HIP graph of two steps (one per gradient buffer), replayed; checked against eager launches",

                   "kernel_ms": {"step_kernel<8,sgd> (fp32 variables ride along)": kern_ms[0],
                                 "tail_kernel": kern_ms[1] if nl > 2 else None,
                                 "finalize_plan_kernel": kern_ms[-1]},
                   "parity_vs_oracle_on_sample": parity},
        "roofline": {"bound": "hbm", "kernel": "step_kernel<8,sgd>", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "algorithmic_bytes_per_launch": alg_bytes_q, "traffic": traffic},
    }
    if cold_ms is not None:     # the dominant kernel with the codes evicted from the memory-side cache between steps
        out["roofline"]["codes_evicted_between_steps"] = {
            "how": "a 512 MiB device-to-device copy between steps; only the step kernel is timed",
            **{name: {"kernel_ms": ms, "achieved": alg_bytes_q / (ms * 1e-3) / 1e9,
                      "frac": alg_bytes_q / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS} for name, ms in cold_ms.items()}}
    del grads, arena0
    torch.cuda.empty_cache()
    if not args.step_only:
        ceil = copy_ceiling(torch)
        out["roofline"]["copy_kernel_GBps"] = ceil        # device-to-device copy of 1 GiB in this run
        out["roofline"]["frac_of_copy_kernel"] = out["roofline"]["achieved"] / ceil
        out["set_conversions"] = set_conversion_leg(torch, omc, wl, n_q, n_f)
        del wl
        torch.cuda.empty_cache()
        out["server_aggregation"] = aggregate_leg(torch, omc, synth, args.blocks)
        torch.cuda.empty_cache()
        out["paper_formats_sgd"] = formats_leg(torch, omc, synth, args.blocks)
        torch.cuda.empty_cache()
        out["other_step_configs"] = other_configs_leg(torch, omc, synth)
        out["forward_gemm"] = gemm_leg(torch, omc, synth)
    if cpu is not None:
        out["cpu_baseline"] = {
            "value": cpu["packed_bytes"] / cpu["sec_per_iter"] / 1e9, "unit": "GB/s",
            "cores": min(16, os.cpu_count() or 1), "kind": "oracle",
            "sample": f"first {min(args.cpu_sample_blocks, args.blocks)} Conformer blocks of the same set "
                      f"({cpu['n_elems']} params), {args.cpu_iters} iterations, "
                      f"{1e3 * cpu['sec_per_iter']:.0f} ms per iteration on {min(16, os.cpu_count() or 1)} threads "
                      f"({args.cpu_iters * cpu['sec_per_iter'] * min(16, os.cpu_count() or 1):.0f} core-seconds)",
        }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
