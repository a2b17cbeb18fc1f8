#!/usr/bin/env python3
"""Benchmark of the OMC hot path on one MI355X.

A "step" is one training iteration over a whole variable set: for every quantized weight matrix
decompress -> parameter update -> recompress (fused in one kernel per code width), for every fp32
variable the update alone, then the per-variable (s, b) finalize -- one omc_step_update_recompress
call with default flags.

Headline workload (the largest single-GPU configuration of the baseline): a Conformer-encoder-shaped
set of about 604 M weight-matrix parameters (24 blocks, d_model 1024, FFN 4096, 16 heads, depthwise
kernel 32), every weight matrix in the 11-bit S1E3M7 code with the per-variable transformation,
biases and norm vectors in fp32, SGD with momentum 0.9 and fp32 momentum, values
N(0, 1/sqrt(fan_in)), gradients N(0, 1e-3); all seeded, synthetic and resident in HBM before the
timed region.  The baseline's other step configurations (the 115 M-parameter set in S1E4M3 under SGD;
the same set half quantized in three formats under Adam) are measured the same way and reported
under `other_step_configs`, each with its own roofline block.

Prints one JSON line.  `value` is compressed-parameter GB/s (packed bytes of the quantized variables
stepped per second, whole step, back-to-back steps as the contract asks).  Every `roofline` block prices
its configuration's dominant kernel: algorithmic HBM bytes of one launch over that launch's duration
(HIP events on the launch stream) against 8 TB/s.  A training loop runs a forward and a backward pass
between two steps, so `achieved` / `frac` are taken with the caches flushed between steps (a 512 MiB
device copy, untimed); the back-to-back figure and the opt-in OMC_OPT_KEEP_CODES policy are listed
beside it.  `cpu_baseline` is the CPU oracle timed on a bounded sample of the headline set on this
machine's host cores, one thread and all cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
LEG_WARMUP_S = 0.15

STEP_CONFIGS = {
    # name: (d_model, blocks, ffn, conv_k, front end), quantized fraction of the matrices (None = all), formats, optimizer, lr, text
    "config4": dict(dims=(1024, 24, 4096, 32, False), frac=None, formats=[(3, 7)], kind="momentum", lr=0.01,
                    text="conformer-encoder-shaped set, 24 blocks d_model=1024 ffn=4096 conv_k=32, all weight matrices in "
                         "S1E3M7 (11-bit) with per-variable transformation, bias/norm vectors fp32, momentum 0.9 lr=0.01 "
                         "(fp32 momentum), grads N(0,1e-3)"),
    "config2": dict(dims=(512, 17, 2048, 32, True), frac=None, formats=[(4, 3)], kind="sgd", lr=0.01,
                    text="conformer-encoder-shaped set, 17 blocks d_model=512 ffn=2048 conv_k=32 + front end, all weight "
                         "matrices in S1E4M3 (8-bit) with per-variable transformation, bias/norm vectors fp32, SGD lr=0.01, "
                         "grads N(0,1e-3)"),
    "config3": dict(dims=(512, 17, 2048, 32, True), frac=0.5, formats=[(4, 3), (3, 7), (5, 10)], kind="adam", lr=1e-3,
                    text="the 17-block set with a seeded 50 % of the weight matrices quantized (S1E4M3 / S1E3M7 / S1E5M10 in "
                         "turn) and the rest fp32 in the same arena, Adam(0.9, 0.999) lr=1e-3 with fp32 moments"),
}
STATE_BYTES = {"sgd": 0.0, "momentum": 8.0, "adam": 16.0}     # optimizer state read + written per element


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


def timed(torch, fn, iters):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for k in range(iters):
        fn(k)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


# ------------------------------------------------------------------------------------------------
# step configurations
# ------------------------------------------------------------------------------------------------
def build_step_workload(torch, omc, synth, name, blocks=None, seed=5):
    """Variable set of one baseline configuration, values drawn on the GPU from a seeded generator and
    compressed by the library itself."""
    import numpy as np
    cfg = STEP_CONFIGS[name]
    d, nb, ffn, ck, fe = cfg["dims"]
    nb = nb if blocks is None else blocks
    specs = synth.conformer_varset(d, nb, ffn, ck, frontend=fe)
    mask = synth.ppq_mask(specs, cfg["frac"], 3) if cfg["frac"] is not None else np.array([s.is_matrix for s in specs])
    fm = [cfg["formats"][i % len(cfg["formats"])] for i in range(len(specs))]
    gfs = [omc.fmt(*fm[i]) if mask[i] else None for i in range(len(specs))]
    sizes = iter([omc.omc_packed_bytes(gfs[i], specs[i].n) for i in range(len(specs)) if mask[i]])
    lay = synth.make_layout(specs, mask, lambda n: next(sizes))
    table = [dict(data_offset=int(lay.data_offset[i]), aux_offset=int(lay.aux_offset[i]), n=s.n, fmt=gfs[i],
                  quantized=bool(mask[i])) for i, s in enumerate(specs)]
    plan = omc.omc_plan_build(omc.make_var_table(table))
    gen = torch.Generator(device="cuda").manual_seed(seed)
    vals = torch.empty(lay.aux_elems, device="cuda")
    for i, s in enumerate(specs):
        a = int(lay.aux_offset[i])
        vals[a:a + s.n].normal_(0.0, 1.0 / np.sqrt(s.fan_in) if s.is_matrix else 0.02, generator=gen)
    grads = [torch.empty(lay.aux_elems, device="cuda").normal_(0.0, 1e-3, generator=gen) for _ in range(2)]
    arena = torch.zeros(lay.arena_bytes, dtype=torch.uint8, device="cuda")
    sb = torch.zeros((len(specs), 2), device="cuda")
    ws = torch.empty(max(plan.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
    omc.omc_compress_set(vals, plan, arena, sb, ws)
    torch.cuda.synchronize()
    kind = cfg["kind"]
    m = torch.zeros(lay.aux_elems, device="cuda") if kind != "sgd" else None
    v = torch.zeros(lay.aux_elems, device="cuda") if kind == "adam" else None
    okind = {"sgd": omc.OMC_SGD, "momentum": omc.OMC_MOMENTUM, "adam": omc.OMC_ADAM}[kind]
    # launches of a step, in the library's order: one fused kernel per code width (ascending; none of these sets has
    # ragged tails or needs a second rounding variant), the first of them also serving the fp32 variables; the finalize
    widths = sorted({1 + sum(fm[i]) for i in range(len(specs)) if mask[i]})
    assert all(s.n % 2048 == 0 for s, q in zip(specs, mask) if q)
    assert plan.launches == len(widths) + 1, (plan.launches, widths)
    st = STATE_BYTES[kind]
    n_f = int(sum(s.n for s, q in zip(specs, mask) if not q))
    launches = []
    for j, B in enumerate(widths):
        n_b = int(sum(s.n for i, s in enumerate(specs) if mask[i] and 1 + sum(fm[i]) == B))
        alg = (2.0 * B / 8.0 + 4.0 + st) * n_b + ((12.0 + st) * n_f if j == 0 else 0.0)
        launches.append({"kernel": f"step_kernel<{B} bit,{kind}>" + (" + fp32 variables" if j == 0 and n_f else ""),
                         "elements": n_b + (n_f if j == 0 else 0), "algorithmic_bytes": alg})
    n_q = int(sum(s.n for s, q in zip(specs, mask) if q))
    packed = int(sum(omc.omc_packed_bytes(gfs[i], s.n) for i, s in enumerate(specs) if mask[i]))
    alg_step = sum(l["algorithmic_bytes"] for l in launches) + 8.0 * int(mask.sum())
    return dict(name=name, cfg=cfg, specs=specs, mask=mask, fm=fm, gfs=gfs, lay=lay, plan=plan, vals=vals, grads=grads,
                arena=arena, sb=sb, ws=ws, m=m, v=v, okind=okind, launches=launches, n_q=n_q, n_f=n_f, packed=packed,
                alg_step=alg_step, t=0)


def step_fn(omc, wl, flags=0):
    def step(k):
        wl["t"] += 1
        omc.omc_step_update_recompress(wl["arena"], wl["plan"], wl["sb"], wl["grads"][k % 2], wl["m"], wl["v"],
                                       omc.opt(wl["okind"], wl["cfg"]["lr"], t=wl["t"], flags=flags), wl["ws"])
    return step


def kernel_times(torch, omc, wl, steps, flags=0, flush=None):
    """Average duration of every launch of a step (HIP events recorded by the library on the launch stream around
    each launch).  flush: (src, dst) of a device copy enqueued before every step, untimed, which leaves nothing of
    the set in the caches."""
    nl = wl["plan"].launches
    ev = omc.HipEvents(2 * nl * steps)
    for k in range(steps):
        if flush is not None:
            flush[1].copy_(flush[0])
        wl["t"] += 1
        omc.omc_step_update_recompress_events(wl["arena"], wl["plan"], wl["sb"], wl["grads"][k % 2], wl["m"], wl["v"],
                                              omc.opt(wl["okind"], wl["cfg"]["lr"], t=wl["t"], flags=flags), wl["ws"], ev,
                                              first=k * 2 * nl)
    torch.cuda.synchronize()
    return [sum(ev.elapsed_ms(k * 2 * nl + 2 * j, k * 2 * nl + 2 * j + 1) for k in range(steps)) / steps
            for j in range(nl)]


def roofline_block(wl, regimes):
    """regimes: {"evicted": ms list, "back_to_back": ms list, "keep_codes": ms list}.  The dominant kernel is the
    launch that takes longest in the evicted regime."""
    ev = regimes["evicted"]
    dom = max(range(len(wl["launches"])), key=lambda j: ev[j])
    L = wl["launches"][dom]

    def rate(ms):
        return L["algorithmic_bytes"] / (ms * 1e-3) / 1e9
    blk = {"bound": "hbm", "kernel": L["kernel"], "achieved": rate(ev[dom]), "peak": HBM_PEAK_GBS, "unit": "GB/s",
           "frac": rate(ev[dom]) / HBM_PEAK_GBS, "traffic": None,
           "regime": "caches flushed between steps (512 MiB device copy before every step, untimed): the state a "
                     "training loop's forward and backward pass leave; default flags",
           "kernel_ms": ev[dom], "algorithmic_bytes_per_launch": L["algorithmic_bytes"],
           "elements_per_launch": L["elements"],
           "back_to_back_steps": {"kernel_ms": regimes["back_to_back"][dom], "achieved": rate(regimes["back_to_back"][dom]),
                                  "frac": rate(regimes["back_to_back"][dom]) / HBM_PEAK_GBS},
           "back_to_back_steps_OMC_OPT_KEEP_CODES": {
               "kernel_ms": regimes["keep_codes"][dom], "achieved": rate(regimes["keep_codes"][dom]),
               "frac": rate(regimes["keep_codes"][dom]) / HBM_PEAK_GBS,
               "note": "opt-in: packed codes come back from the 256 MB memory-side cache; not an HBM figure"},
           "all_launches_ms_evicted": ev, "all_launches_ms_back_to_back": regimes["back_to_back"]}
    # HBM bytes of the same launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, if a committed profile of exactly this
    # kernel and workload exists: not a reading of this run, so it is labelled with its source and `traffic` stays null
    tpath = os.path.join(ROOT, "profiles", f"step_kernel_{wl['name']}_traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as fh:
            tj = json.load(fh)
        if tj.get("elements_per_launch") == L["elements"]:
            blk["traffic_from_profile"] = {"bytes": tj["fetch_bytes_per_launch"] + tj["write_bytes_per_launch"],
                                           "fetch_bytes": tj["fetch_bytes_per_launch"],
                                           "write_bytes": tj["write_bytes_per_launch"], "source": tj.get("source")}
    return blk


def measure_step_config(torch, omc, wl, steps, warmup, clock_warmup_s, flush, regimes=True):
    """Times whole steps (back to back, default flags) and the launches of a step in three regimes."""
    step = step_fn(omc, wl)
    arena0, sb0 = wl["arena"].clone(), wl["sb"].clone()

    def restore():
        wl["arena"].copy_(arena0)
        wl["sb"].copy_(sb0)
        if wl["m"] is not None:
            wl["m"].zero_()
        if wl["v"] is not None:
            wl["v"].zero_()
        wl["t"] = 0
    warm(torch, step, clock_warmup_s)
    restore()
    reg = None
    if regimes:
        nk = min(steps, 20)
        reg = {"back_to_back": kernel_times(torch, omc, wl, nk)}
        restore()
        reg["evicted"] = kernel_times(torch, omc, wl, nk, flush=flush)
        restore()
        warm(torch, step_fn(omc, wl, omc.OMC_OPT_KEEP_CODES), LEG_WARMUP_S)
        reg["keep_codes"] = kernel_times(torch, omc, wl, nk, flags=omc.OMC_OPT_KEEP_CODES)
        restore()
    # ---- timed region: W warm-up steps, then exactly K steps between two synchronisations --------------------
    for k in range(warmup):
        step(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        step(warmup + k)
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - t0) / steps
    restore()
    return ms, reg


def describe(wl, ms):
    return {"workload": wl["cfg"]["text"], "n_quantized_params": wl["n_q"], "n_fp32_params": wl["n_f"],
            "n_variables": len(wl["specs"]), "packed_bytes": wl["packed"], "launches_per_step": wl["plan"].launches,
            "algorithmic_bytes_per_step": wl["alg_step"],
            "step_GBps_algorithmic": wl["alg_step"] / (ms * 1e-3) / 1e9,
            "step_frac_hbm_peak": wl["alg_step"] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "Gparam_per_s": (wl["n_q"] + wl["n_f"]) / (ms * 1e-3) / 1e9}


# ------------------------------------------------------------------------------------------------
# CPU baseline: the oracle on a bounded sample of the headline set
# ------------------------------------------------------------------------------------------------
def cpu_baseline(torch, omc, synth, wl, sample_blocks, iters):
    """The oracle as it stands on the variables of the first `sample_blocks` Conformer blocks of the workload (their
    values and gradients downloaded from the GPU), one thread and all cores, `iters` iterations each.  Returns the
    timings and whether the GPU's first step on those variables equals the oracle's, bit for bit."""
    import numpy as np
    from oracle import omc_oracle as orc
    specs, lay, mask, fm = wl["specs"], wl["lay"], wl["mask"], wl["fm"]
    pick = [i for i, s in enumerate(specs)
            if s.name.startswith("block") and int(s.name.split("/")[0][5:]) < sample_blocks]
    ofs = [orc.Format(*fm[i]) if mask[i] else None for i in pick]
    sizes = iter([orc.packed_bytes(specs[i].n, ofs[j].bits) for j, i in enumerate(pick) if mask[i]])
    sub_mask = mask[pick]
    sub_lay = synth.make_layout([specs[i] for i in pick], sub_mask, lambda n: next(sizes))
    arena = np.zeros(sub_lay.arena_bytes, np.uint8)
    sbt = np.zeros((len(pick), 2), np.float32)
    sbt[:, 0] = 1.0
    grads = [np.zeros(sub_lay.aux_elems, np.float32) for _ in wl["grads"]]
    for j, i in enumerate(pick):
        s, a, b, d = specs[i], int(lay.aux_offset[i]), int(sub_lay.aux_offset[j]), int(sub_lay.data_offset[j])
        x = wl["vals"][a:a + s.n].cpu().numpy()
        for g_host, g_dev in zip(grads, wl["grads"]):
            g_host[b:b + s.n] = g_dev[a:a + s.n].cpu().numpy()
        if sub_mask[j]:
            p, sb = orc.compress(x, ofs[j])
            arena[d:d + p.size] = p
            sbt[j] = sb
        else:
            arena[d:d + 4 * s.n] = x.view(np.uint8)
    table = orc.make_var_table(dict(data_offset=int(sub_lay.data_offset[j]), aux_offset=int(sub_lay.aux_offset[j]),
                                    n=specs[i].n, fmt=ofs[j], quantized=bool(sub_mask[j])) for j, i in enumerate(pick))
    kind = {"sgd": 0, "momentum": 1, "adam": 2}[wl["cfg"]["kind"]]
    arena0, sbt0 = arena.copy(), sbt.copy()
    cores = os.cpu_count() or 1
    out = {"pick": pick, "sub_lay": sub_lay, "sub_mask": sub_mask, "cores": cores,
           "n_elems": int(sum(specs[i].n for i in pick)),
           "packed_bytes": int(sum(orc.packed_bytes(specs[i].n, ofs[j].bits) for j, i in enumerate(pick) if sub_mask[j]))}
    for label, threads in (("one_thread", 1), ("all_cores", cores)):
        arena[:] = arena0
        sbt[:] = sbt0
        m = np.zeros(sub_lay.aux_elems, np.float32) if kind >= 1 else None
        v = np.zeros(sub_lay.aux_elems, np.float32) if kind == 2 else None
        t0 = time.perf_counter()
        for t in range(iters):
            orc.step_varset(arena, table, sbt, grads[t % len(grads)], m, v,
                            orc.Opt(kind=kind, lr=wl["cfg"]["lr"], t=t + 1), threads=threads)
            if t == 0 and label == "one_thread":
                out["first"] = (arena.copy(), sbt.copy(), None if m is None else m.copy())
        out[label] = (time.perf_counter() - t0) / iters
    return out


def parity_on_sample(torch, omc, wl, cpu):
    """One GPU step from the initial state against the oracle's first step on the sampled variables."""
    import numpy as np
    step_fn(omc, wl)(0)
    torch.cuda.synchronize()
    oa, osb, om = cpu["first"]
    ok = True
    for j, i in enumerate(cpu["pick"]):
        s = wl["specs"][i]
        d, e = int(wl["lay"].data_offset[i]), int(cpu["sub_lay"].data_offset[j])
        a, b = int(wl["lay"].aux_offset[i]), int(cpu["sub_lay"].aux_offset[j])
        nb = omc.omc_packed_bytes(wl["gfs"][i], s.n) if wl["mask"][i] else 4 * s.n
        ok &= bool(np.array_equal(wl["arena"][d:d + nb].cpu().numpy(), oa[e:e + nb]))
        if wl["mask"][i]:
            ok &= bool(np.array_equal(wl["sb"][i].cpu().numpy().view(np.uint32), osb[j].view(np.uint32)))
        if om is not None:
            ok &= bool(np.array_equal(wl["m"][a:a + s.n].cpu().numpy().view(np.uint32), om[b:b + s.n].view(np.uint32)))
    return ok


# ------------------------------------------------------------------------------------------------
# other legs
# ------------------------------------------------------------------------------------------------
def copy_ceiling(torch, n=1 << 28, iters=20):
    """GB/s of the runtime's own device-to-device copy of 1 GiB (2 GiB moved), measured in the same run."""
    src = torch.empty(n, device="cuda").normal_()
    dst = torch.empty_like(src)
    warm(torch, lambda k: dst.copy_(src))
    ms = timed(torch, lambda k: dst.copy_(src), iters)
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
        f = lambda k: omc.omc_dequant_gemm(A, codes, gf, sb, C, M, N, K, ws)
        warm(torch, f)
        ms = timed(torch, f, iters)
        tf = 2.0 * M * N * K / (ms * 1e-3) / 1e12
        rec = {"M": M, "N": N, "K": K, "ms": ms, "TFLOPs": tf, "frac_of_bf16_mfma_peak": tf / 2500.0,
               "hbm_bytes": 2 * M * K + K * N + 4 * M * N}
        # the same product with the weights in the paper's 11-bit format (Table 1: S1E3M7), generic decode
        gf11 = omc.fmt(3, 7)
        codes11 = torch.zeros(omc.omc_packed_bytes(gf11, K * N), dtype=torch.uint8, device="cuda")
        sb11 = torch.zeros(2, device="cuda")
        omc.omc_compress(W, K * N, gf11, True, codes11, sb11, wsc)
        f = lambda k: omc.omc_dequant_gemm(A, codes11, gf11, sb11, C, M, N, K, ws)
        warm(torch, f)
        ms = timed(torch, f, iters)
        rec["S1E3M7_ms"] = ms
        rec["S1E3M7_TFLOPs"] = 2.0 * M * N * K / (ms * 1e-3) / 1e12
        del codes11
        # the same layer's input gradient: dX[M, K] = dY[M, N] @ Wbar^T
        del C
        dY = torch.from_numpy(synth.to_bf16_bits(synth.normal_f32(M * N, 1.0, 13)).view(np.int16)).cuda()
        dX = torch.empty((M, K), dtype=torch.float32, device="cuda")
        f = lambda k: omc.omc_dequant_gemm_dx(dY, codes, gf, sb, dX, M, N, K, ws)
        warm(torch, f)
        ms = timed(torch, f, iters)
        rec["dx_ms"] = ms
        rec["dx_TFLOPs"] = 2.0 * M * N * K / (ms * 1e-3) / 1e12
        # and its weight gradient dW[K, N] = X^T @ dY, consumed by the SGD update + recompression
        del dX
        wsd = torch.empty(omc.omc_dw_update_workspace_bytes(gf, M, N, K), dtype=torch.uint8, device="cuda")
        o = omc.opt(omc.OMC_SGD, 0.01)
        f = lambda k: omc.omc_dw_update_recompress(A, dY, codes, gf, sb, True, None, None, o, None, M, N, K, wsd)
        warm(torch, f)
        ms = timed(torch, f, iters)
        rec["dw_update_ms"] = ms
        rec["dw_update_TFLOPs"] = 2.0 * M * N * K / (ms * 1e-3) / 1e12
        rec["dw_workspace_bytes"] = wsd.numel()   # fit partials + parked accumulators of the contraction splits
        out.append(rec)
    return out


def set_conversion_leg(torch, omc, wl, iters=20):
    """Whole-set conversions (start / end of a round): fp32 -> packed arena and back, one call each."""
    lay, plan = wl["lay"], wl["plan"]
    n_q, n_f = wl["n_q"], wl["n_f"]
    arena = torch.empty_like(wl["arena"])
    sb = torch.empty_like(wl["sb"])
    out = torch.empty(lay.aux_elems, device="cuda")
    ws = torch.empty(max(plan.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
    res = {}
    for name, fn, nbytes in (
            ("compress_set", lambda k: omc.omc_compress_set(wl["vals"], plan, arena, sb, ws), 5.0 * n_q + 8.0 * n_f),
            ("decompress_set", lambda k: omc.omc_decompress_set(arena, plan, sb, out), 5.0 * n_q + 8.0 * n_f)):
        warm(torch, fn)
        ms = timed(torch, fn, iters)
        res[name] = {"ms": ms, "algorithmic_GBps": nbytes / (ms * 1e-3) / 1e9,
                     "frac_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    res["transport_bytes"] = plan.transport_bytes
    res["transport_over_fp32"] = plan.transport_bytes / (4.0 * (n_q + n_f))
    return res


def round_boundary_leg(torch, omc, synth, blocks, iters=20):
    """What happens between two rounds on the 115 M-parameter set with the paper's 90 % partial quantization (S1E3M7):
    omc_reselect to another seeded 90 % subset (only the switched matrices are converted, the rest move as bytes), and
    omc_transport_pack of the set into one message."""
    specs = synth.conformer_varset(512, blocks, 2048, 32, frontend=True)
    gf = omc.fmt(3, 7)
    plans, lays = [], []
    for seed in (1, 2):
        mask = synth.ppq_mask(specs, 0.9, seed)
        lay = synth.make_layout(specs, mask, lambda n: omc.omc_packed_bytes(gf, n))
        table = [dict(data_offset=int(lay.data_offset[i]), aux_offset=int(lay.aux_offset[i]), n=s.n, fmt=gf,
                      quantized=bool(mask[i])) for i, s in enumerate(specs)]
        plans.append(omc.omc_plan_build(omc.make_var_table(table)))
        lays.append(lay)
    vals = torch.empty(lays[0].aux_elems, device="cuda").normal_(0.0, 0.03)
    arena_a = torch.zeros(lays[0].arena_bytes, dtype=torch.uint8, device="cuda")
    sb_a = torch.zeros((len(specs), 2), device="cuda")
    ws = torch.empty(max(plans[0].workspace_bytes, 16), dtype=torch.uint8, device="cuda")
    omc.omc_compress_set(vals, plans[0], arena_a, sb_a, ws)
    del vals
    rs = omc.omc_reselect_plan_build(plans[0], plans[1])
    arena_b = torch.zeros(lays[1].arena_bytes, dtype=torch.uint8, device="cuda")
    sb_b = torch.zeros_like(sb_a)
    ws2 = torch.empty(max(rs.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
    f = lambda k: omc.omc_reselect(rs, arena_a, sb_a, arena_b, sb_b, ws2)
    warm(torch, f)
    ms = timed(torch, f, iters)
    alg = float(rs.algorithmic_bytes)
    res = {"reselect": {"ms": ms, "algorithmic_bytes": alg, "algorithmic_GBps": alg / (ms * 1e-3) / 1e9,
                        "frac_hbm_peak": alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                        "fp32_copy_of_the_model_bytes": 4.0 * sum(s.n for s in specs)}}
    nbytes = omc.omc_transport_bytes(plans[1])
    msg = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    f = lambda k: omc.omc_transport_pack(plans[1], arena_b, sb_b, msg)
    warm(torch, f)
    ms = timed(torch, f, iters)
    res["transport_pack"] = {"ms": ms, "message_bytes": nbytes, "algorithmic_GBps": 2.0 * nbytes / (ms * 1e-3) / 1e9,
                             "frac_hbm_peak": 2.0 * nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                             "message_over_fp32": nbytes / (4.0 * sum(s.n for s in specs))}
    return res


def single_compress_leg(torch, omc, n=1 << 26, iters=20):
    """omc_compress / omc_decompress of one 64 M-element variable (S1E4M3)."""
    gf = omc.fmt(4, 3)
    x = torch.empty(n, device="cuda").normal_(0.0, 0.05)
    codes = torch.zeros(omc.omc_packed_bytes(gf, n), dtype=torch.uint8, device="cuda")
    sb = torch.zeros(2, device="cuda")
    ws = torch.empty(omc.omc_compress_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    out = torch.empty(n, device="cuda")
    res = {"elements": n}
    for name, fn in (("compress", lambda k: omc.omc_compress(x, n, gf, True, codes, sb, ws)),
                     ("decompress", lambda k: omc.omc_decompress(codes, n, gf, sb, out))):
        warm(torch, fn)
        ms = timed(torch, fn, iters)
        res[name] = {"ms": ms, "algorithmic_GBps": 5.0 * n / (ms * 1e-3) / 1e9,
                     "frac_hbm_peak": 5.0 * n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    return res


def aggregate_leg(torch, omc, synth, blocks, R=8, iters=20):
    """Server side of a round: mean of R clients' copies of the set, each client with its own 90 %
    subset of the weight matrices in S1E4M3 and the rest in fp32."""
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
    f = lambda k: omc.omc_aggregate_mean(agg, arenas, sbs, out)
    warm(torch, f)
    ms = timed(torch, f, iters)
    return {"clients": R, "params": n_total, "ms": ms, "algorithmic_bytes": alg,
            "algorithmic_GBps": alg / (ms * 1e-3) / 1e9, "frac_hbm_peak": alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "fp32_clients_bytes": 4.0 * n_total * (R + 1)}


def formats_leg(torch, omc, synth, blocks, flush, steps=20):
    """The fused decompress + SGD + recompress kernel on the 115 M-parameter set for every storage format of the
    paper's tables (Tables 1-3: 19-, 13-, 11- and 6-bit), per-variable transformation on and, for the 11-bit format,
    off (the ablation's switch); default flags, caches flushed between steps as in the roofline blocks."""
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
            flush[1].copy_(flush[0])
            omc.omc_step_update_recompress_events(arena, plan, sb, grads[k % 2], None, None, o, ws, ev, first=k * 2 * nl)
        torch.cuda.synchronize()
        ms = sum(ev.elapsed_ms(k * 2 * nl, k * 2 * nl + 1) for k in range(steps)) / steps
        alg = (2.0 * B / 8.0 + 4.0) * n_q
        res.append({"format": f"S1E{E}M{M}", "bits": B, "pvt": pvt, "kernel_ms": ms,
                    "algorithmic_GBps": alg / (ms * 1e-3) / 1e9, "frac_hbm_peak": alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS})
        del arena, sb, ws, plan
    return res


def main():
    global LEG_WARMUP_S
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="config4", choices=sorted(STEP_CONFIGS),
                    help="step configuration timed as the headline (default: the largest, config4)")
    ap.add_argument("--blocks", type=int, default=None, help="override the number of Conformer blocks (smaller runs)")
    ap.add_argument("--cpu-sample-blocks", type=int, default=1)
    ap.add_argument("--cpu-iters", type=int, default=4)
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle leg (for profiler runs)")
    ap.add_argument("--leg-warmup-s", type=float, default=LEG_WARMUP_S,
                    help="untimed wall time before each extra leg's measurement")
    ap.add_argument("--step-only", action="store_true",
                    help="only the headline configuration: no other configurations, no extra legs (for profiler runs)")
    ap.add_argument("--flush-between-steps", action="store_true",
                    help="with --step-only: run the timed steps with the cache-flushing copy before each of them "
                         "(for profiler runs of the evicted regime; the reported ms_per_step then includes the copies)")
    ap.add_argument("--clock-warmup-s", type=float, default=0.5,
                    help="seconds of untimed steps before any measurement, so that the GPU clocks have ramped up")
    ap.add_argument("--gemm-only", action="store_true", help="only the matrix-core leg (for profiler runs)")
    ap.add_argument("--aggregate-only", action="store_true", help="only the server aggregation leg")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device-to-device copy of known size (1 GiB read + 1 GiB written "
                         "per launch) to calibrate profiler byte counters and show the copy ceiling")
    args = ap.parse_args()
    LEG_WARMUP_S = args.leg_warmup_s
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU; --gpus must be 1 "
                 "(no collectives or sharding exist in this library)")

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
        ms = timed(torch, lambda k: dst.copy_(src), 20)
        print(json.dumps({"copy_kernel": "torch Tensor.copy_ fp32", "bytes_read": 4 * n, "bytes_written": 4 * n,
                          "ms": ms, "GBps": 8 * n / (ms * 1e-3) / 1e9}))
        return
    if args.gemm_only:
        print(json.dumps({"forward_gemm": gemm_leg(torch, omc, synth)}))
        return
    if args.aggregate_only:
        print(json.dumps({"server_aggregation": aggregate_leg(torch, omc, synth, 17)}))
        return

    flush = (torch.empty(1 << 27, device="cuda"), torch.empty(1 << 27, device="cuda"))    # 512 MiB each
    wl = build_step_workload(torch, omc, synth, args.config, blocks=args.blocks)

    # ---- CPU baseline (oracle) on a bounded sample + parity of the GPU's first step on that sample --------------
    cpu = parity = None
    if not args.no_cpu:
        cpu = cpu_baseline(torch, omc, synth, wl, args.cpu_sample_blocks, args.cpu_iters)
        arena0, sb0 = wl["arena"].clone(), wl["sb"].clone()
        parity = parity_on_sample(torch, omc, wl, cpu)
        wl["arena"].copy_(arena0)
        wl["sb"].copy_(sb0)
        if wl["m"] is not None:
            wl["m"].zero_()
        wl["t"] = 0
        del arena0, sb0

    if args.step_only and args.flush_between_steps:
        step = step_fn(omc, wl)
        warm(torch, step, args.clock_warmup_s)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            flush[1].copy_(flush[0])
            step(k)
        torch.cuda.synchronize()
        ms_per_step, reg = 1e3 * (time.perf_counter() - t0) / args.steps, None
    else:
        ms_per_step, reg = measure_step_config(torch, omc, wl, args.steps, args.warmup, args.clock_warmup_s, flush,
                                               regimes=True)
    out = {
        "metric": "compressed-param GB/s per decompress+update+recompress step; % HBM peak",
        "value": wl["packed"] / (ms_per_step * 1e-3) / 1e9,
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
        "config": dict(describe(wl, ms_per_step), config=args.config, launch="one library call per step, default flags",
                       parity_vs_oracle_on_sample=parity),
    }
    if reg is not None:
        out["roofline"] = roofline_block(wl, reg)
    if cpu is not None:
        out["cpu_baseline"] = {
            "value": cpu["packed_bytes"] / cpu["all_cores"] / 1e9, "unit": "GB/s", "cores": cpu["cores"], "kind": "oracle",
            "one_thread_value": cpu["packed_bytes"] / cpu["one_thread"] / 1e9,
            "sample": f"variables of the first {args.cpu_sample_blocks} Conformer block(s) of the same set "
                      f"({cpu['n_elems']} params, {cpu['packed_bytes']} packed bytes), {args.cpu_iters} iterations each: "
                      f"{1e3 * cpu['one_thread']:.0f} ms per iteration on one thread, {1e3 * cpu['all_cores']:.0f} ms on "
                      f"{cpu['cores']} threads (os.cpu_count(); OpenMP over variables)",
        }
    del wl
    torch.cuda.empty_cache()
    if not args.step_only:
        others = []
        for name in sorted(STEP_CONFIGS):
            if name == args.config:
                continue
            w2 = build_step_workload(torch, omc, synth, name, blocks=args.blocks)
            ms2, reg2 = measure_step_config(torch, omc, w2, min(args.steps, 50), args.warmup, LEG_WARMUP_S, flush)
            rec = dict(describe(w2, ms2), config=name, ms_per_step=ms2,
                       compressed_param_GBps=w2["packed"] / (ms2 * 1e-3) / 1e9, roofline=roofline_block(w2, reg2))
            if name == "config2":
                rec["set_conversions"] = set_conversion_leg(torch, omc, w2)
            others.append(rec)
            del w2
            torch.cuda.empty_cache()
        out["other_step_configs"] = others
        out["copy_kernel_GBps"] = copy_ceiling(torch)          # the runtime's device-to-device copy of 1 GiB, same run
        out["single_variable_64M"] = single_compress_leg(torch, omc)
        torch.cuda.empty_cache()
        blocks = 17 if args.blocks is None else min(args.blocks, 17)
        out["round_boundary"] = round_boundary_leg(torch, omc, synth, blocks)
        torch.cuda.empty_cache()
        out["server_aggregation"] = aggregate_leg(torch, omc, synth, blocks)
        torch.cuda.empty_cache()
        out["paper_formats_sgd"] = formats_leg(torch, omc, synth, blocks, flush)
        torch.cuda.empty_cache()
        out["forward_gemm"] = gemm_leg(torch, omc, synth)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
