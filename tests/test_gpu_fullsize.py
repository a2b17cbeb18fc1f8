"""Parity at the full benchmark sizes, in the launch configuration bench.py times.

The whole variable set is compressed and stepped on the GPU; the oracle recomputes a sample of
variables (largest, smallest, first, last, one of each shape class, some fp32 ones) from the same
seeded inputs, one by one, and those must be bit-identical: packed codes, (s, b), optimizer state.
Inputs are generated on the device (seeded Philox) and only the sampled slices are copied back."""
import numpy as np
import pytest
import torch

from oracle import omc_oracle as orc
from paper_2205_03494_amd import omc, synth
from gpu_util import bits_equal

pytestmark = pytest.mark.gpu


def pick_samples(specs, mask, k_extra=3):
    idx = set()
    q = [i for i in range(len(specs)) if mask[i]]
    f = [i for i in range(len(specs)) if not mask[i]]
    if q:
        idx.update([q[0], q[-1], max(q, key=lambda i: specs[i].n), min(q, key=lambda i: specs[i].n)])
        seen = set()
        for i in q:                                   # one of each shape class
            if specs[i].shape not in seen and len(seen) < 8:
                seen.add(specs[i].shape)
                idx.add(i)
    if f:
        idx.update([f[0], f[-1], max(f, key=lambda i: specs[i].n)])
        fm = [i for i in f if specs[i].is_matrix]
        idx.update(fm[:k_extra])
    return sorted(idx)


def run_fullsize(specs, mask, fmts, kind, lr, steps, seed, max_sample_elems=14_000_000, first_samples=(), flags=0):
    gfs = [omc.fmt(*fmts[i]) if mask[i] else None for i in range(len(specs))]
    sizes = iter([omc.omc_packed_bytes(gfs[i], specs[i].n) for i in range(len(specs)) if mask[i]])
    lay = synth.make_layout(specs, mask, lambda n: next(sizes))
    gen = torch.Generator(device="cuda").manual_seed(seed)
    vals = torch.empty(lay.aux_elems, device="cuda")
    for i, s in enumerate(specs):                     # N(0, 1/sqrt(fan_in)) matrices, small vectors
        a = int(lay.aux_offset[i])
        std = 1.0 / np.sqrt(s.fan_in) if s.is_matrix else 0.02
        vals[a:a + s.n].normal_(0.0, std, generator=gen)
    grads = [torch.empty(lay.aux_elems, device="cuda").normal_(0.0, 1e-3, generator=gen) for _ in range(2)]
    arena = torch.zeros(lay.arena_bytes, dtype=torch.uint8, device="cuda")
    sb = torch.zeros((len(specs), 2), device="cuda")
    sb[:, 0] = 1.0
    ws = torch.empty(omc.omc_compress_workspace_bytes(max(s.n for s in specs)), dtype=torch.uint8, device="cuda")
    table = []
    for i, s in enumerate(specs):
        a, d = int(lay.aux_offset[i]), int(lay.data_offset[i])
        if mask[i]:
            omc.omc_compress(vals[a:a + s.n], s.n, gfs[i], True, arena[d:d + omc.omc_packed_bytes(gfs[i], s.n)], sb[i], ws)
        else:
            arena[d:d + 4 * s.n] = vals[a:a + s.n].view(torch.uint8)
        table.append(dict(data_offset=d, aux_offset=a, n=s.n, fmt=gfs[i], quantized=bool(mask[i])))
    plan = omc.omc_plan_build(omc.make_var_table(table))
    m = torch.zeros(lay.aux_elems, device="cuda")
    v = torch.zeros(lay.aux_elems, device="cuda")
    ws2 = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device="cuda")

    samples, total = [], 0
    for i in list(first_samples) + [j for j in pick_samples(specs, mask) if j not in first_samples]:
        if total + specs[i].n <= max_sample_elems or not samples:
            samples.append(i)
            total += specs[i].n
    # oracle state of the samples, from the same fp32 values
    ost = {}
    for i in samples:
        s = specs[i]
        a, d = int(lay.aux_offset[i]), int(lay.data_offset[i])
        x = vals[a:a + s.n].cpu().numpy()
        if mask[i]:
            of = orc.Format(*fmts[i])
            p, osb = orc.compress(x, of)
            nb = omc.omc_packed_bytes(gfs[i], s.n)
            assert np.array_equal(arena[d:d + nb].cpu().numpy(), p), f"compress: {s.name}"
            assert bits_equal(sb[i].cpu().numpy(), osb), f"compress (s, b): {s.name}"
            ost[i] = dict(p=p, sb=osb, m=np.zeros(s.n, np.float32), v=np.zeros(s.n, np.float32))
        else:
            ost[i] = dict(w=x.copy(), m=np.zeros(s.n, np.float32), v=np.zeros(s.n, np.float32))
    for t in range(1, steps + 1):
        omc.omc_step_update_recompress(arena, plan, sb, grads[t % 2], m, v, omc.opt(kind, lr, t=t, flags=flags), ws2)
        torch.cuda.synchronize()
        for i in samples:
            s = specs[i]
            a, d = int(lay.aux_offset[i]), int(lay.data_offset[i])
            g = grads[t % 2][a:a + s.n].cpu().numpy()
            o = orc.Opt(kind=kind, lr=lr, t=t)
            st = ost[i]
            if mask[i]:
                orc.step_quantized(st["p"], s.n, orc.Format(*fmts[i]), st["sb"], g, st["m"] if kind >= 1 else None,
                                   st["v"] if kind == 2 else None, o)
                nb = st["p"].size
                assert np.array_equal(arena[d:d + nb].cpu().numpy(), st["p"]), f"step {t} codes: {s.name}"
                assert bits_equal(sb[i].cpu().numpy(), st["sb"]), f"step {t} (s, b): {s.name}"
            else:
                orc.step_fp32(st["w"], g, st["m"] if kind >= 1 else None, st["v"] if kind == 2 else None, o)
                assert bits_equal(arena[d:d + 4 * s.n].cpu().numpy().view(np.float32), st["w"]), f"step {t} fp32: {s.name}"
            if kind >= 1:
                assert bits_equal(m[a:a + s.n].cpu().numpy(), st["m"]), f"step {t} state0: {s.name}"
            if kind == 2:
                assert bits_equal(v[a:a + s.n].cpu().numpy(), st["v"]), f"step {t} state1: {s.name}"
    return len(samples), total


def test_config2_full_size_sgd_8bit():
    specs = synth.conformer_varset(512, 17, 2048, 32, frontend=True)
    mask = np.array([s.is_matrix for s in specs])
    fmts = [(4, 3)] * len(specs)
    ns, total = run_fullsize(specs, mask, fmts, kind=0, lr=0.01, steps=2, seed=2)
    assert ns >= 8 and total > 8_000_000


def test_config3_full_size_partial_quantization_three_formats_adam():
    specs = synth.conformer_varset(512, 17, 2048, 32, frontend=True)
    mask = synth.ppq_mask(specs, 0.5, 3)
    choices = [(4, 3), (3, 7), (5, 10)]
    fmts = [choices[i % 3] for i in range(len(specs))]
    ns, total = run_fullsize(specs, mask, fmts, kind=2, lr=1e-3, steps=2, seed=3, max_sample_elems=12_000_000)
    assert ns >= 6


def test_config3_set_under_sgd_fp32_values_on_both_sides_of_the_cache_budget():
    """Same set as configuration 3 under plain SGD with OMC_OPT_KEEP_CODES: 78 MB of codes stay cached and the
    249 MB of fp32 matrices get what is left of the budget, so their work items fall on both sides of that limit
    within one launch."""
    specs = synth.conformer_varset(512, 17, 2048, 32, frontend=True)
    mask = synth.ppq_mask(specs, 0.5, 3)
    choices = [(4, 3), (3, 7), (5, 10)]
    fmts = [choices[i % 3] for i in range(len(specs))]
    f32 = [i for i in range(len(specs)) if not mask[i] and specs[i].is_matrix]
    done, cut = 0, None
    for k, i in enumerate(f32):                        # fp32 items follow the plan's variable order
        done += 4 * specs[i].n
        if done > (224 << 20) - 78_000_000:
            cut = f32[max(k - 1, 0):k + 2]
            break
    assert cut
    ns, total = run_fullsize(specs, mask, fmts, kind=0, lr=0.01, steps=2, seed=7, max_sample_elems=14_000_000,
                             first_samples=cut + [f32[0], f32[-1]], flags=omc.OMC_OPT_KEEP_CODES)
    assert ns >= 6


@pytest.mark.parametrize("flags", [0, omc.OMC_OPT_KEEP_CODES])
def test_config4_full_size_momentum_11bit(flags):
    specs = synth.conformer_varset(1024, 24, 4096, 32, frontend=False)
    mask = np.array([s.is_matrix for s in specs])
    assert 5.9e8 < sum(s.n for s in specs if s.is_matrix) < 6.2e8
    fmts = [(3, 7)] * len(specs)
    # 832 MB of packed codes: by default all of them stream; with OMC_OPT_KEEP_CODES the step keeps the first 224 MiB
    # cached and streams the rest, as two launches of the fused kernel.  The variable that this limit cuts through
    # and its neighbours are checked first
    done, cut = 0, None
    for i, s in enumerate(specs):
        if mask[i]:
            done += s.n * 11 // 8
            if done > (224 << 20):
                cut = i
                break
    assert cut is not None
    near = [i for i in range(cut - 3, cut + 4) if 0 <= i < len(specs) and mask[i]][:3]
    ns, total = run_fullsize(specs, mask, fmts, kind=1, lr=0.01, steps=2, seed=4, max_sample_elems=16_000_000,
                             first_samples=near, flags=flags)
    assert ns >= 6


def test_large_mixed_set_adam_launches_on_both_sides_of_the_cache_budget():
    """604 M-parameter set, 90 % of the matrices quantized in three widths, Adam: 0.79 GB of packed codes.  The
    step (with OMC_OPT_KEEP_CODES) keeps the first 224 MiB of codes cached: all of the 8-bit group's launch and a part of the 11-bit
    group's, which is launched in two parts, while the 16-bit group streams as a whole; the fp32 matrices ride
    along with the first launch.  Sampled: the variables around the cut, and the usual first / last / largest."""
    specs = synth.conformer_varset(1024, 24, 4096, 32, frontend=False)
    mask = synth.ppq_mask(specs, 0.9, 5)
    choices = [(4, 3), (3, 7), (5, 10)]
    fmts = [choices[i % 3] for i in range(len(specs))]
    bits = lambda i: 1 + sum(fmts[i])
    by_width = {b: [i for i in range(len(specs)) if mask[i] and bits(i) == b] for b in (8, 11, 16)}
    assert sum(specs[i].n for i in by_width[8]) < (224 << 20) < sum(specs[i].n * bits(i) // 8 for b in (8, 11) for i in by_width[b])
    done, near = sum(specs[i].n for i in by_width[8]), []
    for k, i in enumerate(by_width[11]):
        done += specs[i].n * 11 // 8
        if done > (224 << 20):
            near = by_width[11][max(k - 1, 0):k + 2]
            break
    assert near
    first = near + [by_width[8][-1], by_width[16][0]]
    ns, total = run_fullsize(specs, mask, fmts, kind=2, lr=1e-3, steps=2, seed=6, max_sample_elems=24_000_000,
                             first_samples=first, flags=omc.OMC_OPT_KEEP_CODES)
    assert ns >= 8


def _device_values(specs, lay, seed, delta_seed=None):
    gen = torch.Generator(device="cuda").manual_seed(seed)
    vals = torch.empty(lay.aux_elems, device="cuda")
    for i, s in enumerate(specs):
        a = int(lay.aux_offset[i])
        std = 1.0 / np.sqrt(s.fan_in) if s.is_matrix else 0.02
        vals[a:a + s.n].normal_(0.0, std, generator=gen)
    if delta_seed is not None:                          # a client's own small update on top of the shared values
        g2 = torch.Generator(device="cuda").manual_seed(delta_seed)
        vals += torch.empty_like(vals).normal_(0.0, 2e-3, generator=g2)
    return vals


def test_benchmark_set_whole_set_conversions_and_server_aggregation():
    """Config-2 sized set (115 M parameters): omc_compress_set, omc_decompress_set and omc_aggregate_mean over
    four clients with their own 90 % subsets, in the launch configuration bench.py times; the oracle
    recomputes sampled variables one by one."""
    specs = synth.conformer_varset(512, 17, 2048, 32, frontend=True)
    fmt = (4, 3)
    of, gf = orc.Format(*fmt), omc.fmt(*fmt)
    R = 4
    clients = []
    for r in range(R):
        mask = synth.ppq_mask(specs, 0.9, 300 + r)
        lay = synth.make_layout(specs, mask, lambda n: omc.omc_packed_bytes(gf, n))
        table = [dict(data_offset=int(lay.data_offset[i]), aux_offset=int(lay.aux_offset[i]), n=s.n, fmt=gf,
                      quantized=bool(mask[i])) for i, s in enumerate(specs)]
        plan = omc.omc_plan_build(omc.make_var_table(table))
        vals = _device_values(specs, lay, 7, delta_seed=900 + r)
        arena = torch.zeros(lay.arena_bytes, dtype=torch.uint8, device="cuda")
        sb = torch.zeros((len(specs), 2), device="cuda")
        ws = torch.empty(max(plan.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
        omc.omc_compress_set(vals, plan, arena, sb, ws)
        clients.append(dict(mask=mask, lay=lay, plan=plan, vals=vals, arena=arena, sb=sb))
    torch.cuda.synchronize()
    lay0 = clients[0]["lay"]
    # sample: union of the per-client picks, bounded
    samples, total = [], 0
    for i in pick_samples(specs, clients[0]["mask"]):
        if total + specs[i].n <= 9_000_000 or not samples:
            samples.append(i)
            total += specs[i].n
    # 1. compress_set: each client's transported form of the sampled variables
    copies = {i: [] for i in samples}
    for c in clients:
        for i in samples:
            s = specs[i]
            a, d = int(c["lay"].aux_offset[i]), int(c["lay"].data_offset[i])
            x = c["vals"][a:a + s.n].cpu().numpy()
            if c["mask"][i]:
                p, osb = orc.compress(x, of)
                nb = omc.omc_packed_bytes(gf, s.n)
                assert np.array_equal(c["arena"][d:d + nb].cpu().numpy(), p), f"compress_set: {s.name}"
                assert bits_equal(c["sb"][i].cpu().numpy(), osb)
                copies[i].append(orc.decompress(p, s.n, of, osb))
            else:
                assert bits_equal(c["arena"][d:d + 4 * s.n].cpu().numpy().view(np.float32), x), f"compress_set fp32: {s.name}"
                copies[i].append(x)
    # 2. decompress_set of client 0
    out = torch.empty(lay0.aux_elems, device="cuda")
    omc.omc_decompress_set(clients[0]["arena"], clients[0]["plan"], clients[0]["sb"], out)
    torch.cuda.synchronize()
    for i in samples:
        a = int(lay0.aux_offset[i])
        assert bits_equal(out[a:a + specs[i].n].cpu().numpy(), copies[i][0]), f"decompress_set: {specs[i].name}"
    # 3. the server's mean over the four clients
    agg = omc.omc_aggregate_plan_build([c["plan"] for c in clients])
    omc.omc_aggregate_mean(agg, [c["arena"] for c in clients], [c["sb"] for c in clients], out)
    torch.cuda.synchronize()
    for i in samples:
        a = int(lay0.aux_offset[i])
        assert bits_equal(out[a:a + specs[i].n].cpu().numpy(), orc.aggregate_mean(copies[i])), f"aggregate: {specs[i].name}"
    assert torch.isfinite(out).all()


def test_benchmark_set_reselection_and_transport_message():
    """Config-2 sized set with the paper's 90 % partial quantization (S1E3M7), as bench.py's round_boundary leg runs it:
    omc_reselect to another seeded 90 % subset, then omc_transport_pack of the result.  Every moved variable is compared
    byte for byte on the GPU; sampled converted variables against the oracle's compress / decompress; the message's
    payload against the arena it was packed from."""
    specs = synth.conformer_varset(512, 17, 2048, 32, frontend=True)
    fmt = (3, 7)
    of, gf = orc.Format(*fmt), omc.fmt(*fmt)
    plans, lays, masks = [], [], []
    for seed in (1, 2):
        mask = synth.ppq_mask(specs, 0.9, seed)
        lay = synth.make_layout(specs, mask, lambda n: omc.omc_packed_bytes(gf, n))
        table = [dict(data_offset=int(lay.data_offset[i]), aux_offset=int(lay.aux_offset[i]), n=s.n, fmt=gf,
                      quantized=bool(mask[i])) for i, s in enumerate(specs)]
        plans.append(omc.omc_plan_build(omc.make_var_table(table)))
        lays.append(lay); masks.append(mask)
    vals = _device_values(specs, lays[0], 7)
    arena_a = torch.zeros(lays[0].arena_bytes, dtype=torch.uint8, device="cuda")
    sb_a = torch.zeros((len(specs), 2), device="cuda")
    ws = torch.empty(max(plans[0].workspace_bytes, 16), dtype=torch.uint8, device="cuda")
    omc.omc_compress_set(vals, plans[0], arena_a, sb_a, ws)
    del vals
    rs = omc.omc_reselect_plan_build(plans[0], plans[1])
    arena_b = torch.zeros(lays[1].arena_bytes, dtype=torch.uint8, device="cuda")
    sb_b = torch.full((len(specs), 2), 7.0, device="cuda")
    ws2 = torch.empty(max(rs.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
    omc.omc_reselect(rs, arena_a, sb_a, arena_b, sb_b, ws2)
    torch.cuda.synchronize()
    to_q = [i for i in range(len(specs)) if not masks[0][i] and masks[1][i]]
    to_f = [i for i in range(len(specs)) if masks[0][i] and not masks[1][i]]
    assert to_q and to_f
    checked, budget = 0, 9_000_000
    for i, s in enumerate(specs):
        da, db = int(lays[0].data_offset[i]), int(lays[1].data_offset[i])
        nb = omc.omc_packed_bytes(gf, s.n)
        if masks[0][i] == masks[1][i]:                       # moved as bytes: compared in full, on the GPU
            n_bytes = nb if masks[0][i] else 4 * s.n
            assert torch.equal(arena_b[db:db + n_bytes], arena_a[da:da + n_bytes]), f"moved: {s.name}"
            if masks[0][i]:
                assert torch.equal(sb_b[i].view(torch.int32), sb_a[i].view(torch.int32))
        elif budget >= s.n:                                   # converted: the oracle on as many as the budget allows
            budget -= s.n
            checked += 1
            if masks[1][i]:
                p, fit = orc.compress(arena_a[da:da + 4 * s.n].cpu().numpy().view(np.float32).copy(), of)
                assert np.array_equal(arena_b[db:db + nb].cpu().numpy(), p), f"to codes: {s.name}"
                assert bits_equal(sb_b[i].cpu().numpy(), fit)
            else:
                x = orc.decompress(arena_a[da:da + nb].cpu().numpy().copy(), s.n, of, sb_a[i].cpu().numpy())
                assert bits_equal(arena_b[db:db + 4 * s.n].cpu().numpy().view(np.float32), x), f"to fp32: {s.name}"
    assert checked >= 4
    # the message of the new selection: payload = the arena, variable by variable
    nbytes = omc.omc_transport_bytes(plans[1])
    msg = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    omc.omc_transport_pack(plans[1], arena_b, sb_b, msg)
    torch.cuda.synchronize()
    meta = omc.omc_transport_meta_bytes(len(specs))
    table, nvars, sb_off, arena_off, arena_bytes, _ = omc.omc_transport_open(msg[:meta].cpu().numpy(), nbytes)
    assert nvars == len(specs)
    for i, s in enumerate(specs):
        db, dm = int(lays[1].data_offset[i]), arena_off + int(table[i].data_offset)
        n_bytes = omc.omc_packed_bytes(gf, s.n) if masks[1][i] else 4 * s.n
        assert torch.equal(msg[dm:dm + n_bytes], arena_b[db:db + n_bytes]), f"message payload: {s.name}"
    sbm = msg[sb_off:sb_off + 8 * nvars].view(torch.float32).view(nvars, 2)
    q = torch.from_numpy(np.asarray(masks[1])).cuda()
    assert torch.equal(sbm[q].view(torch.int32), sb_b[q].view(torch.int32))


def test_config2_every_variable_free_running():
    """BASELINE config 2 on every one of its 599 variables (not a sample): the whole 115 M-parameter set stepped
    twenty times on both sides without resynchronising; arena and (s, b) table identical at the end.  (Run
    once with the configuration's full 100 iterations, checked every ten: identical throughout.)"""
    from gpu_util import VarSet, to_dev
    specs = synth.conformer_varset(512, 17, 2048, 32, frontend=True)
    mask = np.array([s.is_matrix for s in specs])
    vs = VarSet(specs, mask, (4, 3), seed=0)
    grads = [synth.gradients(vs.lay, 1e-3, 1000 + k) for k in range(2)]
    g_dev = [to_dev(g) for g in grads]
    for t in range(1, 21):
        vs.step_oracle(grads[t % 2], 0, 0.01, t, threads=16)
        vs.step_gpu(g_dev[t % 2], 0, 0.01, t)
    assert vs.compare(0, "after 20 steps") == 0
