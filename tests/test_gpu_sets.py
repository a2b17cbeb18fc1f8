"""GPU parity of the whole-set conversions (start / end of a round, and a change of the set of
quantized variables between rounds, Sec. 2.5) against per-variable oracle calls."""
import numpy as np
import pytest
import torch

from oracle import omc_oracle as orc
from paper_2205_03494_amd import omc, synth
from gpu_util import bits_equal, to_dev

pytestmark = pytest.mark.gpu


def build(specs, mask, fmts, use_pvt=True):
    gfs = [omc.fmt(*fmts[i]) if mask[i] else None for i in range(len(specs))]
    sizes = iter([omc.omc_packed_bytes(gfs[i], specs[i].n) for i in range(len(specs)) if mask[i]])
    lay = synth.make_layout(specs, mask, lambda n: next(sizes))
    table = [dict(data_offset=int(lay.data_offset[i]), aux_offset=int(lay.aux_offset[i]), n=s.n, fmt=gfs[i],
                  quantized=bool(mask[i]), use_pvt=use_pvt) for i, s in enumerate(specs)]
    return lay, omc.omc_plan_build(omc.make_var_table(table))


def oracle_arena(specs, mask, fmts, lay, vals):
    arena = np.zeros(lay.arena_bytes, np.uint8)
    sbt = np.zeros((len(specs), 2), np.float32)
    for i, s in enumerate(specs):
        a, d = int(lay.aux_offset[i]), int(lay.data_offset[i])
        x = vals[a:a + s.n]
        if mask[i]:
            p, sb = orc.compress(x, orc.Format(*fmts[i]))
            arena[d:d + p.size] = p
            sbt[i] = sb
        else:
            arena[d:d + 4 * s.n] = x.view(np.uint8)
    return arena, sbt


def gpu_compress_set(lay, plan, vals, nvars):
    arena = torch.full((lay.arena_bytes,), 0, dtype=torch.uint8, device="cuda")
    sb = torch.full((nvars, 2), 7.0, device="cuda")
    ws = torch.empty(max(plan.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
    omc.omc_compress_set(to_dev(vals), plan, arena, sb, ws)
    torch.cuda.synchronize()
    return arena, sb


def ragged_specs():
    # sizes around the tile and chunk borders, a tail-only variable, vectors
    ns = [1, 31, 2047, 2048, 2049, 4096, 4097, 8192, 8193, 5 * 8192 + 77, 3 * 2048, 40000, 100, 2048 * 9 + 1]
    return [synth.VarSpec(f"v{i}", (n,), max(n, 1), i % 4 != 3) for i, n in enumerate(ns)]


@pytest.mark.parametrize("case", ["conformer", "ragged", "fp32_only", "tails_only"])
def test_compress_set_and_decompress_set(case):
    if case == "conformer":
        specs = synth.conformer_varset(96, 2, 384, 8, frontend=True)
        mask = synth.ppq_mask(specs, 0.6, 4)
    elif case == "ragged":
        specs = ragged_specs()
        mask = np.array([s.is_matrix for s in specs])
    elif case == "fp32_only":
        specs = ragged_specs()
        mask = np.zeros(len(specs), bool)
    else:
        specs = [synth.VarSpec(f"t{i}", (n,), n, True) for i, n in enumerate([5, 700, 2047, 33])]
        mask = np.ones(len(specs), bool)
    choices = [(4, 3), (3, 7), (5, 10), (2, 3), (8, 7)]
    fmts = [choices[i % len(choices)] for i in range(len(specs))]
    lay, plan = build(specs, mask, fmts)
    vals = synth.init_values(lay, 9)
    want_arena, want_sb = oracle_arena(specs, mask, fmts, lay, vals)
    arena, sb = gpu_compress_set(lay, plan, vals, len(specs))
    assert np.array_equal(arena.cpu().numpy(), want_arena)
    gsb = sb.cpu().numpy()
    assert bits_equal(gsb[mask], want_sb[mask])
    assert np.all(gsb[~mask] == 7.0)                       # untouched for fp32 variables
    assert plan.transport_bytes == sum(orc.packed_bytes(s.n, 1 + sum(fmts[i])) + 8 if mask[i] else 4 * s.n
                                       for i, s in enumerate(specs))
    # and back
    out = torch.full((lay.aux_elems,), float("nan"), device="cuda")
    omc.omc_decompress_set(arena, plan, sb, out)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    for i, s in enumerate(specs):
        a, d = int(lay.aux_offset[i]), int(lay.data_offset[i])
        if mask[i]:
            of = orc.Format(*fmts[i])
            nb = orc.packed_bytes(s.n, of.bits)
            want = orc.decompress(want_arena[d:d + nb], s.n, of, want_sb[i])
        else:
            want = vals[a:a + s.n]
        assert bits_equal(o[a:a + s.n], want), s.name
        pad = o[a + s.n:int(lay.aux_offset[i + 1]) if i + 1 < len(specs) else lay.aux_elems]
        assert np.all(np.isnan(pad))                       # nothing written between variables


def test_reselection_between_rounds():
    """The set of quantized variables changes (Sec. 2.5): decompress with the old plan, compress with
    the new one; every variable must come out as the oracle's conversion of the same values."""
    specs = synth.conformer_varset(64, 2, 256, 8, frontend=False)
    fmts = [(3, 7)] * len(specs)
    mask_a, mask_b = synth.ppq_mask(specs, 0.9, 1), synth.ppq_mask(specs, 0.9, 2)
    assert np.any(mask_a != mask_b)
    lay_a, plan_a = build(specs, mask_a, fmts)
    lay_b, plan_b = build(specs, mask_b, fmts)
    vals = synth.init_values(lay_a, 3)
    arena_a, sb_a = gpu_compress_set(lay_a, plan_a, vals, len(specs))
    mid = torch.zeros(lay_a.aux_elems, device="cuda")
    omc.omc_decompress_set(arena_a, plan_a, sb_a, mid)
    arena_b = torch.zeros(lay_b.arena_bytes, dtype=torch.uint8, device="cuda")
    sb_b = torch.zeros((len(specs), 2), device="cuda")
    ws = torch.empty(max(plan_b.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
    omc.omc_compress_set(mid, plan_b, arena_b, sb_b, ws)
    torch.cuda.synchronize()
    oa, osb = oracle_arena(specs, mask_a, fmts, lay_a, vals)
    mid_ref = np.zeros(lay_a.aux_elems, np.float32)
    of = orc.Format(3, 7)
    for i, s in enumerate(specs):
        a, d = int(lay_a.aux_offset[i]), int(lay_a.data_offset[i])
        mid_ref[a:a + s.n] = (orc.decompress(oa[d:d + orc.packed_bytes(s.n, 11)], s.n, of, osb[i]) if mask_a[i]
                              else vals[a:a + s.n])
    ob, osb_b = oracle_arena(specs, mask_b, fmts, lay_b, mid_ref)
    assert np.array_equal(arena_b.cpu().numpy(), ob)
    assert bits_equal(sb_b.cpu().numpy()[mask_b], osb_b[mask_b])
