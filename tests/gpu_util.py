"""Helpers for the GPU parity tests: run the same seeded inputs through libomc and the oracle."""
import numpy as np
import torch

from oracle import omc_oracle as orc
from paper_2205_03494_amd import omc, synth


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def pair(E, M, bias=None):
    """The same format for both sides."""
    return orc.Format(E, M, bias), omc.fmt(E, M, omc.OMC_BIAS_DEFAULT if bias is None else bias)


def bits_equal(a, b):
    a = np.ascontiguousarray(a)
    b = np.ascontiguousarray(b)
    return a.shape == b.shape and np.array_equal(a.view(np.uint8), b.view(np.uint8))


def gpu_compress(v, gf, use_pvt=True, canary=64):
    """-> (packed bytes, sb).  Also checks that nothing is written past the packed buffer."""
    n = v.size
    nb = omc.omc_packed_bytes(gf, n)
    codes = torch.full((nb + canary,), 0xA5, dtype=torch.uint8, device="cuda")
    sb = torch.zeros(2, dtype=torch.float32, device="cuda")
    ws = torch.empty(max(omc.omc_compress_workspace_bytes(n), 16), dtype=torch.uint8, device="cuda")
    omc.omc_compress(to_dev(v), n, gf, use_pvt, codes, sb, ws)
    torch.cuda.synchronize()
    out = codes.cpu().numpy()
    assert np.all(out[nb:] == 0xA5), "compress wrote past the packed buffer"
    return out[:nb].copy(), sb.cpu().numpy()


def gpu_decompress(packed, n, gf, sb=None, canary=16):
    out = torch.full((n + canary,), float("nan"), dtype=torch.float32, device="cuda")
    omc.omc_decompress(to_dev(packed), n, gf, None if sb is None else to_dev(np.asarray(sb, np.float32)), out)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert np.all(np.isnan(o[n:])), "decompress wrote past its output"
    return o[:n].copy()


class VarSet:
    """A variable set held twice: numpy arrays for the oracle, device tensors for libomc."""

    def __init__(self, specs, quant_mask, fmts, seed, use_pvt=True, values=None):
        # fmts: per-variable (E, M) or None, or one (E, M) for all quantized variables
        self.specs = list(specs)
        nv = len(self.specs)
        if isinstance(fmts, tuple):
            fmts = [fmts if q else None for q in quant_mask]
        self.fmts = fmts
        self.mask = np.asarray(quant_mask, dtype=bool)
        sizes = [omc.omc_packed_bytes(omc.fmt(*fmts[i]), s.n) if self.mask[i] else 4 * s.n
                 for i, s in enumerate(self.specs)]
        it = iter([sz for sz, q in zip(sizes, self.mask) if q])   # make_layout asks for quantized ones only
        self.lay = synth.make_layout(self.specs, self.mask, lambda n: next(it))
        lay = self.lay
        vals = synth.init_values(lay, seed) if values is None else values
        self.init = vals
        arena = np.zeros(lay.arena_bytes, np.uint8)
        sbt = np.zeros((nv, 2), np.float32)
        sbt[:, 0] = 1.0
        desc = []
        for i, s in enumerate(self.specs):
            a, d = int(lay.aux_offset[i]), int(lay.data_offset[i])
            x = vals[a:a + s.n]
            if self.mask[i]:
                of = orc.Format(*fmts[i])
                p, sb = orc.compress(x, of, use_pvt)
                assert p.size == sizes[i] == orc.packed_bytes(s.n, of.bits)
                arena[d:d + p.size] = p
                sbt[i] = sb
            else:
                arena[d:d + 4 * s.n] = x.view(np.uint8)
            desc.append(dict(data_offset=d, aux_offset=a, n=s.n, quantized=bool(self.mask[i]),
                             use_pvt=use_pvt))
        self.o_table = orc.make_var_table(dict(d, fmt=orc.Format(*fmts[i]) if self.mask[i] else None)
                                          for i, d in enumerate(desc))
        self.g_table = omc.make_var_table([dict(d, fmt=omc.fmt(*fmts[i]) if self.mask[i] else None)
                                           for i, d in enumerate(desc)])
        self.plan = omc.omc_plan_build(self.g_table)
        assert self.plan.arena_bytes <= lay.arena_bytes and self.plan.aux_elems <= lay.aux_elems
        # oracle state
        self.o_arena, self.o_sb = arena, sbt
        self.o_m = np.zeros(lay.aux_elems, np.float32)
        self.o_v = np.zeros(lay.aux_elems, np.float32)
        # device state
        self.upload()
        self.ws = torch.empty(max(self.plan.workspace_bytes, 16), dtype=torch.uint8, device="cuda")

    def upload(self):
        self.g_arena = to_dev(self.o_arena)
        self.g_sb = to_dev(self.o_sb)
        self.g_m = to_dev(self.o_m)
        self.g_v = to_dev(self.o_v)

    def step_oracle(self, g, kind, lr, t, threads=8):
        orc.step_varset(self.o_arena, self.o_table, self.o_sb, g, self.o_m, self.o_v,
                        orc.Opt(kind=kind, lr=lr, t=t), threads=threads)

    def step_gpu(self, g_dev, kind, lr, t, flags=0):
        omc.omc_step_update_recompress(self.g_arena, self.plan, self.g_sb, g_dev, self.g_m, self.g_v,
                                       omc.opt(kind, lr, t=t, flags=flags), self.ws)

    def compare(self, kind, what=""):
        """Bit-exact on the arena (codes and fp32 values) and optimizer state; returns the number
        of (s, b) entries that differ and asserts they are at most 1 ulp apart."""
        torch.cuda.synchronize()
        ga = self.g_arena.cpu().numpy()
        bad = np.nonzero(ga != self.o_arena)[0]
        assert bad.size == 0, f"{what}: arena differs at {bad.size} bytes, first {bad[:5]}"
        if kind >= 1:
            assert bits_equal(self.g_m.cpu().numpy(), self.o_m), f"{what}: state0 differs"
        if kind == 2:
            assert bits_equal(self.g_v.cpu().numpy(), self.o_v), f"{what}: state1 differs"
        gsb = self.g_sb.cpu().numpy()
        diff = gsb.view(np.int32).astype(np.int64) - self.o_sb.view(np.int32).astype(np.int64)
        both_nan = np.isnan(gsb) & np.isnan(self.o_sb)
        diff[both_nan] = 0
        assert np.all(np.abs(diff) <= 1), f"{what}: (s, b) off by more than 1 ulp: {np.abs(diff).max()}"
        return int(np.count_nonzero(diff))
