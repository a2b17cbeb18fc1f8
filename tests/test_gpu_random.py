"""GPU parity on seeded random variable sets: sizes, formats, which variables are quantized, optimizer, and the
per-variable transformation switch are all drawn from a generator, so that shapes nobody thought of (ragged
tails next to full tiles, one-element variables, every code width in one arena) go through the fused step, the
whole-set conversions and the aggregation.  Same bar as the other tests: bit-exact against the oracle."""
import numpy as np
import pytest
import torch

from oracle import omc_oracle as orc
from paper_2205_03494_amd import omc, synth
from gpu_util import VarSet, bits_equal, to_dev

pytestmark = pytest.mark.gpu

SIZES = [1, 2, 7, 31, 32, 33, 100, 511, 2047, 2048, 2049, 4096, 6000, 8191, 8192, 8193, 10240, 16384, 20000, 40961]


def random_set(seed):
    rng = np.random.default_rng(1000 + seed)
    nv = int(rng.integers(3, 13))
    specs, mask, fmts = [], [], []
    for i in range(nv):
        n = int(rng.choice(SIZES)) if rng.random() < 0.7 else int(rng.integers(1, 50000))
        q = bool(rng.random() < 0.75)
        specs.append(synth.VarSpec(f"v{i}", (n,), max(1, n // 64), q))
        mask.append(q)
        if q:
            E = int(rng.integers(1, 9))
            M = int(rng.integers(0, 24))                 # every mantissa width a format may have
            if rng.random() < 0.5:                       # the formats the paper uses come up more often
                E, M = [(4, 3), (3, 7), (5, 10), (2, 3), (4, 14), (3, 9)][int(rng.integers(0, 6))]
            fmts.append((E, M))
        else:
            fmts.append(None)
    return specs, mask, fmts, rng


@pytest.mark.parametrize("seed", range(24))
def test_random_sets_step(seed):
    specs, mask, fmts, rng = random_set(seed)
    kind = int(rng.integers(0, 3))
    lr = [0.05, 0.05, 1e-3][kind]
    use_pvt = bool(rng.random() < 0.8)
    vs = VarSet(specs, mask, fmts, seed=seed, use_pvt=use_pvt)
    for t in range(1, 4):
        g = synth.gradients(vs.lay, 0.02, 7000 + 10 * seed + t)
        vs.step_oracle(g, kind, lr, t)
        vs.step_gpu(to_dev(g), kind, lr, t)
        assert vs.compare(kind, f"seed {seed} t={t}") == 0   # (s, b) bit for bit as well


@pytest.mark.parametrize("seed", range(24, 36))
def test_random_sets_conversions(seed):
    """compress_set from the fp32 values must give the arena and table the oracle built variable by variable;
    decompress_set must give back the oracle's decompressed values."""
    specs, mask, fmts, rng = random_set(seed)
    use_pvt = bool(rng.random() < 0.8)
    vs = VarSet(specs, mask, fmts, seed=seed, use_pvt=use_pvt)
    lay = vs.lay
    arena = torch.zeros(lay.arena_bytes, dtype=torch.uint8, device="cuda")
    sb = torch.zeros((len(specs), 2), device="cuda")
    omc.omc_compress_set(to_dev(vs.init), vs.plan, arena, sb, vs.ws)
    out = torch.full((lay.aux_elems,), float("nan"), device="cuda")
    omc.omc_decompress_set(arena, vs.plan, sb, out)
    torch.cuda.synchronize()
    ga, gsb, go = arena.cpu().numpy(), sb.cpu().numpy(), out.cpu().numpy()
    for i, s in enumerate(specs):
        a, d = int(lay.aux_offset[i]), int(lay.data_offset[i])
        if mask[i]:
            of = orc.Format(*fmts[i])
            nb = orc.packed_bytes(s.n, of.bits)
            assert np.array_equal(ga[d:d + nb], vs.o_arena[d:d + nb]), f"seed {seed} variable {i}: codes"
            assert bits_equal(gsb[i], vs.o_sb[i]), f"seed {seed} variable {i}: (s, b)"
            assert bits_equal(go[a:a + s.n], orc.decompress(vs.o_arena[d:d + nb], s.n, of, vs.o_sb[i])), f"seed {seed} variable {i}"
        else:
            assert np.array_equal(ga[d:d + 4 * s.n], vs.o_arena[d:d + 4 * s.n])
            assert bits_equal(go[a:a + s.n], vs.init[a:a + s.n])


@pytest.mark.parametrize("EM", [(4, 20), (4, 23), (8, 21), (5, 23), (7, 22), (3, 18), (1, 16), (8, 16), (6, 17), (2, 19)])
def test_wide_mantissa_formats(EM):
    """With 16 or more mantissa bits the fit cancels almost everything: b = (sum V - s sum Vt) / n is a difference
    of sums that agree to ~2^-M, so plain fp64 additions are not enough; the kernels of these formats carry the
    rounding error of every addition along, and (s, b) must equal the oracle's (exactly rounded sums) bit for bit,
    in compress and after free-running steps under every optimizer."""
    from gpu_util import gpu_compress, gpu_decompress, pair
    of, gf = pair(*EM)
    n = 3 * 8192 + 2048 + 77
    x = synth.normal_f32(n, 0.05, 5 + EM[1])
    packed, sb = gpu_compress(x, gf)
    want, wsb = orc.compress(x, of)
    assert np.array_equal(packed, want)
    assert bits_equal(sb, wsb), (sb, wsb)
    assert bits_equal(gpu_decompress(packed, n, gf, sb), orc.decompress(packed, n, of, sb))
    for kind, lr in ((0, 0.05), (1, 0.05), (2, 1e-3)):
        vs = VarSet([synth.VarSpec("w", (n,), 64, True), synth.VarSpec("u", (5000,), 64, True)], [True, True], EM, seed=3)
        for t in range(1, 4):
            g = synth.gradients(vs.lay, 0.02, 800 + t)
            vs.step_oracle(g, kind, lr, t)
            vs.step_gpu(to_dev(g), kind, lr, t)
        assert vs.compare(kind, f"S1E{EM[0]}M{EM[1]} kind {kind}") == 0


@pytest.mark.parametrize("seed", range(40, 52))
def test_random_sets_aggregation(seed):
    """Random number of clients, each quantizing its own random subset of a random variable set."""
    from test_gpu_aggregate import run_case
    specs, mask, fmts, rng = random_set(seed)
    fmts = [f if f is not None else (4, 3) for f in fmts]              # a format for whoever quantizes the variable
    R = int(rng.integers(1, 9))
    masks = [np.array([bool(m and rng.random() < 0.8) for m in mask]) for _ in range(R)]
    run_case(specs, fmts, masks, seed=seed)


@pytest.mark.parametrize("seed", range(60, 72))
def test_random_gemm_shapes(seed):
    """Forward and input-gradient GEMM on random multiples of the tile sizes and random formats of at most seven
    mantissa bits, against the oracle on every row."""
    from test_gpu_gemm import check, run_gemm, run_gemm_dx
    from gpu_util import pair
    rng = np.random.default_rng(2000 + seed)
    E, Mb = int(rng.integers(1, 9)), int(rng.integers(0, 8))
    if rng.random() < 0.4:
        E, Mb = 4, 3
    of, gf = pair(E, Mb)
    M = 256 * int(rng.integers(1, 3))
    N = 128 * int(rng.integers(1, 4))
    K = 128 * int(rng.integers(1, 5)) if rng.random() < 0.7 else 2048 + 128 * int(rng.integers(0, 3))
    A = synth.to_bf16_bits(synth.normal_f32(M * K, 1.0, seed))
    W = synth.normal_f32(K * N, 1 / np.sqrt(K), seed + 1)
    packed, sb = orc.compress(W, of)
    if (E, Mb) == (4, 3) and rng.random() < 0.5:                        # plant a top code: the generic decode must take over
        codes = orc.unpack(packed, K * N, 8)
        codes[int(rng.integers(0, K * N))] = 0x7F
        packed = orc.pack(codes, 8)
    C = run_gemm(A, packed, gf, sb, M, N, K)
    check(C, orc.dequant_gemm(A, packed, of, sb, M, N, K, threads=8), (0, M))
    dY = synth.to_bf16_bits(synth.normal_f32(M * N, 1.0, seed + 2))
    dX = run_gemm_dx(dY, packed, gf, sb, M, N, K)
    check(dX, orc.dequant_gemm_dx(dY, packed, of, sb, M, N, K, threads=8), (0, M))


@pytest.mark.parametrize("seed", range(80, 90))
def test_random_weight_gradient_steps(seed):
    """The fused weight-gradient step on random shapes, formats, optimizers: the two-stage check of test_gpu_dw."""
    from test_gpu_dw import run_case
    rng = np.random.default_rng(3000 + seed)
    EM = [(4, 3), (3, 7), (2, 3), (4, 14), (5, 10), (5, 2), (8, 7), (6, 9), (4, 18), (8, 23)][int(rng.integers(0, 10))]
    M = 32 * int(rng.integers(1, 40))
    N = 128 * int(rng.integers(1, 4))
    K = 256 * int(rng.integers(1, 3))
    kind = int(rng.integers(0, 3))
    run_case(EM, M, N, K, kind, [0.05, 0.05, 1e-3][kind], use_pvt=bool(rng.random() < 0.8), steps=2)


@pytest.mark.parametrize("kind,lr,EM", [(0, 0.01, (4, 3)), (1, 0.01, (3, 7)), (2, 1e-3, (4, 3))])
def test_hundred_free_running_steps(kind, lr, EM):
    """BASELINE config 2 runs 100 update / recompress iterations: a small Conformer-shaped set stepped 100 times on
    both sides without ever resynchronising; codes, fp32 variables, optimizer state and (s, b) must still be
    identical at the end (any earlier difference would have grown)."""
    specs = synth.conformer_varset(64, 2, 256, 8, frontend=True)
    mask = synth.ppq_mask(specs, 1.0, 0)
    vs = VarSet(specs, mask, EM, seed=21)
    grads = [synth.gradients(vs.lay, 1e-3, 9000 + k) for k in range(4)]
    g_dev = [to_dev(g) for g in grads]
    for t in range(1, 101):
        vs.step_oracle(grads[t % 4], kind, lr, t)
        vs.step_gpu(g_dev[t % 4], kind, lr, t)
    assert vs.compare(kind, "after 100 steps") == 0
