"""GPU parity of the dequant-fused forward GEMM against the oracle's fp64 GEMM on the decompressed
weights.  Tolerance (the reading of "relative tolerance 1e-3"): |C - C_ref| <= 1e-3 |C_ref| + 1e-3 rms(C_ref)."""
import numpy as np
import pytest
import torch

from oracle import omc_oracle as orc
from paper_2205_03494_amd import omc, synth
from gpu_util import pair, to_dev

pytestmark = pytest.mark.gpu


def run_gemm(A_bits, packed, gf, sb, M, N, K):
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(omc.omc_dequant_gemm_workspace_bytes(M), dtype=torch.uint8, device="cuda")
    omc.omc_dequant_gemm(to_dev(A_bits), to_dev(packed), gf, None if sb is None else to_dev(sb), C, M, N, K, ws)
    torch.cuda.synchronize()
    return C.cpu().numpy()


def tile_sample_rows(M, seed, tile=256, per_quarter=1):
    """Rows to check at full size: from every 256-row tile of the output one row out of each 64-row quarter (the
    share of one wave of the four-wave kernels), at seeded offsets."""
    rng = np.random.default_rng(seed)
    rows = [t * tile + 64 * q + int(rng.integers(0, 64)) for t in range(M // tile) for q in range(4) for _ in range(per_quarter)]
    return np.array(sorted(set(rows)))


def check_rows(C, ref, rows):
    """check() on a list of rows: ref holds the oracle's result for exactly those rows, in order."""
    return check(C[rows], ref, (0, len(rows)))


def check(C, ref, rows):
    ref = np.asarray(ref)
    got = C[rows[0]:rows[1]].astype(np.float64)
    rms = np.sqrt(np.mean(ref ** 2))
    err = np.abs(got - ref)
    assert np.all(err <= 1e-3 * np.abs(ref) + 1e-3 * rms), float((err / (np.abs(ref) + rms)).max())
    return float(np.linalg.norm(got - ref) / np.linalg.norm(ref))


@pytest.mark.parametrize("EM", [(4, 3), (5, 2), (3, 4), (2, 3), (3, 7), (8, 7), (4, 3, 4)])
@pytest.mark.parametrize("shape", [(256, 128, 32), (256, 256, 96), (512, 128, 160), (256, 128, 2048), (512, 256, 2112)])
def test_small_shapes_all_rows(EM, shape):
    of, gf = pair(*EM)
    M, N, K = shape
    A = synth.to_bf16_bits(synth.normal_f32(M * K, 1.0, 1))
    W = synth.normal_f32(K * N, 1 / np.sqrt(K), 2)
    packed, sb = orc.compress(W, of)
    C = run_gemm(A, packed, gf, sb, M, N, K)
    rel = check(C, orc.dequant_gemm(A, packed, of, sb, M, N, K, threads=8), (0, M))
    assert rel < 1e-5
    # without the transformation
    C = run_gemm(A, packed, gf, None, M, N, K)
    check(C, orc.dequant_gemm(A, packed, of, None, M, N, K, threads=8), (0, M))


def test_identity_pattern_pins_the_tile_layout():
    # A = one-hot rows, W = distinct representable values: C must reproduce W's rows exactly
    of, gf = pair(4, 3)
    M, N, K = 256, 128, 64
    A = np.zeros((M, K), np.float32)
    A[np.arange(M), np.arange(M) % K] = 1.0
    codes = (np.arange(K * N) * 7 + 3) % 120 + 1
    W = orc.decode(codes.astype(np.uint32), of)
    packed = orc.pack(codes.astype(np.uint32), 8)
    C = run_gemm(synth.to_bf16_bits(A.ravel()), packed, gf, None, M, N, K)
    want = W.reshape(K, N)[np.arange(M) % K]
    assert np.array_equal(C, want)


@pytest.mark.parametrize("shape", [(8192, 4096, 1024), (8192, 1024, 4096)])
def test_config5_shapes_sampled_rows(shape):
    M, N, K = shape
    of, gf = pair(4, 3)
    A = synth.to_bf16_bits(synth.normal_f32(M * K, 1.0, 11))
    W = synth.normal_f32(K * N, 1 / np.sqrt(K), 12)
    packed, sb = orc.compress(W, of)
    C = run_gemm(A, packed, gf, sb, M, N, K)
    assert np.all(np.isfinite(C))
    # rows of C depend on their own row of A only: the oracle multiplies the sampled rows as a matrix of their own
    rows = tile_sample_rows(M, seed=K)
    assert rows.size == 4 * (M // 256)
    ref = orc.dequant_gemm(np.ascontiguousarray(A.reshape(M, K)[rows]).ravel(), packed, of, sb, rows.size, N, K, threads=8)
    assert check_rows(C, ref, rows) < 1e-5
    for r0 in (0, M - 24):                                      # and two runs of consecutive rows at the ends
        ref = orc.dequant_gemm(A, packed, of, sb, M, N, K, rows=(r0, r0 + 24), threads=8)
        assert check(C, ref, (r0, r0 + 24)) < 1e-5


@pytest.mark.parametrize("K", [256, 2048])                  # 2048: the kernel for long contractions on small grids
@pytest.mark.parametrize("top_at", [None, 0, -1, 12345])
def test_every_byte_code_exact_with_and_without_the_top_code(top_at, K):
    """S1E4M3 / bias 7 takes the hardware FP8 conversion unless the weights hold a top code (value 480);
    the pre-pass must find one anywhere in the stream, and both decodes must give the exact code values."""
    of, gf = pair(4, 3)
    M, N = 256, 128
    A = np.zeros((M, K), np.float32)
    pick = (np.arange(M) * 7 + 3) % K
    A[np.arange(M), pick] = 1.0
    codes = ((np.arange(K * N, dtype=np.int64) * 37 + 11) % 254).astype(np.uint32)
    codes = np.where(codes >= 127, codes + 1, codes)          # 0..126, 128..254: no top code, both signs, subnormals
    if top_at is not None:
        codes[top_at] = 0x7F if top_at != -1 else 0xFF
    W = orc.decode(codes, of)
    C = run_gemm(synth.to_bf16_bits(A.ravel()), orc.pack(codes, 8), gf, None, M, N, K)
    want = W.reshape(K, N)[pick]
    assert np.array_equal(C, want)


def run_gemm_dx(dY_bits, packed, gf, sb, M, N, K):
    dX = torch.full((M, K), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(omc.omc_dequant_gemm_workspace_bytes(M), dtype=torch.uint8, device="cuda")
    omc.omc_dequant_gemm_dx(to_dev(dY_bits), to_dev(packed), gf, None if sb is None else to_dev(sb), dX, M, N, K, ws)
    torch.cuda.synchronize()
    return dX.cpu().numpy()


@pytest.mark.parametrize("EM", [(4, 3), (5, 2), (2, 3), (3, 7), (8, 7), (4, 3, 4)])
@pytest.mark.parametrize("shape", [(256, 32, 128), (256, 96, 256), (512, 160, 128), (256, 2048, 128), (512, 2112, 256)])
def test_dx_small_shapes_all_rows(EM, shape):
    of, gf = pair(*EM)
    M, N, K = shape
    dY = synth.to_bf16_bits(synth.normal_f32(M * N, 1.0, 5))
    W = synth.normal_f32(K * N, 1 / np.sqrt(K), 2)
    packed, sb = orc.compress(W, of)
    dX = run_gemm_dx(dY, packed, gf, sb, M, N, K)
    rel = check(dX, orc.dequant_gemm_dx(dY, packed, of, sb, M, N, K, threads=8), (0, M))
    assert rel < 1e-5
    dX = run_gemm_dx(dY, packed, gf, None, M, N, K)
    check(dX, orc.dequant_gemm_dx(dY, packed, of, None, M, N, K, threads=8), (0, M))


@pytest.mark.parametrize("N", [64, 2048])                   # 2048: the kernel for long contractions on small grids
@pytest.mark.parametrize("top_at", [None, 777])
def test_dx_identity_pattern_pins_the_transposed_layout(top_at, N):
    # dY = one-hot rows: dX must reproduce columns of W exactly, with and without a top code (both decodes)
    of, gf = pair(4, 3)
    M, K = 256, 128
    dY = np.zeros((M, N), np.float32)
    pick = (np.arange(M) * 5 + 1) % N
    dY[np.arange(M), pick] = 1.0
    codes = ((np.arange(K * N, dtype=np.int64) * 37 + 11) % 254).astype(np.uint32)
    codes = np.where(codes >= 127, codes + 1, codes)
    if top_at is not None:
        codes[top_at] = 0x7F
    W = orc.decode(codes, of).reshape(K, N)
    dX = run_gemm_dx(synth.to_bf16_bits(dY.ravel()), orc.pack(codes, 8), gf, None, M, N, K)
    want = W[:, pick].T
    assert np.array_equal(dX, want)


@pytest.mark.parametrize("shape", [(8192, 4096, 1024), (8192, 1024, 4096)])
def test_dx_config5_shapes_sampled_rows(shape):
    M, N, K = shape
    of, gf = pair(4, 3)
    dY = synth.to_bf16_bits(synth.normal_f32(M * N, 1.0, 13))
    W = synth.normal_f32(K * N, 1 / np.sqrt(K), 12)
    packed, sb = orc.compress(W, of)
    dX = run_gemm_dx(dY, packed, gf, sb, M, N, K)
    assert np.all(np.isfinite(dX))
    rows = tile_sample_rows(M, seed=N)
    ref = orc.dequant_gemm_dx(np.ascontiguousarray(dY.reshape(M, N)[rows]).ravel(), packed, of, sb, rows.size, N, K, threads=8)
    assert check_rows(dX, ref, rows) < 1e-5
    for r0 in (0, M - 24):
        ref = orc.dequant_gemm_dx(dY, packed, of, sb, M, N, K, rows=(r0, r0 + 24), threads=8)
        assert check(dX, ref, (r0, r0 + 24)) < 1e-5


@pytest.mark.parametrize("shape", [(256, 128, 32), (512, 256, 160), (256, 128, 4096), (256, 2048, 128)])
def test_large_offset_makes_the_row_sum_term_count(shape):
    """With the fitted (s, b) of zero-mean weights b is tiny and the b * rowsum(A) term hides inside the tolerance;
    a hand-made pair with a large offset makes both GEMMs depend on their row sums."""
    of, gf = pair(4, 3)
    M, N, K = shape
    A = synth.to_bf16_bits(synth.normal_f32(M * K, 1.0, 1) + np.float32(0.5))
    W = synth.normal_f32(K * N, 1 / np.sqrt(K), 2)
    packed, _ = orc.compress(W, of)
    sb = np.array([0.75, 0.125], np.float32)
    C = run_gemm(A, packed, gf, sb, M, N, K)
    check(C, orc.dequant_gemm(A, packed, of, sb, M, N, K, threads=8), (0, M))
    dY = synth.to_bf16_bits(synth.normal_f32(M * N, 1.0, 5) + np.float32(0.5))
    dX = run_gemm_dx(dY, packed, gf, sb, M, N, K) if K % 128 == 0 else None
    if dX is not None:
        check(dX, orc.dequant_gemm_dx(dY, packed, of, sb, M, N, K, threads=8), (0, M))
