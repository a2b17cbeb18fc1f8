"""GPU parity of the fused backward step of a linear layer (weight gradient on the matrix cores,
consumed by the update in the same kernel).  Two-stage check, because the gradient is a long fp32
accumulation while the update decides integer codes:
  1. the gradient the kernel used (dW_out) against the oracle's fp64 X^T dY, to the GEMM tolerance;
  2. codes, (s, b) and optimizer state against the oracle's step fed with exactly that gradient: bit for bit.
Every case is run a second time on its own copies of the buffers with dW_out = NULL -- the call a training loop
makes, where the gradient is not written anywhere -- and must leave the same codes, (s, b) and state, bit for bit."""
import numpy as np
import pytest
import torch

from oracle import omc_oracle as orc
from paper_2205_03494_amd import omc, synth
from gpu_util import bits_equal, pair, to_dev
from test_gpu_gemm import check

pytestmark = pytest.mark.gpu


def run_case(EM, M, N, K, kind, lr, use_pvt=True, steps=2, grad_scale=1.0, rows=None):
    want_dw = True
    of, gf = pair(*EM)
    n = K * N
    W = synth.normal_f32(n, 0.05, 2)
    packed, sb = orc.compress(W, of, use_pvt=use_pvt)
    st0 = np.zeros(n, np.float32) if kind >= 1 else None
    st1 = np.zeros(n, np.float32) if kind == 2 else None
    codes_d, sb_d = to_dev(packed), to_dev(sb)
    st0_d = None if st0 is None else to_dev(st0)
    st1_d = None if st1 is None else to_dev(st1)
    ws = torch.empty(omc.omc_dw_update_workspace_bytes(gf, M, N, K), dtype=torch.uint8, device="cuda")
    dW_d = torch.full((K, N), float("nan"), device="cuda") if want_dw else None
    # the same steps without a gradient copy, on separate buffers (workspace included)
    codes_n, sb_n = codes_d.clone(), sb_d.clone()
    st0_n = None if st0_d is None else st0_d.clone()
    st1_n = None if st1_d is None else st1_d.clone()
    ws_n = torch.empty_like(ws)
    for t in range(1, steps + 1):
        X = synth.to_bf16_bits(synth.normal_f32(M * K, 1.0, 10 + t))
        dY = synth.to_bf16_bits(synth.normal_f32(M * N, grad_scale / M, 20 + t))
        X_d, dY_d = to_dev(X), to_dev(dY)
        omc.omc_dw_update_recompress(X_d, dY_d, codes_d, gf, sb_d, use_pvt, st0_d, st1_d,
                                     omc.opt(kind, lr, t=t), dW_d, M, N, K, ws)
        omc.omc_dw_update_recompress(X_d, dY_d, codes_n, gf, sb_n, use_pvt, st0_n, st1_n,
                                     omc.opt(kind, lr, t=t), None, M, N, K, ws_n)
        torch.cuda.synchronize()
        assert torch.equal(codes_n, codes_d), f"dW_out = NULL: codes differ at step {t}"
        assert torch.equal(sb_n.view(torch.int32), sb_d.view(torch.int32)), f"dW_out = NULL: (s, b) differ at step {t}"
        if st0_d is not None:
            assert torch.equal(st0_n.view(torch.int32), st0_d.view(torch.int32)), f"dW_out = NULL: state0 differs at step {t}"
        if st1_d is not None:
            assert torch.equal(st1_n.view(torch.int32), st1_d.view(torch.int32)), f"dW_out = NULL: state1 differs at step {t}"
        g = dW_d.cpu().numpy()
        assert np.all(np.isfinite(g))
        if rows is None:
            check(g, orc.gemm_dw(X, dY, M, N, K, threads=8), (0, K))
        else:
            for r0 in rows:
                check(g, orc.gemm_dw(X, dY, M, N, K, rows=(r0, r0 + 16), threads=8), (r0, r0 + 16))
        orc.step_quantized(packed, n, of, sb, g.ravel(), st0, st1, orc.Opt(kind=kind, lr=lr, t=t), use_pvt=use_pvt)
        assert np.array_equal(codes_d.cpu().numpy(), packed), f"codes differ at step {t}"
        assert bits_equal(sb_d.cpu().numpy(), sb), (sb_d.cpu().numpy(), sb)
        if st0 is not None:
            assert bits_equal(st0_d.cpu().numpy(), st0)
        if st1 is not None:
            assert bits_equal(st1_d.cpu().numpy(), st1)


@pytest.mark.parametrize("kind,lr", [(0, 0.05), (1, 0.05), (2, 1e-3)])
@pytest.mark.parametrize("EM", [(4, 3), (5, 2), (3, 4), (4, 3, 4)])
def test_small_shapes(EM, kind, lr):
    run_case(EM, 96, 128, 256, kind, lr)


@pytest.mark.parametrize("shape", [(32, 128, 256), (160, 256, 512), (64, 384, 256)])
def test_tile_grid_and_minimal_contraction(shape):
    M, N, K = shape
    run_case((4, 3), M, N, K, 0, 0.05)


@pytest.mark.parametrize("M,kind,lr", [(1024, 0, 0.05), (4096, 1, 0.05), (2048, 2, 1e-3)])
def test_contraction_split_between_workgroups(M, kind, lr):
    """Few tiles and many rows: the M rows are shared out between workgroups and the last one to arrive at a
    tile sums the partial accumulators in a fixed order; two runs must agree bit for bit with each other
    (run_case compares the second step too) and with the oracle's step on the gradient that was used."""
    run_case((4, 3), M, 128, 256, kind, lr, steps=2)
    run_case((4, 3), M, 256, 512, kind, lr, steps=1)


def test_without_the_transformation_and_with_saturating_updates():
    run_case((4, 3), 64, 128, 256, 0, 0.05, use_pvt=False)
    run_case((2, 5), 64, 128, 256, 0, 50.0, grad_scale=100.0)      # most weights end at the format's limits


def test_config5_layer_sampled_gradient_rows():
    # the feed-forward layer of the benchmark shape: X [8192 x 1024], W [1024 x 4096]
    run_case((4, 3), 8192, 4096, 1024, 0, 0.01, steps=1, rows=(0, 300, 500, 700, 1008))   # every 256-row tile, full width


@pytest.mark.parametrize("kind,lr", [(0, 0.05), (1, 0.05), (2, 1e-3)])
@pytest.mark.parametrize("EM", [(3, 7), (2, 3), (5, 7), (4, 14), (8, 7), (5, 10)])
def test_other_code_widths_take_the_two_kernel_path(EM, kind, lr):
    """6-, 11-, 13-, 16- and 19-bit formats: the accumulators pass through the workspace and the slab kernel
    updates the rows; same two-stage check."""
    run_case(EM, 96, 128, 256, kind, lr)


def test_other_code_widths_with_split_contraction_and_several_tiles():
    run_case((3, 7), 2048, 256, 512, 1, 0.05, steps=2)
    run_case((2, 3), 1024, 128, 256, 0, 0.05, steps=2, grad_scale=20.0)


@pytest.mark.parametrize("EM", [(4, 18), (5, 23), (8, 16)])
def test_wide_mantissa_formats_keep_exact_fit_sums(EM):
    """16 and more mantissa bits: the slab kernel carries the rounding errors of the fit's sums like the streaming
    kernels of these formats do, so (s, b) still match the oracle bit for bit."""
    run_case(EM, 96, 128, 256, 1, 0.05)
    run_case(EM, 1024, 256, 512, 0, 0.05, steps=1)


def test_fp32_as_a_format_is_plain_sgd():
    """S1E8M23 stores fp32 itself; without the transformation the fused step must equal w - lr * dW in fp32."""
    M, N, K = 64, 128, 256
    gf = omc.fmt(8, 23)
    W = synth.normal_f32(K * N, 0.05, 2)
    codes = to_dev(W.view(np.uint8).copy())
    sb = torch.tensor([1.0, 0.0], device="cuda")
    X = synth.to_bf16_bits(synth.normal_f32(M * K, 1.0, 11))
    dY = synth.to_bf16_bits(synth.normal_f32(M * N, 1.0 / M, 21))
    ws = torch.empty(omc.omc_dw_update_workspace_bytes(gf, M, N, K), dtype=torch.uint8, device="cuda")
    dW = torch.zeros((K, N), device="cuda")
    omc.omc_dw_update_recompress(to_dev(X), to_dev(dY), codes, gf, sb, False, None, None, omc.opt(0, 0.05), dW, M, N, K, ws)
    torch.cuda.synchronize()
    g = dW.cpu().numpy().ravel()
    step = (np.float32(0.05) * g).astype(np.float32)
    want = (W - step).astype(np.float32)
    assert bits_equal(codes.cpu().numpy().view(np.float32), want)
    assert sb.cpu().numpy().tolist() == [1.0, 0.0]


def test_large_matrix_takes_the_in_kernel_epilogue_on_256_row_tiles():
    # 4096 x 4096 weights = 512 tiles of 256 x 128: no split, the update runs in the GEMM kernel's epilogue
    run_case((4, 3), 64, 4096, 4096, 1, 0.05, steps=1, rows=(0, 2000, 4080))


@pytest.mark.parametrize("EM,kind,lr", [((4, 3), 0, 0.05), ((3, 7), 1, 0.05), ((2, 3), 2, 1e-3)])
def test_long_contraction_on_a_small_grid_takes_the_sixteen_wave_kernel(EM, kind, lr):
    """64 tiles and 4096 rows: two workgroups of 16 waves per tile (eight multiplying, eight staging), each over
    2048 rows; the accumulators pass through the workspace in the four-wave kernel's layout."""
    run_case(EM, 4096, 2048, 1024, kind, lr, steps=2, rows=(0, 16, 320, 1008))
