"""The library only enqueues kernels on the caller's stream (no allocation, no memset, no host
synchronisation), so its calls can be captured into a HIP graph.  Replays, with eager work and
synchronisations in between, must reproduce the eager results bit for bit."""
import numpy as np
import pytest
import torch

from paper_2205_03494_amd import omc, synth
from test_gpu_sets import build

pytestmark = pytest.mark.gpu


def test_captured_round_replays_like_eager_launches():
    specs = synth.conformer_varset(64, 2, 256, 8, frontend=False)
    fmts = [(4, 3) if i % 2 else (3, 7) for i in range(len(specs))]
    mask = synth.ppq_mask(specs, 0.8, 3)
    lay, plan = build(specs, mask, fmts)
    vals = torch.from_numpy(synth.init_values(lay, 1)).cuda()
    grads = [torch.from_numpy(synth.gradients(lay, 5e-3, 70 + k)).cuda() for k in range(2)]
    arena = torch.zeros(lay.arena_bytes, dtype=torch.uint8, device="cuda")
    sb = torch.zeros((len(specs), 2), device="cuda")
    mom = torch.zeros(lay.aux_elems, device="cuda")
    out = torch.zeros(lay.aux_elems, device="cuda")
    ws = torch.empty(max(plan.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
    o = omc.opt(omc.OMC_MOMENTUM, 0.05)
    M, N, K = 256, 128, 128
    A = torch.from_numpy(synth.to_bf16_bits(synth.normal_f32(M * K, 1.0, 5)).view(np.int16)).cuda()
    wcodes = torch.randint(0, 120, (K * N,), dtype=torch.uint8, device="cuda")
    wsb = torch.tensor([0.5, 0.125], device="cuda")
    C = torch.zeros((M, N), device="cuda")
    gws = torch.empty(omc.omc_dequant_gemm_workspace_bytes(M), dtype=torch.uint8, device="cuda")
    K2 = 2048                                        # a long contraction on a small grid (dX: the sixteen-wave kernel)
    A2 = torch.from_numpy(synth.to_bf16_bits(synth.normal_f32(M * K2, 1.0, 6)).view(np.int16)).cuda()
    wcodes2 = torch.randint(0, 120, (K2 * N,), dtype=torch.uint8, device="cuda")
    C2 = torch.zeros((M, N), device="cuda")
    dX2 = torch.zeros((M, K), device="cuda")
    dY2 = torch.from_numpy(synth.to_bf16_bits(synth.normal_f32(M * K2, 1.0, 7)).view(np.int16)).cuda()   # [M x 2048]
    wcodes3 = torch.randint(0, 120, (K * K2,), dtype=torch.uint8, device="cuda")                          # W [K x 2048]

    # the round's end: another quantized subset for the next round, and the set as one message
    mask2 = synth.ppq_mask(specs, 0.8, 4)
    lay2, plan2 = build(specs, mask2, fmts)
    rs = omc.omc_reselect_plan_build(plan, plan2)
    arena2 = torch.zeros(lay2.arena_bytes, dtype=torch.uint8, device="cuda")
    sb2 = torch.zeros((len(specs), 2), device="cuda")
    rws = torch.empty(max(rs.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
    msg = torch.zeros(omc.omc_transport_bytes(plan2), dtype=torch.uint8, device="cuda")
    n1 = 50000 + 77
    one = torch.from_numpy(synth.normal_f32(n1, 0.05, 9)).cuda()
    one_codes = torch.zeros(omc.omc_packed_bytes(omc.fmt(3, 7), n1), dtype=torch.uint8, device="cuda")
    one_sb = torch.zeros(2, device="cuda")

    def one_round(stream=None):
        # a client's round in miniature: compress the set, two training steps, a forward GEMM, decompress
        omc.omc_compress_set(vals, plan, arena, sb, ws, stream=stream)
        omc.omc_step_update_recompress(arena, plan, sb, grads[0], mom, None, o, ws, stream=stream)
        omc.omc_step_update_recompress(arena, plan, sb, grads[1], mom, None, o, ws, stream=stream)
        omc.omc_dequant_gemm(A, wcodes, omc.fmt(4, 3), wsb, C, M, N, K, gws, stream=stream)
        omc.omc_dequant_gemm(A2, wcodes2, omc.fmt(4, 3), wsb, C2, M, N, K2, gws, stream=stream)
        omc.omc_dequant_gemm_dx(dY2, wcodes3, omc.fmt(4, 3), wsb, dX2, M, K2, K, gws, stream=stream)
        omc.omc_decompress_set(arena, plan, sb, out, stream=stream)
        omc.omc_reselect(rs, arena, sb, arena2, sb2, rws, stream=stream)
        omc.omc_transport_pack(plan2, arena2, sb2, msg, stream=stream)
        omc.omc_compress_noalloc(one, n1, omc.fmt(3, 7), True, one_codes, one_sb, stream=stream)   # allocates nothing: capturable

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (arena, sb, mom, out, C, C2, dX2, arena2, sb2, msg, one_codes, one_sb)]

    mom.zero_()
    one_round()
    want = snapshot()

    cap = torch.cuda.Stream()
    cap.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    mom.zero_()
    with torch.cuda.graph(g, stream=cap):
        one_round(cap)
    for rep in range(4):
        mom.zero_()                                  # eager work between the replays
        arena.zero_(); out.zero_(); C.zero_(); C2.zero_(); dX2.zero_(); sb.zero_()
        arena2.zero_(); sb2.zero_(); msg.zero_(); one_codes.zero_(); one_sb.zero_()
        torch.cuda.synchronize()
        g.replay()
        got = snapshot()
        for a, b in zip(got, want):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"replay {rep} differs"
