"""omc_compress_noalloc (the entry point for callers that cannot allocate device memory: its workspace is a
device array inside the library) against omc_compress on the same inputs: packed codes and (s, b) bit for bit.
Two calls in a row share the array, the second on a smaller input; then a third, larger again, a format with
error-carrying sums, and the size limit."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2205_03494_amd import omc, synth
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


def both(x, gf, use_pvt=True):
    n = x.size
    xd = to_dev(x)
    nb = omc.omc_packed_bytes(gf, n)
    want_codes = torch.zeros(nb, dtype=torch.uint8, device="cuda")
    want_sb = torch.zeros(2, device="cuda")
    ws = torch.empty(omc.omc_compress_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    omc.omc_compress(xd, n, gf, use_pvt, want_codes, want_sb, ws)
    got_codes = torch.full((nb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    got_sb = torch.full((2,), float("nan"), device="cuda")
    omc.omc_compress_noalloc(xd, n, gf, use_pvt, got_codes, got_sb)
    torch.cuda.synchronize()
    assert torch.equal(got_codes[:nb], want_codes), "codes differ from omc_compress"
    assert bool((got_codes[nb:] == 0xA5).all()), "wrote past the packed buffer"
    assert torch.equal(got_sb.view(torch.int32), want_sb.view(torch.int32)), (got_sb, want_sb)
    return got_sb.cpu().numpy()


def test_two_calls_in_a_row_the_second_smaller_then_more():
    gf = omc.fmt(4, 3)
    big = synth.normal_f32(3_000_000 + 1234, 0.05, 1)        # 733 partial sums + a ragged tail
    small = synth.normal_f32(70_000 + 5, 0.2, 2)             # 18 partial sums: most of the first call's remain in the array
    sb_big = both(big, gf)
    sb_small = both(small, gf)
    assert not np.array_equal(sb_big, sb_small)
    both(synth.normal_f32(500, 0.05, 3), gf)                 # a tail alone
    both(big, omc.fmt(3, 7))
    both(synth.normal_f32(200_000 + 77, 0.05, 4), omc.fmt(4, 20))     # sums with error words
    both(small, omc.fmt(2, 3), use_pvt=False)
    sb_again = both(big, gf)
    assert np.array_equal(sb_again.view(np.uint32), sb_big.view(np.uint32))


def test_size_limit_and_argument_checks():
    gf = omc.fmt(4, 3)
    nmax = omc.omc_compress_noalloc_max_elems()
    assert omc.omc_compress_workspace_bytes(nmax) <= 2 << 20 < omc.omc_compress_workspace_bytes(nmax + 4096)
    A = 0x100000
    assert omc._compress_noalloc(A, nmax + 1, gf, 1, 0x40000000000, A, None) == 3      # beyond the array: OMC_ERR_SIZE
    assert omc._compress_noalloc(None, 10, gf, 1, A, A, None) == 1
    assert omc._compress_noalloc(A + 4, 10, gf, 1, 0x200000, A, None) == 4
    assert omc._compress_noalloc(A, 10, omc.fmt(0, 1), 1, 0x200000, A, None) == 2
