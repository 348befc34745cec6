"""blossom_select_blocks_static (the entry point that allocates nothing) against blossom_select_blocks
and the oracle: two calls in a row on one GPU, the second with a smaller input, so that whatever the
first call left in the library's static scratch array must not leak into the second."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from gpu_util import Dev, params
from paper_2512_13368_amd import binding as B
from paper_2512_13368_amd.inputs import WORKLOADS, make_inputs, with_shape


def _both(w):
    x = make_inputs(w)
    dv = Dev(x)
    p = params(w)
    want = B.select_blocks(p, dv.Q, dv.K, dv.vl)
    got = torch.full_like(want, -9)
    print(f"static select {w.name} B{w.B} H{w.H} L{w.L} d{w.d} b{w.block} k{w.topk} {w.dtype}", flush=True)
    B.select_blocks_static(p, dv.Q, dv.K, dv.vl, got)
    torch.cuda.synchronize()
    assert torch.equal(got, want)
    np.testing.assert_array_equal(got.cpu().numpy(), oracle.select_blocks(x.Q, x.K, x.valid_len, w.block, w.topk))


@pytest.mark.gpu
def test_static_scratch_two_calls_second_smaller():
    big = with_shape(WORKLOADS["cfg3"], name="static-big", B=16)                        # 1 MiB of scratch
    small = with_shape(WORKLOADS["cfg1"], name="static-small", B=3, L=45, len_lo=3, len_hi=45)
    _both(big)
    _both(small)
    _both(with_shape(WORKLOADS["cfg2"], name="static-fp32", B=8))
    _both(WORKLOADS["cfg4"])                                                            # 8 MiB: the largest benchmark shape


def test_static_scratch_rejects_sizes_beyond_its_maximum():
    # 8*B*H*NB*d = 8*64*8*128*64 = 32 MiB > 16 MiB: refused before anything is launched (fake pointers)
    p = B.Params(64, 8, 8192, 64, 64, 16, 128, B.BF16)
    cp = p.c()
    vp = ctypes.c_void_p
    rc = B.lib().blossom_select_blocks_static(ctypes.byref(cp), vp(16), vp(16), vp(16), vp(16), None)
    assert rc == -8 and "16 MiB" in B.strerror(rc)
