"""GPU parity of the rotary position embedding fused into the pooling pass (blossom_rope_select_blocks)
and of the backward that rotates dQ and dK back (blossom_attn_bwd_rope), against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, Dev, assert_close, host, params
from paper_2512_13368_amd import binding as B
from paper_2512_13368_amd.inputs import WORKLOADS, make_inputs, rope_tables, with_shape

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,shape", [
    ("cfg1", dict()),                                                              # scalar kernels, fp32, d = 32
    ("cfg2", dict(B=6, H=8, d=8, L=197, len_lo=30, len_hi=197, topk=4, window=8)),  # the paper's head size
    ("cfg2", dict(B=5, dtype="bf16", qkv_scaled=True)),                             # scalar kernels, bf16
    ("cfg3", dict(B=4, L=32 * 9 + 11, len_lo=40, len_hi=32 * 9 + 11)),              # matrix cores, b = 32, ragged
    ("cfg4", dict(B=2, H=2, L=64 * 9, len_lo=200, len_hi=64 * 9)),                  # matrix cores, b = 64
])
def test_rope_select_forward_backward(name, shape):
    w = with_shape(WORKLOADS[name], name=name + "-rope", **shape)
    x = make_inputs(w, want_dO=True)
    cos, sin = rope_tables(w.L, w.d)
    bf16 = w.dtype == "bf16"
    tol = TOL[w.dtype]
    print(f"rope case {w.name} B{w.B} H{w.H} L{w.L} d{w.d} b{w.block} {w.dtype}", flush=True)
    dv = Dev(x)
    cos_d, sin_d = torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda()
    p = params(w, save_for_bwd=1)
    Q_rot, K_rot, sel = B.rope_select_blocks(p, dv.Q, dv.K, cos_d, sin_d, dv.vl)
    f = B.attn_fwd(p, Q_rot, K_rot, dv.V, dv.vl, sel, dv.gw, dv.gb)
    g = B.attn_bwd(p, Q_rot, K_rot, dv.V, dv.vl, sel, dv.gw, dv.gb, f, dv.dO, rope=(cos_d, sin_d))
    g_plain = B.attn_bwd(p, Q_rot, K_rot, dv.V, dv.vl, sel, dv.gw, dv.gb, f, dv.dO)
    torch.cuda.synchronize()

    # rotated tensors: the same bits (every position, padding included); selection: exact
    Qr, Kr = oracle.rope(x.Q, cos, sin, to_bf16=bf16), oracle.rope(x.K, cos, sin, to_bf16=bf16)
    np.testing.assert_array_equal(Q_rot.float().cpu().numpy(), Qr)
    np.testing.assert_array_equal(K_rot.float().cpu().numpy(), Kr)
    sel_ref = oracle.select_blocks(Qr, Kr, x.valid_len, w.block, w.topk)
    np.testing.assert_array_equal(sel.cpu().numpy(), sel_ref)
    # the rotation changed the selection input for real
    assert not np.array_equal(Qr[:, :, 1:], x.Q[:, :, 1:])

    flat = lambda t: host(t).reshape(w.B * w.H, *t.shape[2:])
    fr = oracle.attn_fwd(Qr, Kr, x.V, x.valid_len, sel_ref, x.gate_w, x.gate_b, w.block, w.topk, w.window)
    assert_close(flat(f.O), fr.O, tol, "O")
    gr = oracle.attn_bwd(Qr, Kr, x.V, x.valid_len, sel_ref, x.gate_w, x.gate_b, x.dO, w.block, w.topk, w.window)
    assert_close(flat(g.dQ), oracle.rope_bwd(gr.dQ, cos, sin), tol, "dQ (rotated back)")
    assert_close(flat(g.dK), oracle.rope_bwd(gr.dK, cos, sin), tol, "dK (rotated back)")
    assert_close(flat(g.dV), gr.dV, tol, "dV")
    assert_close(host(g.d_gate_w), gr.d_gate_w, tol, "d_gate_w")
    # without the tables the same call gives the gradients w.r.t. the rotated tensors; dV is the same either way
    assert_close(flat(g_plain.dQ), gr.dQ, tol, "dQ (w.r.t. rotated Q)")
    assert torch.equal(g_plain.dV, g.dV)
    for r in range(w.B):  # gradients of padding stay exactly zero
        p0 = w.L - int(x.valid_len[r])
        if p0 > 0:
            assert float(g.dQ[r, :, :p0].abs().max()) == 0.0 and float(g.dK[r, :, :p0].abs().max()) == 0.0


def test_rope_serving_mode_and_random_angles():
    # serving mode rotates all of K and the last query block; arbitrary tables (not cos/sin of anything) are legal input
    w = with_shape(WORKLOADS["cfg3"], name="rope-serve", B=3, H=2, L=32 * 6 + 7, len_lo=50, len_hi=32 * 6 + 7)
    x = make_inputs(w)
    rng = np.random.default_rng(5)
    ang = rng.uniform(-3.0, 3.0, (w.L, w.d // 2))
    cos, sin = np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)
    dv = Dev(x)
    cos_d, sin_d = torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda()
    Q_all, K_all, sel_all = B.rope_select_blocks(params(w), dv.Q, dv.K, cos_d, sin_d, dv.vl)
    Q_last = torch.full_like(Q_all, 7.0)
    _, K_last, sel_last = B.rope_select_blocks(params(w, last_block_only=1), dv.Q, dv.K, cos_d, sin_d, dv.vl, Q_rot=Q_last,
                                               sel=torch.full_like(sel_all, -7))
    torch.cuda.synchronize()
    lo = (w.NB - 1) * w.block
    assert torch.equal(K_last, K_all) and torch.equal(Q_last[:, :, lo:], Q_all[:, :, lo:])
    assert bool((Q_last[:, :, :lo] == 7.0).all())
    assert torch.equal(sel_last[:, :, -1], sel_all[:, :, -1])
    np.testing.assert_array_equal(Q_all.float().cpu().numpy(), oracle.rope(x.Q, cos, sin, to_bf16=True))
