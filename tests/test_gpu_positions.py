"""GPU parity of blossom_select_positions (the selection rule as printed, Eq. 8-13) with the oracle: the
selected block ids must agree bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import to_dev
from paper_2512_13368_amd import binding as B
from paper_2512_13368_amd.inputs import round_to_bf16

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,Bn,H,G,L,d,l,s,lsel,k,scale", [
    ("fp32", 3, 8, 4, 200, 8, 32, 16, 16, 4, 0.0),     # the paper's own setting (Appendix E): hidden 64 over 8 heads, 4 groups
    ("fp32", 2, 8, 2, 100, 16, 32, 16, 16, 4, 0.0),    # 2 key/value heads
    ("bf16", 2, 4, 4, 333, 64, 32, 16, 64, 6, 0.125),  # no sharing, l' = 64 (four stride steps per selection block), scaled scores
    ("bf16", 2, 4, 1, 1000, 32, 8, 8, 8, 5, 0.0),      # l = s = l' (no overlap), one group of four heads, 125 blocks: two candidate slots
    ("fp32", 2, 2, 2, 50, 32, 16, 4, 8, 3, 1.0),       # l > l', four-fold overlap
    ("fp32", 1, 2, 1, 20, 8, 32, 16, 16, 4, 0.0),      # shorter than one compression block: own block only
    ("bf16", 1, 2, 2, 4096, 64, 32, 16, 16, 16, 0.0),  # 256 selection blocks, 255 compression blocks
    ("fp32", 2, 4, 2, 1024, 16, 32, 16, 16, 5, 0.0),   # 64 selection blocks, 63 compression blocks: the longest a lane per position takes
    ("fp32", 2, 4, 2, 1040, 16, 32, 16, 16, 5, 0.0),   # one selection block more: a wavefront per position
    ("bf16", 3, 6, 2, 257, 32, 16, 8, 16, 8, 0.5),     # three heads per group, k beyond the candidates of early positions
])
def test_select_positions_matches_the_oracle(dtype, Bn, H, G, L, d, l, s, lsel, k, scale):
    rng = np.random.default_rng(31 + L + d + k)
    Q = rng.standard_normal((Bn, H, L, d)).astype(np.float32)
    K = rng.standard_normal((Bn, G, L, d)).astype(np.float32)
    if dtype == "bf16":
        Q, K = round_to_bf16(Q / np.sqrt(d)), round_to_bf16(K / np.sqrt(d))
    vl = rng.integers(1, L + 1, Bn).astype(np.int32)
    vl[0] = L
    print(f"positions case {dtype} B{Bn} H{H} G{G} L{L} d{d} l{l} s{s} l'{lsel} k{k}", flush=True)
    p = B.Params(Bn, H, L, d, lsel, k, 1, B.F32 if dtype == "fp32" else B.BF16)
    got = B.select_positions(p, G, l, s, to_dev(Q, dtype), to_dev(K, dtype), torch.from_numpy(vl).cuda(), score_scale=scale)
    torch.cuda.synchronize()
    ref = oracle.select_positions(Q, K, vl, l, s, lsel, k, score_scale=(scale if scale > 0 else 1.0))
    np.testing.assert_array_equal(got.cpu().numpy(), ref)


def test_select_positions_ties_and_limits():
    # equal keys everywhere: every score ties, the lowest block indices must win at every position
    Bn, H, G, L, d = 1, 2, 1, 96, 8
    Q = np.ones((Bn, H, L, d), np.float32)
    K = np.ones((Bn, G, L, d), np.float32)
    vl = np.array([L], np.int32)
    p = B.Params(Bn, H, L, d, 8, 3, 1, B.F32)
    got = B.select_positions(p, G, 8, 4, to_dev(Q, "fp32"), to_dev(K, "fp32"), torch.from_numpy(vl).cuda())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got.cpu().numpy(), oracle.select_positions(Q, K, vl, 8, 4, 8, 3))
    with pytest.raises(B.BlossomError):   # more than 512 selection blocks
        B.select_positions(B.Params(1, 2, 8 * 600, 8, 8, 3, 1, B.F32), 1, 8, 4, torch.zeros((1, 2, 4800, 8), device="cuda"),
                           torch.zeros((1, 1, 4800, 8), device="cuda"), torch.tensor([4800], dtype=torch.int32, device="cuda"))
    with pytest.raises(B.BlossomError):   # stride must divide both block sizes
        B.select_positions(B.Params(1, 2, 64, 8, 8, 3, 1, B.F32), 1, 8, 3, torch.zeros((1, 2, 64, 8), device="cuda"),
                           torch.zeros((1, 1, 64, 8), device="cuda"), torch.tensor([64], dtype=torch.int32, device="cuda"))


@pytest.mark.parametrize("dtype,Bn,H,G,L,d,l,s,lsel,k,window,stis_mode,stis_block", [
    ("fp32", 3, 8, 4, 200, 8, 32, 16, 16, 4, 8, 1, 1),    # the paper's own setting: hidden 64 over 8 heads, mask block 1, window 8
    ("fp32", 2, 8, 2, 100, 16, 32, 16, 16, 4, 8, 0, 0),   # 2 key/value heads, plain window
    ("fp32", 2, 4, 1, 197, 32, 16, 8, 8, 3, 12, 0, 0),    # one group of four heads, selection block 8, ragged tail
    ("bf16", 2, 4, 4, 333, 16, 32, 16, 16, 6, 20, 1, 16),  # bf16 storage, no sharing, mask block = selection block
])
def test_attention_under_a_per_position_selection(dtype, Bn, H, G, L, d, l, s, lsel, k, window, stis_mode, stis_block):
    # the printed path end to end on the GPU: blossom_select_positions -> blossom_attn_fwd_positions, against
    # the oracle's attention under the same per-position selection (its K, V and selection rows repeated per head)
    from gpu_util import TOL, assert_close, host
    rng = np.random.default_rng(77 + L + d + k)
    Q = rng.standard_normal((Bn, H, L, d)).astype(np.float32)
    K = rng.standard_normal((Bn, G, L, d)).astype(np.float32)
    V = rng.standard_normal((Bn, G, L, d)).astype(np.float32)
    if dtype == "bf16":
        Q, K, V = (round_to_bf16(x / np.sqrt(d)) for x in (Q, K, V))
    gw = (rng.standard_normal((H, 2 * d)) * 0.3).astype(np.float32)
    gb = (rng.standard_normal(H) * 0.5).astype(np.float32)
    vl = rng.integers(1, L + 1, Bn).astype(np.int32)
    vl[0] = L
    print(f"per-position attention {dtype} B{Bn} H{H} G{G} L{L} d{d} l'{lsel} k{k} w{window} stis {stis_mode}/{stis_block}", flush=True)
    dt = B.F32 if dtype == "fp32" else B.BF16
    p_sel = B.Params(Bn, H, L, d, lsel, k, 1, dt)
    p = B.Params(Bn, H, L, d, lsel, k, window, dt, stis_mode=stis_mode, stis_block=stis_block)
    Qd, Kd, Vd = to_dev(Q, dtype), to_dev(K, dtype), to_dev(V, dtype)
    vld = torch.from_numpy(vl).cuda()
    sel_pos = B.select_positions(p_sel, G, l, s, Qd, Kd, vld)
    f = B.attn_fwd_positions(p, G, Qd, Kd, Vd, vld, sel_pos, torch.from_numpy(gw).cuda(), torch.from_numpy(gb).cuda(),
                             want_branches=True)
    torch.cuda.synchronize()
    sel_ref = oracle.select_positions(Q, K, vl, l, s, lsel, k)
    np.testing.assert_array_equal(sel_pos.cpu().numpy(), sel_ref)
    rep = H // G
    fr = oracle.attn_fwd(Q, np.repeat(K, rep, 1), np.repeat(V, rep, 1), vl, np.repeat(sel_ref, rep, 1), gw, gb, lsel, k, window,
                         per_position=True, stis_block=(stis_block if stis_mode else 0))
    tol = TOL[dtype]
    flat = lambda t: host(t).reshape(Bn * H, *t.shape[2:])
    assert_close(flat(f.o_lt), fr.o_lt, tol, "o_lt")
    assert_close(flat(f.o_st), fr.o_st, tol, "o_st")
    assert_close(flat(f.O), fr.O, tol, "O")
    assert_close(flat(f.lse_lt), fr.lse_lt, tol, "lse_lt")
    assert_close(flat(f.lse_st), fr.lse_st, tol, "lse_st")
    for r in range(Bn):   # pad rows are exactly zero
        p0 = L - int(vl[r])
        if p0 > 0:
            assert float(f.O[r, :, :p0].float().abs().max()) == 0.0
    # the same call without the branch outputs gives the same O
    f2 = B.attn_fwd_positions(p, G, Qd, Kd, Vd, vld, sel_pos, torch.from_numpy(gw).cuda(), torch.from_numpy(gb).cuda())
    assert torch.equal(f2.O, f.O)


@pytest.mark.parametrize("dtype,Bn,H,G,L,d,l,s,lsel,k,window,stis_mode,stis_block", [
    ("fp32", 3, 8, 4, 200, 8, 32, 16, 16, 4, 8, 1, 1),     # the paper's own setting: hidden 64 over 8 heads, 4 groups
    ("fp32", 3, 8, 2, 100, 16, 32, 16, 16, 4, 8, 0, 0),    # four heads per key/value head, plain window
    ("fp32", 2, 4, 1, 197, 32, 16, 8, 8, 3, 12, 0, 0),     # one group, selection block 8: 25 key blocks over 8 wavefronts, ragged tail
    ("bf16", 2, 4, 4, 333, 16, 32, 16, 16, 6, 20, 1, 16),  # bf16 storage, no sharing, three rounds of key blocks
    ("fp32", 2, 2, 1, 16, 16, 16, 16, 16, 1, 1, 0, 0),     # one block, own block only, self only
])
def test_backward_under_a_per_position_selection(dtype, Bn, H, G, L, d, l, s, lsel, k, window, stis_mode, stis_block):
    # forward + backward under the selection blossom_select_positions writes, against the oracle's backward under
    # the same per-position rows (its K, V and rows repeated per head; the gradients of a shared key head added up)
    from gpu_util import TOL, assert_close, host
    rng = np.random.default_rng(177 + L + d + k)
    Q = rng.standard_normal((Bn, H, L, d)).astype(np.float32)
    K = rng.standard_normal((Bn, G, L, d)).astype(np.float32)
    V = rng.standard_normal((Bn, G, L, d)).astype(np.float32)
    dO = rng.standard_normal((Bn, H, L, d)).astype(np.float32)
    if dtype == "bf16":
        Q, K, V, dO = (round_to_bf16(x / np.sqrt(d)) for x in (Q, K, V, dO))
    gw = (rng.standard_normal((H, 2 * d)) * 0.3).astype(np.float32)
    gb = (rng.standard_normal(H) * 0.5).astype(np.float32)
    vl = rng.integers(1, L + 1, Bn).astype(np.int32)
    vl[0] = L
    if Bn > 2:
        vl[2] = min(L, lsel + 3)     # a row whose first blocks hold no valid position
    print(f"per-position backward {dtype} B{Bn} H{H} G{G} L{L} d{d} l'{lsel} k{k} w{window} stis {stis_mode}/{stis_block}", flush=True)
    dt = B.F32 if dtype == "fp32" else B.BF16
    p_sel = B.Params(Bn, H, L, d, lsel, k, 1, dt)
    p = B.Params(Bn, H, L, d, lsel, k, window, dt, stis_mode=stis_mode, stis_block=stis_block)
    Qd, Kd, Vd, dOd = (to_dev(x, dtype) for x in (Q, K, V, dO))
    vld, gwd, gbd = torch.from_numpy(vl).cuda(), torch.from_numpy(gw).cuda(), torch.from_numpy(gb).cuda()
    sel_pos = B.select_positions(p_sel, G, l, s, Qd, Kd, vld)
    f = B.attn_fwd_positions(p, G, Qd, Kd, Vd, vld, sel_pos, gwd, gbd, want_branches=True)
    poison = lambda shape: torch.full(shape, float("nan"), dtype=Qd.dtype, device="cuda")
    out = B.BwdOut(poison((Bn, H, L, d)), poison((Bn, G, L, d)), poison((Bn, G, L, d)),
                   torch.full((H, 2 * d), float("nan"), device="cuda"), torch.full((H,), float("nan"), device="cuda"))
    g = B.attn_bwd_positions(p, G, Qd, Kd, Vd, vld, sel_pos, gwd, gbd, f, dOd, out=out)
    torch.cuda.synchronize()
    sel_ref = oracle.select_positions(Q, K, vl, l, s, lsel, k)
    np.testing.assert_array_equal(sel_pos.cpu().numpy(), sel_ref)
    rep = H // G
    gr = oracle.attn_bwd(Q, np.repeat(K, rep, 1), np.repeat(V, rep, 1), vl, np.repeat(sel_ref, rep, 1), gw, gb, dO, lsel, k,
                         window, per_position=True, stis_block=(stis_block if stis_mode else 0))
    tol = TOL[dtype]
    assert_close(host(g.dQ), gr.dQ.reshape(Bn, H, L, d), tol, "dQ")
    assert_close(host(g.dK), gr.dK.reshape(Bn, G, rep, L, d).sum(2), tol, "dK")
    assert_close(host(g.dV), gr.dV.reshape(Bn, G, rep, L, d).sum(2), tol, "dV")
    assert_close(host(g.d_gate_w), gr.d_gate_w, tol, "d_gate_w")
    assert_close(host(g.d_gate_b), gr.d_gate_b, tol, "d_gate_b")
    for r in range(Bn):   # padding rows get exact zeros
        p0 = L - int(vl[r])
        if p0 > 0:
            assert float(g.dQ[r, :, :p0].float().abs().max()) == 0.0
            assert float(g.dK[r, :, :p0].float().abs().max()) == 0.0
            assert float(g.dV[r, :, :p0].float().abs().max()) == 0.0
    # a second call into the same buffers gives the same bits (no atomics, nothing accumulated across calls)
    first = [t.clone() for t in (g.dQ, g.dK, g.dV, g.d_gate_w, g.d_gate_b)]
    g2 = B.attn_bwd_positions(p, G, Qd, Kd, Vd, vld, sel_pos, gwd, gbd, f, dOd, out=g)
    torch.cuda.synchronize()
    for a, b2 in zip(first, (g2.dQ, g2.dK, g2.dV, g2.d_gate_w, g2.d_gate_b)):
        assert torch.equal(a, b2)


def test_per_position_attention_limits():
    z = lambda *s: torch.zeros(s, device="cuda")
    vl = torch.tensor([64], dtype=torch.int32, device="cuda")
    gw = z(2, 16)
    with pytest.raises(B.BlossomError):   # groups must divide the heads
        B.attn_fwd_positions(B.Params(1, 3, 64, 8, 16, 2, 8, B.F32), 2, z(1, 3, 64, 8), z(1, 2, 64, 8), z(1, 2, 64, 8), vl,
                             torch.zeros((1, 2, 64, 2), dtype=torch.int32, device="cuda"), z(3, 16))
    with pytest.raises(B.BlossomError):   # selection block 32 is outside the kernels that serve this form
        B.attn_fwd_positions(B.Params(1, 2, 64, 8, 32, 2, 8, B.F32), 1, z(1, 2, 64, 8), z(1, 1, 64, 8), z(1, 1, 64, 8), vl,
                             torch.zeros((1, 1, 64, 2), dtype=torch.int32, device="cuda"), gw)
    with pytest.raises(B.BlossomError):   # the backward keeps Q, dO and the row constants of a head in LDS: L = 480 at d = 32 is beyond
        pb = B.Params(1, 2, 480, 32, 16, 2, 8, B.F32)
        f = B.FwdOut(z(1, 2, 480, 32), z(1, 2, 480, 32), z(1, 2, 480, 32), z(1, 2, 480), z(1, 2, 480))
        B.attn_bwd_positions(pb, 1, z(1, 2, 480, 32), z(1, 1, 480, 32), z(1, 1, 480, 32),
                             torch.tensor([480], dtype=torch.int32, device="cuda"),
                             torch.zeros((1, 1, 480, 2), dtype=torch.int32, device="cuda"), z(2, 64), None, f, z(1, 2, 480, 32))
