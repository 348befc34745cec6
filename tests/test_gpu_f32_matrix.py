"""GPU parity of the fp32 matrix-instruction kernels for short sequences (fp32 or bf16 storage, d in {8, 16, 32},
block 8 or 16, K/V or Q/dO of a whole head resident in LDS): forward, dQ and dK/dV against the CPU oracle, at
the shapes where those kernels take over from the scalar-ALU ones and at the edges of that range."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, Dev, assert_close, host, params
from paper_2512_13368_amd import binding as B
from paper_2512_13368_amd.inputs import WORKLOADS, make_inputs, rope_tables, with_shape
from test_gpu_parity import run_case

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("b,L,topk,window", [
    (16, 200, 4, 16),    # the short-sequence recommender shape (cfg2), with backward
    (16, 197, 4, 16),    # ragged last block
    (16, 208, 5, 40),    # the longest sequence the resident kernels take at block 16
    (8, 200, 4, 8),      # block 8: half-filled 16-row tiles, 25 blocks over 8 wavefronts
    (8, 51, 2, 8),       # ragged, block 8
    (16, 16, 1, 1),      # one block, own block only, self only
    (16, 33, 3, 500),    # window beyond the sequence, top-k = number of blocks
])
def test_short_sequences_forward_backward(b, L, topk, window):
    w = with_shape(WORKLOADS["cfg2"], name=f"f32mc-b{b}-L{L}", B=7, H=3, L=L, block=b, topk=topk, window=window,
                   len_lo=1, len_hi=L, seed=900 + b + L)
    x = make_inputs(w, want_dO=True)
    # a full row, a row starting inside a block, one shorter than a block, a single item, an empty row
    x.valid_len[:5] = [L, max(1, L - b - 3), min(L, b // 2 + 1), 1, 0]
    run_case(w, x=x, backward=True, check_dense=True, gate_scale=0.4)


def test_sharp_softmax_and_holes():
    # large logits move the running maximum of the forward's online softmax from tile to tile;
    # caller-built selection rows with holes are skipped where they stand
    w = with_shape(WORKLOADS["cfg2"], name="f32mc-sharp", B=4, H=2, L=150, topk=5, window=24, len_lo=40, len_hi=150,
                   seed=951)
    x = make_inputs(w, want_dO=True)
    x.Q *= np.float32(3.0)

    def punch(sel):
        NB = sel.shape[2]
        for I in range(NB):
            row = sel[:, :, I]
            full = (row >= 0).sum(-1) >= 3
            row[full, 0] = NB + 2          # an id past the last block, up front
            row[full, 1] = -1              # a hole
        return sel

    run_case(w, x=x, backward=True, sel_edit=punch)


def test_rope_backward_and_serving_mode():
    w = with_shape(WORKLOADS["cfg2"], name="f32mc-rope", B=5, H=2, L=120, len_lo=10, len_hi=120, seed=977)
    x = make_inputs(w, want_dO=True)
    cos, sin = rope_tables(w.L, w.d)
    dv = Dev(x)
    cos_d, sin_d = torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda()
    p = params(w, save_for_bwd=1)
    Q_rot, K_rot, sel = B.rope_select_blocks(p, dv.Q, dv.K, cos_d, sin_d, dv.vl)
    f = B.attn_fwd(p, Q_rot, K_rot, dv.V, dv.vl, sel, dv.gw, dv.gb)
    g = B.attn_bwd(p, Q_rot, K_rot, dv.V, dv.vl, sel, dv.gw, dv.gb, f, dv.dO, rope=(cos_d, sin_d))
    torch.cuda.synchronize()
    Qr, Kr = oracle.rope(x.Q, cos, sin), oracle.rope(x.K, cos, sin)
    sel_ref = oracle.select_blocks(Qr, Kr, x.valid_len, w.block, w.topk)
    np.testing.assert_array_equal(sel.cpu().numpy(), sel_ref)
    flat = lambda t: host(t).reshape(w.B * w.H, *t.shape[2:])
    tol = TOL[w.dtype]
    fr = oracle.attn_fwd(Qr, Kr, x.V, x.valid_len, sel_ref, x.gate_w, x.gate_b, w.block, w.topk, w.window)
    gr = oracle.attn_bwd(Qr, Kr, x.V, x.valid_len, sel_ref, x.gate_w, x.gate_b, x.dO, w.block, w.topk, w.window)
    assert_close(flat(f.O), fr.O, tol, "O")
    assert_close(flat(g.dQ), oracle.rope_bwd(gr.dQ, cos, sin), tol, "dQ (rotated back)")
    assert_close(flat(g.dK), oracle.rope_bwd(gr.dK, cos, sin), tol, "dK (rotated back)")
    assert_close(flat(g.dV), gr.dV, tol, "dV")
    # serving mode: only the last query block is written, and it equals the full run's
    O = torch.full_like(f.O, 3.0)
    B.attn_fwd(params(w, last_block_only=1), Q_rot, K_rot, dv.V, dv.vl, sel, dv.gw, dv.gb, out=B.FwdOut(O))
    torch.cuda.synchronize()
    lo = (w.NB - 1) * w.block
    assert torch.equal(O[:, :, lo:], f.O[:, :, lo:]) and bool((O[:, :, :lo] == 3.0).all())


def test_just_outside_the_resident_range():
    # one block more than the resident kernels take: the scalar-ALU kernels serve the shape, same answers
    run_case(with_shape(WORKLOADS["cfg2"], name="f32-L224", B=3, H=2, L=224, len_lo=30, len_hi=224, seed=990),
             backward=True)


@pytest.mark.parametrize("dtype,d,b,L,topk,window,sblk", [
    ("fp32", 8, 16, 197, 4, 8, 1),      # the paper's own hyperparameters: hidden 64 over 8 heads, mask block 1
    ("fp32", 16, 16, 200, 4, 8, 1),     # ML-1M head size
    ("bf16", 8, 8, 120, 3, 8, 2),       # bf16 storage, block 8, a small mask block
    ("bf16", 16, 16, 150, 4, 24, 16),   # mask block = selection block
    ("bf16", 32, 16, 200, 4, 16, 0),    # bf16 storage, plain window
    ("fp32", 32, 8, 90, 3, 8, 4),
])
def test_head_sizes_storage_types_and_full_short_term_mask(dtype, d, b, L, topk, window, sblk):
    w = with_shape(WORKLOADS["cfg2"], name=f"res-{dtype}-d{d}-b{b}-s{sblk}", B=5, H=16 // (d // 8 if d < 32 else 4),
                   L=L, d=d, block=b, topk=topk, window=window, dtype=dtype, qkv_scaled=(dtype == "bf16"), len_lo=1,
                   len_hi=L, stis_block=sblk, seed=1200 + d + b + sblk)
    x = make_inputs(w, want_dO=True)
    x.valid_len[:4] = [L, max(1, L - b - 3), min(L, b // 2 + 1), 0]
    run_case(w, x=x, backward=True, check_dense=True, gate_scale=0.4)


def test_long_rows_with_more_than_64_kb_of_lds():
    # the efficiency-study length 1000 at the paper's hyperparameters: K and V of a head take 96 KB of LDS,
    # dK/dV's Q, dO and row constants 120 KB; one workgroup per CU
    w = with_shape(WORKLOADS["cfg2"], name="res-L1000", B=8, H=8, L=1000, d=8, block=16, topk=4, window=8, len_lo=300,
                   len_hi=1000, stis_block=1, seed=1301)
    run_case(w, backward=True, pairs=[0, 7, 21, 38, 63])


def test_seeded_random_shapes_in_the_resident_range():
    # 60 seeded draws over storage type, head size, block size, length, top-k, window, mask block and form
    rng = np.random.default_rng(4242)
    for case in range(60):
        dtype = "bf16" if rng.random() < 0.35 else "fp32"
        d = int(rng.choice([8, 16, 32]))
        b = int(rng.choice([8, 16]))
        nb = int(rng.integers(1, 27))
        L = max(2, nb * b - int(rng.integers(0, b)))
        topk = int(rng.choice([1, 2, 3, 4, 5, nb, nb + 3]))
        window = int(rng.choice([1, 2, b - 1, b, b + 1, 2 * b + 5, 3 * b, L, L + 7]))
        bidir = bool(rng.random() < 0.25)
        sblk = int(rng.choice([0, 0, b, 1, 3, 2 * b, 4, b // 2]))
        if bidir and sblk == 0:
            sblk = int(rng.choice([1, b, 4]))
        w = with_shape(WORKLOADS["cfg1"], name=f"rr{case}", B=4, H=int(rng.choice([2, 3, 16])), L=L, d=d, block=b,
                       topk=max(1, topk), window=max(1, window), dtype=dtype, len_lo=0, len_hi=L,
                       qkv_scaled=(dtype == "bf16"), seed=424200 + case, stis_block=sblk, bidir=bidir)
        x = make_inputs(w, want_dO=True)
        x.valid_len[:] = [L, int(rng.integers(0, L + 1)), int(rng.integers(0, L + 1)), min(L, 1 + int(rng.integers(0, b)))]
        same = w.topk >= w.NB and (w.window >= L or sblk >= L)
        run_case(w, x=x, backward=True, check_dense=(case % 4 == 0 and not bidir), gate_scale=0.4, branches_coincide=same)
