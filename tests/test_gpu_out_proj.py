"""GPU parity of blossom_out_proj_ln (Eq. 4 output projection, residual and LayerNorm of Sec. 3.6) with the oracle."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, assert_close, host, to_dev
from paper_2512_13368_amd import binding as B
from paper_2512_13368_amd.inputs import round_to_bf16

pytestmark = pytest.mark.gpu


def _inputs(dtype, Bn, H, L, d, Dm, seed):
    rng = np.random.default_rng(seed)
    O = rng.standard_normal((Bn, H, L, d)).astype(np.float32)
    Wt = (rng.standard_normal((Dm, H * d)) / np.sqrt(H * d)).astype(np.float32)
    Hp = rng.standard_normal((Bn, L, Dm)).astype(np.float32)
    if dtype == "bf16":
        O, Wt, Hp = (round_to_bf16(x) for x in (O, Wt, Hp))
    gamma = (1.0 + 0.2 * rng.standard_normal(Dm)).astype(np.float32)
    beta = (0.3 * rng.standard_normal(Dm)).astype(np.float32)
    bias = (0.5 * rng.standard_normal(Dm)).astype(np.float32)
    return O, Wt, Hp, gamma, beta, bias


@pytest.mark.parametrize("dtype,Bn,H,L,d,Dm,with_bias", [
    ("bf16", 2, 8, 300, 64, 512, True),    # the L = 8192 workload's layer (8 heads of 64): matrix cores, ragged last tile
    ("bf16", 3, 4, 128, 64, 256, False),   # the L = 1024 workloads' layer (4 heads of 64): two position halves per workgroup
    ("bf16", 1, 4, 77, 64, 256, True),     # shorter than one tile
    ("bf16", 2, 2, 130, 64, 512, False),   # projection to a wider model (H*d = 128)
    ("fp32", 3, 2, 200, 32, 64, True),     # the short-sequence shapes (hidden 64), scalar kernel
    ("fp32", 2, 8, 61, 8, 64, False),      # the paper's own setting: 8 heads of 8
    ("bf16", 2, 8, 50, 16, 128, True),     # bf16 outside the matrix-core shapes
    ("fp32", 1, 8, 19, 64, 512, True),     # fp32 at the large layer: two features per thread
    ("fp32", 1, 3, 40, 8, 72, False),      # a feature count that is no multiple of the thread groups
])
def test_out_proj_ln_matches_the_oracle(dtype, Bn, H, L, d, Dm, with_bias):
    O, Wt, Hp, gamma, beta, bias = _inputs(dtype, Bn, H, L, d, Dm, 500 + L + Dm)
    eps = 1e-5
    print(f"out_proj_ln {dtype} B{Bn} H{H} L{L} d{d} Dm{Dm} bias {with_bias}", flush=True)
    p = B.Params(Bn, H, L, d, 16, 1, 1, B.F32 if dtype == "fp32" else B.BF16)
    gd, bd = torch.from_numpy(gamma).cuda(), torch.from_numpy(beta).cuda()
    biasd = torch.from_numpy(bias).cuda() if with_bias else None
    S, mean, rstd = B.out_proj_ln(p, Dm, to_dev(O, dtype), to_dev(Wt, dtype), to_dev(Hp, dtype), gd, bd, eps, bias=biasd,
                                  want_stats=True)
    torch.cuda.synchronize()
    ref, mref, rref = oracle.out_proj_ln(O, Wt, Hp, gamma, beta, eps, bias=bias if with_bias else None, want_stats=True)
    tol = TOL[dtype]
    assert_close(host(S), ref, tol, "S")
    assert_close(host(mean), mref, 1e-4, "mean")     # the statistics are fp32 whatever the storage type
    assert_close(host(rstd), rref, 1e-4, "rstd")
    # the same call without the statistics gives the same rows, into a caller's buffer
    out = torch.full_like(S, 7.0)
    S2 = B.out_proj_ln(p, Dm, to_dev(O, dtype), to_dev(Wt, dtype), to_dev(Hp, dtype), gd, bd, eps, bias=biasd, S=out)
    torch.cuda.synchronize()
    assert S2 is out and torch.equal(S2, S)


def test_out_proj_ln_seeded_random_shapes():
    # 30 seeded draws over both kernels: storage type, head size and count, model width (multiples of 8), length
    rng = np.random.default_rng(20251)
    for case in range(30):
        dtype = "bf16" if rng.random() < 0.5 else "fp32"
        d = int(rng.choice([8, 16, 32, 64]))
        H = int(rng.integers(1, 9))
        if dtype == "bf16" and d == 64 and rng.random() < 0.7:
            Dm = int(rng.choice([256, 512]))                       # the matrix-core kernel
        else:
            Dm = 8 * int(rng.integers(1, 65))
        Bn, L = int(rng.integers(1, 4)), int(rng.integers(1, 301))
        with_bias = bool(rng.random() < 0.5)
        eps = float(rng.choice([1e-12, 1e-5, 1e-3]))
        O, Wt, Hp, gamma, beta, bias = _inputs(dtype, Bn, H, L, d, Dm, 7000 + case)
        print(f"out_proj_ln draw {case}: {dtype} B{Bn} H{H} L{L} d{d} Dm{Dm} bias {with_bias} eps {eps}", flush=True)
        p = B.Params(Bn, H, L, d, 16, 1, 1, B.F32 if dtype == "fp32" else B.BF16)
        S, mean, rstd = B.out_proj_ln(p, Dm, to_dev(O, dtype), to_dev(Wt, dtype), to_dev(Hp, dtype), torch.from_numpy(gamma).cuda(),
                                      torch.from_numpy(beta).cuda(), eps, bias=torch.from_numpy(bias).cuda() if with_bias else None,
                                      want_stats=True)
        torch.cuda.synchronize()
        ref, mref, rref = oracle.out_proj_ln(O, Wt, Hp, gamma, beta, eps, bias=bias if with_bias else None, want_stats=True)
        assert_close(host(S), ref, TOL[dtype], f"S (draw {case})")
        assert_close(host(mean), mref, 1e-4, f"mean (draw {case})")
        assert_close(host(rstd), rref, 1e-4, f"rstd (draw {case})")


def test_out_proj_ln_after_the_attention():
    # the layer as a model runs it: selection, attention, then the fused projection + residual + LayerNorm
    # on the attention's own output buffer; against the oracle's chain
    from gpu_util import Dev, params
    from paper_2512_13368_amd.inputs import WORKLOADS, make_inputs, with_shape
    w = with_shape(WORKLOADS["cfg5"], name="layer", B=2, L=320, len_lo=100, len_hi=320, seed=1234)
    x = make_inputs(w)
    dv = Dev(x)
    p = params(w)
    sel = B.select_blocks(p, dv.Q, dv.K, dv.vl)
    f = B.attn_fwd(p, dv.Q, dv.K, dv.V, dv.vl, sel, dv.gw, dv.gb)
    Dm = w.H * w.d
    _, Wt, Hp, gamma, beta, _ = _inputs("bf16", w.B, w.H, w.L, w.d, Dm, 99)
    S = B.out_proj_ln(p, Dm, f.O, to_dev(Wt, "bf16"), to_dev(Hp, "bf16"), torch.from_numpy(gamma).cuda(),
                      torch.from_numpy(beta).cuda(), 1e-5)
    torch.cuda.synchronize()
    sel_ref = oracle.select_blocks(x.Q, x.K, x.valid_len, w.block, w.topk)
    fr = oracle.attn_fwd(x.Q, x.K, x.V, x.valid_len, sel_ref, x.gate_w, x.gate_b, w.block, w.topk, w.window)
    ref = oracle.out_proj_ln(fr.O.reshape(w.B, w.H, w.L, w.d), Wt, Hp, gamma, beta, 1e-5)
    assert_close(host(S), ref, TOL["bf16"], "S after attention")
    # a padding row carries no attention output: LayerNorm of the layer's input alone
    r = int(np.argmin(x.valid_len))
    p0 = w.L - int(x.valid_len[r])
    assert p0 > 0
    z = Hp[r, :p0].astype(np.float64)
    ln = (z - z.mean(-1, keepdims=True)) / np.sqrt(z.var(-1, keepdims=True) + 1e-5) * gamma + beta
    assert_close(host(S[r, :p0]), ln, TOL["bf16"], "padding rows")


def test_out_proj_ln_limits():
    z = lambda *s: torch.zeros(s, device="cuda")
    with pytest.raises(B.BlossomError):   # d_model beyond the scalar kernel's range
        B.out_proj_ln(B.Params(1, 2, 16, 8, 16, 1, 1, B.F32), 2048, z(1, 2, 16, 8), z(2048, 16), z(1, 16, 2048), z(2048), z(2048), 1e-5)
    with pytest.raises(B.BlossomError):   # negative epsilon
        B.out_proj_ln(B.Params(1, 2, 16, 8, 16, 1, 1, B.F32), 16, z(1, 2, 16, 8), z(16, 16), z(1, 16, 16), z(16), z(16), -1.0)
