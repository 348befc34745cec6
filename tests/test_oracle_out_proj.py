"""Pins of the oracle's layer around the attention (Sec. 2.1 Eq. 4: concatenated heads times W^O; Sec. 3.6,
the equation after Eq. 19: residual and LayerNorm): library routines, closed forms, a hand case."""
import numpy as np
import torch

import oracle


def _case(B, H, L, d, Dm, seed, bias=True):
    rng = np.random.default_rng(seed)
    O = rng.standard_normal((B, H, L, d))
    Wt = rng.standard_normal((Dm, H * d)) / np.sqrt(H * d)
    Hp = rng.standard_normal((B, L, Dm))
    g = 1.0 + 0.2 * rng.standard_normal(Dm)
    be = 0.3 * rng.standard_normal(Dm)
    bi = 0.5 * rng.standard_normal(Dm) if bias else None
    return O, Wt, Hp, g, be, bi


def test_against_library_linear_and_layer_norm():
    # the heads laid side by side (head 0 first), one linear layer, residual, LayerNorm: the library's routines in float64
    for B, H, L, d, Dm, seed, bias in ((2, 3, 7, 4, 10, 1, True), (1, 8, 33, 8, 64, 2, False), (2, 2, 5, 16, 24, 3, True)):
        O, Wt, Hp, g, be, bi = _case(B, H, L, d, Dm, seed, bias)
        S, mean, rstd = oracle.out_proj_ln(O, Wt, Hp, g, be, 1e-5, bias=bi, want_stats=True)
        t = lambda a: None if a is None else torch.from_numpy(a)
        c = t(O).permute(0, 2, 1, 3).reshape(B, L, H * d)
        z = t(Hp) + torch.nn.functional.linear(c, t(Wt), t(bi))
        ref = torch.nn.functional.layer_norm(z, (Dm,), t(g), t(be), 1e-5).numpy()
        assert np.max(np.abs(S - ref)) < 1e-12
        assert np.max(np.abs(mean - z.mean(-1).numpy())) < 1e-12
        assert np.max(np.abs(rstd - 1.0 / np.sqrt(z.var(-1, unbiased=False).numpy() + 1e-5))) < 1e-10


def test_hand_case_and_head_order():
    # two heads of two channels, W^O the identity: z = H_prev + [head 0 | head 1]; LayerNorm of (1, 2, 3, 6):
    # mean 3, variance 3.5
    O = np.zeros((1, 2, 1, 2))
    O[0, 0, 0] = [1.0, 2.0]
    O[0, 1, 0] = [3.0, 6.0]
    Hp = np.zeros((1, 1, 4))
    S = oracle.out_proj_ln(O, np.eye(4), Hp, np.ones(4), np.zeros(4), 0.0)
    want = (np.array([1.0, 2.0, 3.0, 6.0]) - 3.0) / np.sqrt(3.5)
    assert np.max(np.abs(S[0, 0] - want)) < 1e-15
    # a transposed weight would be caught: row n of Wt makes output n
    Wt = np.zeros((4, 4))
    Wt[2, 1] = 1.0      # output 2 = channel 1 of head 0
    Wt[0, 3] = 1.0      # output 0 = channel 1 of head 1
    S2 = oracle.out_proj_ln(O, Wt, Hp, np.ones(4), np.zeros(4), 0.0)
    z = np.array([6.0, 0.0, 2.0, 0.0])
    assert np.max(np.abs(S2[0, 0] - (z - 2.0) / np.sqrt(np.mean((z - 2.0) ** 2)))) < 1e-15
    # gamma scales, beta shifts, the bias enters before the normalisation
    # a constant row (z = 6 everywhere) has zero variance: the output is beta exactly, whatever gamma
    S3 = oracle.out_proj_ln(O, Wt, Hp, np.full(4, 2.0), np.full(4, -1.0), 1e-5, bias=np.array([0.0, 6.0, 4.0, 6.0]))
    assert np.all(S3[0, 0] == -1.0)


def test_invariants():
    B, H, L, d, Dm = 2, 4, 9, 8, 32
    O, Wt, Hp, g, be, bi = _case(B, H, L, d, Dm, 11)
    S, mean, rstd = oracle.out_proj_ln(O, Wt, Hp, g, be, 1e-6, bias=bi, want_stats=True)
    # with gamma = 1, beta = 0 every row has mean 0 and variance var/(var + eps)
    S1 = oracle.out_proj_ln(O, Wt, Hp, np.ones(Dm), np.zeros(Dm), 1e-6, bias=bi)
    assert np.max(np.abs(S1.mean(-1))) < 1e-14
    var = 1.0 / rstd ** 2 - 1e-6
    assert np.max(np.abs(S1.var(-1) - var / (var + 1e-6))) < 1e-12
    # a constant added to every feature of the bias moves the mean and nothing else
    S2, mean2, rstd2 = oracle.out_proj_ln(O, Wt, Hp, g, be, 1e-6, bias=bi + 3.0, want_stats=True)
    assert np.max(np.abs(S2 - S)) < 1e-12 and np.max(np.abs(mean2 - mean - 3.0)) < 1e-12 and np.max(np.abs(rstd2 - rstd)) < 1e-12
    # a zero projection leaves LayerNorm(H_prev + bias); zero attention output (a padding row) does the same
    Sz = oracle.out_proj_ln(O, np.zeros_like(Wt), Hp, g, be, 1e-6, bias=bi)
    S0 = oracle.out_proj_ln(np.zeros_like(O), Wt, Hp, g, be, 1e-6, bias=bi)
    assert np.array_equal(Sz, S0)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(Hp + bi), (Dm,), torch.from_numpy(g), torch.from_numpy(be), 1e-6).numpy()
    assert np.max(np.abs(Sz - ref)) < 1e-12
    # rows are independent: permuting the positions permutes the output
    perm = np.random.default_rng(5).permutation(L)
    Sp = oracle.out_proj_ln(O[:, :, perm], Wt, Hp[:, perm], g, be, 1e-6, bias=bi)
    assert np.array_equal(Sp, S[:, perm])
