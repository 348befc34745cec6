"""Pins of the oracle's selection rule as the paper prints it (Sec. 3.4, Eq. 8-13): overlapping
compression blocks, per-position softmax scores, the score mapping of Eq. 11, the group sum of Eq. 12 and
top-k per position; and of the attention under such a per-position selection."""
import itertools
import math

import numpy as np
import pytest
import torch

import oracle


def _rand(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float32)


def test_canonical_exponential():
    assert oracle.canon_exp(0.0) == 1.0
    xs = np.concatenate([np.linspace(-90.0, 0.0, 2001), -np.logspace(-6, 1.9, 200)])
    got = np.array([oracle.canon_exp(float(np.float32(x))) for x in xs])
    ref = np.exp(xs.astype(np.float32).astype(np.float64))
    ok = ref > 1e-37
    # the argument is reduced with one fp32 multiply by log2(e): a relative error of 2^-24 in y = x*log2(e)
    # is an absolute one of |y|*2^-24 in the exponent; on top of that a few units in the last place
    bound = 3e-7 + np.abs(xs) * 1.4427 * 2.0 ** -24 * math.log(2.0) * 1.5
    assert np.all(np.abs(got[ok] - ref[ok]) / ref[ok] <= bound[ok])
    order = np.argsort(xs)
    assert np.all(np.diff(got[order]) >= 0)                       # monotone
    assert oracle.canon_exp(-100.0) == 0.0                        # below the normal range: exactly zero
    assert oracle.canon_exp(float(np.float32(-math.log(2.0)))) == pytest.approx(0.5, rel=2e-7)


@pytest.mark.parametrize("L,l,s", [(256, 32, 16), (512, 32, 16), (1024, 32, 16), (2048, 32, 16), (50, 8, 4), (31, 32, 16)])
def test_compression_block_count_and_selected_keys_of_table4(L, l, s):
    # Appendix D, Table 4 (compression 32, stride 16, selection block 16, k = 4): a late position scores
    # M = floor((L-32)/16)+1 compression blocks (15, 31, 63, 127 at the table's lengths) and attends the
    # k*l' = 64 keys of its selected blocks (the own block among them, cut at the position itself).
    lsel, k = 16 if l == 32 else l, 4
    Q, K = _rand((1, 2, L, 8), 1), _rand((1, 1, L, 8), 2)
    vl = np.array([L], np.int32)
    sel, sc = oracle.select_positions(Q, K, vl, l, s, lsel, k, want_scores=True)
    M = (L - l) // s + 1 if L >= l else 0
    if l == 32 and L >= 256:
        assert M == {256: 15, 512: 31, 1024: 63, 2048: 127}[L]
    t = L - 1
    # every compression block lies in the past of the last position: all M of them carry probability
    # mass, which the mapping of Eq. 11 spreads over the selection blocks: (l'/s)*(l/s) terms per block
    total = float(sc[0, 0, t].sum())
    if M > 0:
        terms = (lsel // s) * (l // s)
        assert total == pytest.approx(2 * terms, rel=1e-5) or total < 2 * terms   # two heads, each softmax sums to 1
    row = [int(j) for j in sel[0, 0, t] if j >= 0]
    NBs = -(-L // lsel)
    assert row == sorted(row) and row[-1] == t // lsel and len(row) == min(k, NBs)
    keys = sum(min((j + 1) * lsel, t + 1) - j * lsel for j in row)
    if l == 32 and L >= 256:
        assert keys == k * lsel                                    # 64


def test_uniform_scores_hand_case_and_eq11_mapping():
    # all keys equal => every eligible compression block has the same logit => S_cmp = 1/n_eligible, and
    # Eq. 11 turns into counting how many eligible compression blocks map to each selection block
    L, d, l, s, lsel = 64, 4, 8, 4, 8
    Q = np.ones((1, 1, L, d), np.float32)
    K = np.ones((1, 1, L, d), np.float32)
    vl = np.array([L], np.int32)
    sel, sc = oracle.select_positions(Q, K, vl, l, s, lsel, 3, want_scores=True)
    M = (L - l) // s + 1
    ra, rc = lsel // s, l // s
    for t in (7, 8, 23, 40, 63):
        elig = [m for m in range(M) if m * s + l - 1 <= t]
        n = len(elig)
        for j in range(L // lsel):
            cnt = sum(1 for a in range(ra) for c in range(rc) if (ra * j - a - c) in elig)
            want = cnt / n if n else 0.0
            assert sc[0, 0, t, j] == pytest.approx(want, abs=1e-6), (t, j)
    # at t = 40 (own block 5): eligible blocks m = 0..8; counts per selection block j: 1, 4, 4, 4, 4, (own)
    # -> ties among j = 1..4 resolve to the lowest indices: {1, 2} plus the own block 5
    assert [int(x) for x in sel[0, 0, 40]] == [1, 2, 5]
    assert [int(x) for x in sel[0, 0, 7]] == [0, -1, -1]           # first block: nothing earlier
    # Eq. 11 with l = s = l' is the identity on the compression scores
    Q2, K2 = _rand((1, 1, 40, 4), 3), _rand((1, 1, 40, 4), 4)
    _, sc1 = oracle.select_positions(Q2, K2, np.array([40], np.int32), 8, 8, 8, 2, want_scores=True)
    t = 39
    logits = np.array([float(Q2[0, 0, t] @ K2[0, 0, 8 * m:8 * m + 8].mean(0)) for m in range(4)])  # blocks ending <= 39: m = 0..3 (m = 4 ends at 39)
    logits = np.array([float(Q2[0, 0, t] @ K2[0, 0, 8 * m:8 * m + 8].mean(0)) for m in range(5)])
    p = np.exp(logits - logits.max())
    p /= p.sum()
    assert np.allclose(sc1[0, 0, t], p, rtol=2e-6, atol=1e-7)


def test_group_sum_and_top_k_brute_force():
    B, H, G, L, d, l, s, lsel, k = 2, 4, 2, 70, 8, 8, 4, 8, 3
    Q, K = _rand((B, H, L, d), 5), _rand((B, G, L, d), 6)
    vl = np.array([70, 41], np.int32)
    sel, sc = oracle.select_positions(Q, K, vl, l, s, lsel, k, want_scores=True)
    # Eq. 12: the group score is the sum of the heads' scores: running each head alone against the
    # same key head and adding gives the same numbers
    for g in range(G):
        tot = np.zeros_like(sc[:, g])
        for hh in range(H // G):
            _, one = oracle.select_positions(Q[:, g * 2 + hh:g * 2 + hh + 1], K[:, g:g + 1], vl, l, s, lsel, k, want_scores=True)
            tot = tot + one[:, 0]
        assert np.allclose(sc[:, g], tot, rtol=1e-6, atol=1e-7)
    # Eq. 13 by brute force on the returned scores
    for r in range(B):
        p0 = L - int(vl[r])
        for g in range(G):
            for t in range(L):
                row = [int(j) for j in sel[r, g, t] if j >= 0]
                if t < p0:
                    assert row == []
                    continue
                jt, jf = t // lsel, p0 // lsel
                cand = list(range(jf, jt))
                take = min(k - 1, len(cand))
                assert row == sorted(row) and row[-1] == jt and len(row) == take + 1
                score = lambda S: tuple(sorted((float(sc[r, g, t, j]) for j in S), reverse=True))
                best = max(score(S) for S in itertools.combinations(cand, take))
                assert score(row[:-1]) == best
                assert tuple(row[:-1]) == min(S for S in itertools.combinations(cand, take) if score(S) == best)
    # duplicated query heads double every score and leave the selection unchanged
    sel2 = oracle.select_positions(np.concatenate([Q[:, :1], Q[:, :1]], 1), K[:, :1], vl, l, s, lsel, k)
    sel1 = oracle.select_positions(Q[:, :1], K[:, :1], vl, l, s, lsel, k)
    assert np.array_equal(sel2, sel1)


def test_attention_under_a_per_position_selection():
    # the long-term branch reads one selection row per position; with k covering every block it is
    # dense causal attention (library routine), and it differs from it otherwise
    B, H, L, d, lsel = 1, 2, 48, 8, 8
    Q, K, V = _rand((B, H, L, d), 7), _rand((B, H, L, d), 8), _rand((B, H, L, d), 9)
    vl = np.array([41], np.int32)
    gw = np.zeros((H, 2 * d), np.float32)
    big = np.full((H,), 1e4, np.float32)                          # gate forced to the long-term branch
    for k in (6, 2):
        selg = oracle.select_positions(Q, K[:, :1], vl, 8, 4, lsel, k)   # one key/value group
        sel = np.repeat(selg, H, axis=1)                           # every head of the group reads the group's rows
        f = oracle.attn_fwd(Q, np.repeat(K[:, :1], H, 1), V, vl, sel, gw, big, lsel, k, 1, per_position=True)
        p0 = L - 41
        q, kk, v = (torch.from_numpy(t[0, :, p0:].astype(np.float64)) for t in (Q, np.repeat(K[:, :1], H, 1), V))
        ref = torch.nn.functional.scaled_dot_product_attention(q, kk, v, is_causal=True).numpy()
        err = np.max(np.abs(f.O.reshape(H, L, d)[:, p0:] - ref))
        assert (err < 1e-12) if k == 6 else (err > 1e-3)
    # masks: row t of the long-term mask is exactly the causal part of its own selected blocks
    M_lt, _ = oracle.build_masks(L, lsel, 2, 1, 41, selg[0, 0], per_position=True)
    for t in range(L):
        want = np.zeros(L, np.uint8)
        if t >= p0:
            for j in selg[0, 0, t]:
                if j >= 0:
                    want[max(j * lsel, p0):min((j + 1) * lsel, t + 1)] = 1
        assert np.array_equal(M_lt[t], want), t


def test_per_position_backward_finite_differences():
    # the gradients under a per-position selection are the central differences of the oracle's own forward
    # (float64), also with every head of a group reading the same K, V and selection rows: the gradient
    # of a shared key is then the sum over the heads that read it
    B, H, G, L, d, lsel, k, w = 1, 4, 2, 37, 4, 8, 2, 3
    rng = np.random.default_rng(12)
    Q, dO = rng.standard_normal((B, H, L, d)), rng.standard_normal((B, H, L, d))
    K, V = rng.standard_normal((B, G, L, d)), rng.standard_normal((B, G, L, d))
    vl = np.array([30], np.int32)
    gw = rng.standard_normal((H, 2 * d)) * 0.3
    gb = rng.standard_normal(H) * 0.2
    selg = oracle.select_positions(Q.astype(np.float32), K.astype(np.float32), vl, 8, 4, lsel, k)
    rep = H // G
    sel = np.repeat(selg, rep, 1)
    kw = dict(f64=True, stis_block=2, per_position=True)
    g = oracle.attn_bwd(Q, np.repeat(K, rep, 1), np.repeat(V, rep, 1), vl, sel, gw, gb, dO, lsel, k, w, **kw)
    dK = g.dK.reshape(B, G, rep, L, d).sum(2)
    dV = g.dV.reshape(B, G, rep, L, d).sum(2)
    dQ = g.dQ.reshape(B, H, L, d)
    loss = lambda q_, k_, v_: float(np.sum(oracle.attn_fwd(q_, np.repeat(k_, rep, 1), np.repeat(v_, rep, 1), vl, sel, gw, gb,
                                                           lsel, k, w, **kw).O * dO.reshape(B * H, L, d)))
    eps = 1e-6
    for name, arr, grad in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        heads = arr.shape[1]
        for idx in [(0, 0, 9, 1), (0, heads - 1, 36, 3), (0, 0, 20, 0), (0, heads - 1, 7, 2), (0, 0, 31, 2)]:
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += eps
            lo[idx] -= eps
            args = lambda a: (a if name == "Q" else Q, a if name == "K" else K, a if name == "V" else V)
            fd = (loss(*args(hi)) - loss(*args(lo))) / (2 * eps)
            got = grad[idx]
            assert abs(fd - got) <= 1e-6 * (abs(fd) + 1.0), (name, idx, fd, got)
    p0 = L - 30
    assert np.all(dQ[:, :, :p0] == 0) and np.all(dK[:, :, :p0] == 0) and np.all(dV[:, :, :p0] == 0)
    assert np.abs(dK[:, :, p0:]).min() > 0
    # two positions of one block with different selection rows exist (else this would not test the per-position form)
    assert any(not np.array_equal(selg[0, 0, t], selg[0, 0, t + 1]) for t in range(p0, L - 1) if t // lsel == (t + 1) // lsel)
