"""Pins of the oracle's bidirectional form: Eq. 15 exactly as printed (symmetric window, power-of-two
block distances on both sides, last block; Sec. 3.5) with no causal mask in either branch, as a
bidirectional backbone uses it (Sec. 4.2)."""
import itertools

import numpy as np
import pytest
import torch

import oracle


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


@pytest.mark.parametrize("L,b,w,blk,n", [(64, 8, 5, 8, 64), (50, 8, 3, 4, 37), (96, 16, 20, 1, 96), (45, 8, 1, 8, 45)])
def test_symmetric_mask_against_the_printed_cases_and_the_causal_form(L, b, w, blk, n):
    NB = -(-L // b)
    sel = np.full((NB, 2), -1, np.int32)
    for I in range(NB):
        sel[I, 0] = I
    _, M = oracle.build_masks(L, b, 2, w, n, sel, stis_block=blk, bidir=True)
    _, Mc = oracle.build_masks(L, b, 2, w, n, sel, stis_block=blk)
    p0 = L - n
    # the three cases of Eq. 15, retyped from the paper, on valid pairs
    for i in range(L):
        for j in range(L):
            want = 0
            if i >= p0 and j >= p0:
                bq, bk = i // blk, j // blk
                dist = abs(bq - bk)
                want = int(abs(i - j) < w or (dist >= 1 and dist & (dist - 1) == 0) or j >= L - blk)
            assert M[i, j] == want, (i, j)
    # its causal half is the causal form (pinned on its own), the rest lies strictly above the diagonal
    assert np.array_equal(np.tril(M), Mc)
    # window and power-of-two terms are symmetric; only last-block columns break the symmetry
    keep = np.ones((L, L), bool)
    keep[:, L - blk:] = False
    keep[L - blk:, :] = False
    assert np.array_equal((M & keep), (M & keep).T)
    # every valid row sees the whole last block
    assert np.all(M[p0:, max(p0, L - blk):] == 1)


def test_participating_keys_per_row_closed_form():
    # full row, mask block 1, window w: a row far from both ends sees 2w-1 window keys, the power-of-two
    # distances 2^r >= w on each side that stay inside the row, and the last position
    L, w = 256, 8
    sel = np.full((L // 16, 1), -1, np.int32)
    _, M = oracle.build_masks(L, 16, 1, w, L, sel, stis_block=1, bidir=True)
    for i in (100, 128, 37):
        far = sum(1 for r in range(3, 9) for s in (-1, 1) if 0 <= i + s * (1 << r) < L and (i + s * (1 << r)) != L - 1)
        assert int(M[i].sum()) == (2 * w - 1) + far + 1


def test_bidirectional_selection_brute_force_and_hand_case():
    # hand case: integer data, block size 2, three blocks; query block 0 must pick from the LATER blocks
    Q = np.zeros((1, 1, 6, 2), np.float32)
    K = np.zeros((1, 1, 6, 2), np.float32)
    Q[0, 0, 0:2] = [[1, 0], [1, 0]]           # Qsum_0 = (2, 0)
    Q[0, 0, 2:4] = [[0, 1], [0, 1]]           # Qsum_1 = (0, 2)
    Q[0, 0, 4:6] = [[1, 1], [1, 1]]           # Qsum_2 = (2, 2)
    K[0, 0, 0:2] = [[1, 4], [3, 4]]           # Kmean_0 = (2, 4)
    K[0, 0, 2:4] = [[5, 0], [5, 2]]           # Kmean_1 = (5, 1)
    K[0, 0, 4:6] = [[3, 3], [3, 3]]           # Kmean_2 = (3, 3)
    vl = np.array([6], np.int32)
    sel, sc = oracle.select_blocks(Q, K, vl, 2, 2, want_scores=True, bidir=True)
    # scores: I=0: J1 -> 10, J2 -> 6;  I=1: J0 -> 8, J2 -> 6;  I=2: J0 -> 12, J1 -> 12 (tie -> lower index)
    assert sc[0, 0, 1] == 10 and sc[0, 0, 2] == 6 and sc[0, 1, 0] == 8 and sc[0, 1, 2] == 6
    assert sc[0, 2, 0] == 12 and sc[0, 2, 1] == 12
    assert sel[0, 0].tolist() == [[0, 1], [0, 1], [0, 2]]
    # the causal selection of the same data differs where a later block wins
    selc = oracle.select_blocks(Q, K, vl, 2, 2)
    assert selc[0, 0].tolist() == [[0, -1], [0, 1], [0, 2]]

    # brute force: the chosen set has the largest sorted score tuple among all (k-1)-subsets of the other
    # valid blocks, and among the maximisers the smallest index set
    rng = np.random.default_rng(11)
    B, H, L, d, b, k = 2, 2, 45, 8, 8, 3
    Q, K = _rand((B, H, L, d), 12), _rand((B, H, L, d), 13)
    vl = np.array([45, 29], np.int32)
    sel, sc = oracle.select_blocks(Q, K, vl, b, k, want_scores=True, bidir=True)
    NB = -(-L // b)
    for r in range(B):
        J_first = (L - int(vl[r])) // b
        for h in range(H):
            for I in range(NB):
                row = [int(t) for t in sel[r, h, I] if t >= 0]
                if (I + 1) * b <= L - int(vl[r]):
                    assert row == []
                    continue
                cand = [J for J in range(J_first, NB) if J != I]
                take = min(k - 1, len(cand))
                assert row == sorted(row) and I in row and len(row) == take + 1
                mine = tuple(sorted((float(sc[r * H + h, I, J]) for J in row if J != I), reverse=True))
                best = max(tuple(sorted((float(sc[r * H + h, I, J]) for J in S), reverse=True))
                           for S in itertools.combinations(cand, take))
                assert mine == best
                winners = [S for S in itertools.combinations(cand, take)
                           if tuple(sorted((float(sc[r * H + h, I, J]) for J in S), reverse=True)) == best]
                assert tuple(J for J in row if J != I) == min(winners)


def test_bidirectional_dense_limit_is_library_attention_with_a_key_padding_mask():
    # top-k covering every block and a window >= L: both branches are full attention over the valid keys
    B, H, L, d, b = 2, 2, 37, 8, 8
    Q, K, V = _rand((B, H, L, d), 1), _rand((B, H, L, d), 2), _rand((B, H, L, d), 3)
    vl = np.array([37, 20], np.int32)
    NB = -(-L // b)
    sel = oracle.select_blocks(Q, K, vl, b, NB, bidir=True)
    gw = np.zeros((H, 2 * d), np.float32)
    f = oracle.attn_fwd(Q, K, V, vl, sel, gw, None, b, NB, L, bidir=True)
    for r in range(B):
        p0 = L - int(vl[r])
        q, k, v = (torch.from_numpy(t[r, :, p0:].astype(np.float64)) for t in (Q, K, V))
        ref = torch.nn.functional.scaled_dot_product_attention(q, k, v).numpy()
        for h in range(H):
            for got in (f.o_lt, f.o_st, f.O):
                assert np.max(np.abs(got[r * H + h, p0:] - ref[h])) < 1e-12
            assert np.all(f.O[r * H + h, :p0] == 0)


def test_bidirectional_backward_finite_differences():
    B, H, L, d, b, k, w = 1, 2, 21, 4, 4, 2, 3
    rng = np.random.default_rng(5)
    Q, K, V, dO = (rng.standard_normal((B, H, L, d)) for _ in range(4))
    vl = np.array([17], np.int32)
    gw = rng.standard_normal((H, 2 * d)) * 0.3
    gb = rng.standard_normal(H) * 0.2
    sel = oracle.select_blocks(Q.astype(np.float32), K.astype(np.float32), vl, b, k, bidir=True)
    kw = dict(f64=True, stis_block=2, bidir=True)
    g = oracle.attn_bwd(Q, K, V, vl, sel, gw, gb, dO, b, k, w, **kw)
    loss = lambda q_, k_, v_, gw_, gb_: float(np.sum(oracle.attn_fwd(q_, k_, v_, vl, sel, gw_, gb_, b, k, w, **kw).O
                                                      * dO.reshape(B * H, L, d)))
    eps = 1e-6
    for name, arr, grad in (("Q", Q, g.dQ), ("K", K, g.dK), ("V", V, g.dV)):
        for idx in [(0, 0, 5, 1), (0, 1, 16, 3), (0, 0, 20, 0), (0, 1, 4, 2), (0, 0, 9, 2)]:
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += eps
            lo[idx] -= eps
            args = lambda a: (a if name == "Q" else Q, a if name == "K" else K, a if name == "V" else V, gw, gb)
            fd = (loss(*args(hi)) - loss(*args(lo))) / (2 * eps)
            got = grad[idx[1], idx[2], idx[3]]
            assert abs(fd - got) <= 1e-6 * (abs(fd) + 1.0), (name, idx, fd, got)
    # padding gets no gradient; a key AFTER the query now does
    assert np.all(g.dQ[:, :4] == 0) and np.all(g.dK[:, :4] == 0)
    assert np.abs(g.dK[:, 20]).max() > 0
