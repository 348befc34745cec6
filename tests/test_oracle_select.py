"""Pins for the oracle's block selection (Eq. 8-13 with one block size).

None of these tests re-implements the selection loop: they check it against a
hand-computed integer case, brute-force subset enumeration, float64 scores,
structural invariants and invariances.
"""
import itertools
import os

import numpy as np
import pytest

from paper_2512_13368_amd.inputs import WORKLOADS, make_inputs, with_shape

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden_case():
    L, d = 16, 2
    K = np.zeros((1, 1, L, d), np.float32)
    Q = np.zeros((1, 1, L, d), np.float32)
    K[0, 0, 0:2] = [100, 100]
    K[0, 0, 2] = [1, 0]
    K[0, 0, 3] = [3, 0]
    K[0, 0, 4:8] = [0, 2]
    K[0, 0, 8:12] = [2, 0]
    K[0, 0, 12:16] = [1, 1]
    Q[0, 0, 0:2] = [50, 50]
    Q[0, 0, 2:4] = [1, 1]
    Q[0, 0, 4:8] = [1, 0]
    Q[0, 0, 8:12] = [0, 1]
    Q[0, 0, 12:16] = [1, 0]
    return Q, K, np.array([14], np.int32)


def test_hand_computed_integer_case(oracle):
    Q, K, vl = _golden_case()
    expected = {}
    with open(os.path.join(GOLDEN, "select_integer_case.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, rows = line.split(":")
            expected[int(k)] = np.array([[int(t) for t in r.split()] for r in rows.split("|")], np.int32)
    assert sorted(expected) == [2, 3, 4]
    for k, exp in expected.items():
        sel = oracle.select_blocks(Q, K, vl, 4, k)
        np.testing.assert_array_equal(sel[0, 0], exp)


def test_signed_zero_scores_tie(oracle):
    # block 0 keys are all zero, block 1 is orthogonal to the query sum: both scores are zero (the
    # products are -0 and +0; the fused-multiply-add chain starts from +0, so both sums are +0),
    # they compare equal and index 0 wins.
    L, d, b = 12, 2, 4
    Q = np.zeros((1, 1, L, d), np.float32)
    K = np.zeros((1, 1, L, d), np.float32)
    Q[0, 0, 8:12] = [-1, 0]
    K[0, 0, 4:8] = [0, 1]
    sel, sc = oracle.select_blocks(Q, K, np.array([L], np.int32), b, 2, want_scores=True)
    assert sc[0, 2, 0] == 0.0 and sc[0, 2, 1] == 0.0
    np.testing.assert_array_equal(sel[0, 0, 2], [0, 2])


def _check_structure(sel, vl, L, b, k):
    B, H, NB, kk = sel.shape
    assert kk == k and NB == -(-L // b)
    for r in range(B):
        p0 = L - int(vl[r])
        J_first = p0 // b
        for h in range(H):
            for I in range(NB):
                row = sel[r, h, I]
                hi = min((I + 1) * b, L)
                if hi <= p0:
                    assert np.all(row == -1)
                    continue
                cnt = min(k, I - J_first + 1)
                got = row[:cnt]
                assert np.all(row[cnt:] == -1)
                assert np.all(np.diff(got) > 0)           # ascending, unique
                assert got[-1] == I                       # own block, and it is the largest
                assert got[0] >= J_first


def _brute_force(scores_row, cands, take):
    """Best `take`-subset: maximal descending-sorted score tuple; among maximisers the
    lexicographically smallest ascending index tuple."""
    best = None
    for comb in itertools.combinations(cands, take):
        key = tuple(sorted((float(scores_row[j]) for j in comb), reverse=True))
        if best is None or key > best[0] or (key == best[0] and comb < best[1]):
            best = (key, comb)
    return list(best[1]) if best else []


@pytest.mark.parametrize("case", [
    dict(name="cfg1"),
    dict(L=64, d=8, b=8, k=3, B=3, H=2, lo=5, hi=64, seed=7),
    dict(L=61, d=4, b=4, k=5, B=2, H=1, lo=0, hi=61, seed=8),
    dict(L=48, d=16, b=16, k=2, B=2, H=2, lo=48, hi=48, seed=9),
])
def test_bruteforce_topk_and_float64_scores(oracle, case):
    if "name" in case:
        w = WORKLOADS[case["name"]]
    else:
        w = with_shape(WORKLOADS["cfg1"], B=case["B"], H=case["H"], L=case["L"], d=case["d"],
                       block=case["b"], topk=case["k"], len_lo=case["lo"], len_hi=case["hi"],
                       seed=case["seed"])
    x = make_inputs(w)
    sel, sc = oracle.select_blocks(x.Q, x.K, x.valid_len, w.block, w.topk, want_scores=True)
    _check_structure(sel, x.valid_len, w.L, w.block, w.topk)
    NB, b = w.NB, w.block
    for r in range(w.B):
        p0 = w.L - int(x.valid_len[r])
        J_first = p0 // b
        for h in range(w.H):
            q64 = x.Q[r, h].astype(np.float64)
            k64 = x.K[r, h].astype(np.float64)
            for I in range(NB):
                lo, hi = I * b, min((I + 1) * b, w.L)
                if hi <= p0:
                    continue
                cands = list(range(J_first, I))
                # scores against an independent float64 pooling (valid positions only)
                qs = q64[max(lo, p0):hi].sum(0)
                for J in cands:
                    km = k64[max(J * b, p0):(J + 1) * b].mean(0)
                    ref = float(qs @ km)
                    tol = 1e-5 * (np.abs(qs) @ np.abs(km)) + 1e-30
                    assert abs(float(sc[r * w.H + h, I, J]) - ref) <= tol
                take = min(w.topk - 1, len(cands))
                expect = _brute_force(sc[r * w.H + h, I], cands, take) + [I]
                got = [int(t) for t in sel[r, h, I] if t >= 0]
                assert got == expect


def test_planted_duplicate_blocks_tie_break(oracle):
    # identical key blocks give bit-identical scores: the lower index must win
    w = with_shape(WORKLOADS["cfg1"], B=1, H=1, L=40, d=8, block=8, topk=3, len_lo=40, len_hi=40, seed=3)
    x = make_inputs(w)
    K = x.K.copy()
    K[0, 0, 16:24] = K[0, 0, 0:8]          # block 2 := block 0
    K[0, 0, 24:32] = K[0, 0, 0:8]          # block 3 := block 0
    sel, sc = oracle.select_blocks(x.Q, K, x.valid_len, 8, 3, want_scores=True)
    assert sc[0, 4, 0] == sc[0, 4, 2] == sc[0, 4, 3]
    row = [int(t) for t in sel[0, 0, 4]]
    picked = set(row[:-1])
    # among the three tied blocks the chosen ones must be the lowest-indexed
    tied_chosen = sorted(picked & {0, 2, 3})
    assert tied_chosen == [0, 2, 3][:len(tied_chosen)]


def test_invariances(oracle):
    w = with_shape(WORKLOADS["cfg2"], B=6, L=200, seed=11)
    x = make_inputs(w)
    base = oracle.select_blocks(x.Q, x.K, x.valid_len, w.block, w.topk)
    _check_structure(base, x.valid_len, w.L, w.block, w.topk)
    # power-of-two scaling of Q or K is exact in fp32 and cannot change any comparison
    np.testing.assert_array_equal(oracle.select_blocks(x.Q * 4, x.K, x.valid_len, w.block, w.topk), base)
    np.testing.assert_array_equal(oracle.select_blocks(x.Q, x.K * 0.25, x.valid_len, w.block, w.topk), base)
    # pad contents are ignored
    Q2, K2 = x.Q.copy(), x.K.copy()
    for r in range(w.B):
        p0 = w.L - int(x.valid_len[r])
        Q2[r, :, :p0] = 1e6
        K2[r, :, :p0] = -1e6
    np.testing.assert_array_equal(oracle.select_blocks(Q2, K2, x.valid_len, w.block, w.topk), base)
    # permuting rows and heads permutes the result
    pr = np.random.default_rng(0).permutation(w.B)
    np.testing.assert_array_equal(
        oracle.select_blocks(x.Q[pr][:, ::-1], x.K[pr][:, ::-1], x.valid_len[pr], w.block, w.topk),
        base[pr][:, ::-1])
    # a listed subset gives the same rows
    sub = oracle.select_blocks(x.Q, x.K, x.valid_len, w.block, w.topk, bh_list=[3, 7])
    np.testing.assert_array_equal(sub.reshape(-1, w.NB, w.topk)[[3, 7]], base.reshape(-1, w.NB, w.topk)[[3, 7]])


def test_edge_lengths(oracle):
    w = with_shape(WORKLOADS["cfg1"], B=4, L=50, seed=5)
    x = make_inputs(w)
    vl = np.array([0, 1, 50, 8], np.int32)
    sel = oracle.select_blocks(x.Q, x.K, vl, w.block, w.topk)
    _check_structure(sel, vl, w.L, w.block, w.topk)
    assert np.all(sel[0] == -1)                       # empty row
    assert np.all(sel[1, :, :-1] == -1) and np.all(sel[1, :, -1, 0] == w.NB - 1)
    # k = 1: only the own block
    sel1 = oracle.select_blocks(x.Q, x.K, vl, w.block, 1)
    assert np.all(sel1[2, :, :, 0] == np.arange(w.NB))
    # k larger than the number of blocks: every past block is taken
    selk = oracle.select_blocks(x.Q, x.K, vl, w.block, 12)
    for I in range(w.NB):
        np.testing.assert_array_equal(selk[2, 0, I, :I + 1], np.arange(I + 1))


# ---- caller-supplied compressed keys (Eq. 9 with the caller's phi) ---------------------------------

def test_compressed_keys_hand_case(oracle):
    # 4 blocks of 2 positions, d = 2, all valid.  Query sums per block: (2,0), (0,2), (2,2), (1,0).
    # Compressed keys: phi_0 = (1,0), phi_1 = (0,3), phi_2 = (5,5) (never a candidate of an earlier block).
    # Block 2 scores: 2*1 + 2*0 = 2 against block 0, 2*0 + 2*3 = 6 against block 1 -> picks 1.
    # Block 3 scores: 1, 0, 5 -> picks 2; with k = 3 also 0.
    L, d, b = 8, 2, 2
    Q = np.zeros((1, 1, L, d), np.float32)
    Q[0, 0, 0:2] = [1, 0]
    Q[0, 0, 2:4] = [0, 1]
    Q[0, 0, 4:6] = [1, 1]
    Q[0, 0, 6] = [1, 0]
    Kc = np.array([[[[1, 0], [0, 3], [5, 5], [9, 9]]]], np.float32)
    vl = np.array([L], np.int32)
    sel, sc = oracle.select_blocks_cmp(Q, Kc, vl, b, 2, want_scores=True)
    np.testing.assert_array_equal(sel[0, 0], [[0, -1], [0, 1], [1, 2], [2, 3]])
    np.testing.assert_array_equal(sc[0, 2, :2], [2.0, 6.0])
    np.testing.assert_array_equal(sc[0, 3, :3], [1.0, 0.0, 5.0])
    sel3 = oracle.select_blocks_cmp(Q, Kc, vl, b, 3)
    np.testing.assert_array_equal(sel3[0, 0], [[0, -1, -1], [0, 1, -1], [0, 1, 2], [0, 2, 3]])


def test_compressed_keys_equal_to_block_means_give_the_same_selection(oracle):
    # phi = mean over the block's valid keys, accumulated here in fp32 in ascending position
    # (np.float32 scalars round after every operation): the two entry points must then agree exactly
    w = with_shape(WORKLOADS["cfg1"], B=3, H=2, L=83, block=8, topk=3, seed=77)
    x = make_inputs(w)
    B, H, L, d = x.Q.shape
    NB = w.NB
    Kc = np.zeros((B, H, NB, d), np.float32)
    for r in range(B):
        p0 = L - int(x.valid_len[r])
        for h in range(H):
            for J in range(NB):
                acc = np.zeros(d, np.float32)
                cnt = 0
                for t in range(max(J * w.block, p0), min((J + 1) * w.block, L)):
                    acc = (acc + x.K[r, h, t].astype(np.float32)).astype(np.float32)
                    cnt += 1
                if cnt:
                    Kc[r, h, J] = acc / np.float32(cnt)
    np.testing.assert_array_equal(oracle.select_blocks_cmp(x.Q, Kc, x.valid_len, w.block, w.topk),
                                  oracle.select_blocks(x.Q, x.K, x.valid_len, w.block, w.topk))


def test_compressed_keys_brute_force(oracle):
    # float64 scores from the definition; the chosen past blocks must be a best subset of their size
    rng = np.random.default_rng(5)
    B, H, L, d, b, k = 2, 2, 37, 6, 5, 3
    NB = -(-L // b)
    Q = rng.standard_normal((B, H, L, d)).astype(np.float32)
    Kc = rng.standard_normal((B, H, NB, d)).astype(np.float32)
    vl = np.array([L, 22], np.int32)
    sel = oracle.select_blocks_cmp(Q, Kc, vl, b, k)
    for r in range(B):
        p0 = L - int(vl[r])
        J_first = p0 // b
        for h in range(H):
            for I in range(NB):
                lo, hi = max(I * b, p0), min((I + 1) * b, L)
                if hi <= p0:
                    assert (sel[r, h, I] == -1).all()
                    continue
                qsum = Q[r, h, lo:hi].astype(np.float64).sum(0)
                cand = list(range(J_first, I))
                sc = {J: float(qsum @ Kc[r, h, J].astype(np.float64)) for J in cand}
                got = [int(J) for J in sel[r, h, I] if J >= 0]
                assert got[-1] == I and got == sorted(got)
                past = got[:-1]
                assert len(past) == min(k - 1, len(cand))
                if past:
                    worst_in = min(sc[J] for J in past)
                    best_out = max([sc[J] for J in cand if J not in past], default=-np.inf)
                    assert worst_in >= best_out - 1e-5
