"""The benchmark's closed-form count of unmasked pairs (its FLOP figure) against the oracle's
materialised masks."""
import numpy as np

import bench
from paper_2512_13368_amd.inputs import WORKLOADS, make_inputs, with_shape


def test_pair_counts_match_materialised_masks(oracle):
    for w in (WORKLOADS["cfg1"], with_shape(WORKLOADS["cfg2"], B=7),
              with_shape(WORKLOADS["cfg3"], B=2, H=1, L=300, len_lo=0, len_hi=300),
              with_shape(WORKLOADS["cfg2"], B=5, stis_block=1, window=8),
              with_shape(WORKLOADS["cfg3"], B=3, H=1, L=301, len_lo=0, len_hi=301, stis_block=32),
              with_shape(WORKLOADS["cfg1"], B=6, L=77, stis_block=5, window=3, len_lo=1, len_hi=77)):
        x = make_inputs(w)
        x.valid_len[0] = 0
        sel = oracle.select_blocks(x.Q, x.K, x.valid_len, w.block, w.topk)
        f = oracle.attn_fwd(x.Q, x.K, x.V, x.valid_len, sel, x.gate_w, x.gate_b, w.block, w.topk, w.window,
                            stis_block=w.stis_block)
        lt, st, dense = bench.algorithmic_pairs(w, x.valid_len, sel)
        assert (lt, st) == (f.nnz_lt, f.nnz_st)
        assert dense == sum(int(n) * (int(n) + 1) // 2 for n in x.valid_len) * w.H
