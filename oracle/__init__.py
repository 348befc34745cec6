"""CPU oracle for the Blossom attention hot path -- TEST INFRASTRUCTURE.

Thin ctypes marshalling around ``blossom_oracle.c`` (plain C, fp64 attention,
canonical fp32 block scoring).  Only ``tests/``, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py`` may import this package; the
product path never does, and this package never imports the HIP binding.

All arithmetic lives in the C file; this module only converts numpy arrays to
pointers and allocates outputs.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "blossom_oracle.c")
_LIB = os.path.join(_HERE, "libblossom_oracle.so")

_c_int = ctypes.c_int
_c_dbl = ctypes.c_double
_vp = ctypes.c_void_p


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  No fast-math, no FMA contraction."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.oracle_num_threads.restype = _c_int
        L.oracle_select_blocks.restype = _c_int
        L.oracle_select_blocks.argtypes = [_c_int] * 6 + [_vp, _vp, _vp, _vp, _c_int, _vp, _vp]
        L.oracle_select_blocks_bidir.restype = _c_int
        L.oracle_select_blocks_bidir.argtypes = [_c_int] * 6 + [_vp, _vp, _vp, _vp, _c_int, _vp, _vp]
        L.oracle_select_blocks_cmp.restype = _c_int
        L.oracle_select_blocks_cmp.argtypes = [_c_int] * 6 + [_vp, _vp, _vp, _vp, _c_int, _vp, _vp]
        L.oracle_build_masks.restype = _c_int
        L.oracle_build_masks.argtypes = [_c_int] * 7 + [_vp, _vp, _vp]
        L.oracle_masked_attention.restype = _c_int
        L.oracle_masked_attention.argtypes = [_c_int, _c_int, _vp, _vp, _vp, _vp, _c_dbl, _vp, _vp]
        L.oracle_attn_fwd.restype = _c_int
        L.oracle_attn_fwd.argtypes = ([_c_int] * 9 + [_c_dbl, _c_int] + [_vp] * 7 + [_vp, _c_int]
                                      + [_vp] * 7)
        L.oracle_out_proj_ln.restype = _c_int
        L.oracle_out_proj_ln.argtypes = [_c_int] * 5 + [_vp] * 6 + [_c_dbl] + [_vp] * 3
        L.oracle_attn_bwd.restype = _c_int
        L.oracle_attn_bwd.argtypes = ([_c_int] * 9 + [_c_dbl, _c_int] + [_vp] * 8 + [_vp, _c_int]
                                      + [_vp] * 5)
        L.oracle_dense_causal_fwd.restype = _c_int
        L.oracle_dense_causal_fwd.argtypes = ([_c_int] * 4 + [_c_dbl, _c_int] + [_vp] * 4
                                              + [_vp, _c_int, _vp, _vp])
        L.oracle_select_positions.restype = _c_int
        L.oracle_select_positions.argtypes = [_c_int] * 9 + [_c_dbl, _vp, _vp, _vp, _vp, _vp]
        L.oracle_canon_exp.restype = ctypes.c_float
        L.oracle_canon_exp.argtypes = [ctypes.c_float]
        L.oracle_rope.restype = _c_int
        L.oracle_rope.argtypes = [_c_int, _c_int, _c_int, _vp, _vp, _vp, _c_int, _vp]
        L.oracle_rope_bwd.restype = _c_int
        L.oracle_rope_bwd.argtypes = [_c_int, _c_int, _c_int, _vp, _vp, _vp, _vp]
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _p(a):
    return None if a is None else a.ctypes.data_as(_vp)


def _in(a, f64):
    return np.ascontiguousarray(a, dtype=np.float64 if f64 else np.float32)


def _bh(bh_list, B, H):
    if bh_list is None:
        return None, B * H
    a = np.ascontiguousarray(bh_list, dtype=np.int32)
    assert a.ndim == 1 and a.size > 0 and a.min() >= 0 and a.max() < B * H
    return a, int(a.size)


def _stis(stis_block, block, bidir):
    """Mask block as the C side takes it: 0 = causal window only, n = causal Eq. 15 with mask block n,
    -n = the bidirectional form (Eq. 15 as printed, no causal mask in either branch) with mask block n."""
    if not bidir:
        return int(stis_block)
    return -int(stis_block if stis_block > 0 else block)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def select_blocks(Q, K, valid_len, block, topk, bh_list=None, want_scores=False, bidir=False):
    """Steps 1-3.  Q, K: [B,H,L,d] float32.  Returns sel [B,H,NB,k] int32 (rows of pairs
    not in bh_list are left at -2) and, if asked, scores [n_bh,NB,NB] float32.  bidir: candidates on
    both sides of the query block (bidirectional backbone)."""
    Q = _in(Q, False)
    K = _in(K, False)
    B, H, L, d = Q.shape
    NB = -(-L // block)
    vl = np.ascontiguousarray(valid_len, dtype=np.int32)
    assert vl.shape == (B,)
    bh, n_bh = _bh(bh_list, B, H)
    sel = np.full((B, H, NB, topk), -2, dtype=np.int32)
    scores = np.zeros((n_bh, NB, NB), dtype=np.float32) if want_scores else None
    fn = lib().oracle_select_blocks_bidir if bidir else lib().oracle_select_blocks
    rc = fn(B, H, L, d, block, topk, _p(Q), _p(K), _p(vl), _p(bh), n_bh, _p(sel), _p(scores))
    _check(rc, "select_blocks")
    return (sel, scores) if want_scores else sel


def select_blocks_cmp(Q, Kcmp, valid_len, block, topk, bh_list=None, want_scores=False):
    """Steps 2-3 with caller-supplied compressed keys (Eq. 9 with the caller's phi): Q [B,H,L,d],
    Kcmp [B,H,NB,d] float32.  Same returns as select_blocks."""
    Q = _in(Q, False)
    Kcmp = _in(Kcmp, False)
    B, H, L, d = Q.shape
    NB = -(-L // block)
    assert Kcmp.shape == (B, H, NB, d)
    vl = np.ascontiguousarray(valid_len, dtype=np.int32)
    assert vl.shape == (B,)
    bh, n_bh = _bh(bh_list, B, H)
    sel = np.full((B, H, NB, topk), -2, dtype=np.int32)
    scores = np.zeros((n_bh, NB, NB), dtype=np.float32) if want_scores else None
    rc = lib().oracle_select_blocks_cmp(B, H, L, d, block, topk, _p(Q), _p(Kcmp), _p(vl), _p(bh), n_bh,
                                        _p(sel), _p(scores))
    _check(rc, "select_blocks_cmp")
    return (sel, scores) if want_scores else sel


def build_masks(L, block, topk, window, n_valid, sel_bh, stis_block=0, bidir=False, per_position=False):
    """The two materialised masks of one (row, head): uint8 [L,L] each.

    stis_block = 0: the short-term mask is the causal local window; >= 1: the causal form of all
    three terms of Eq. 15 with that mask block size."""
    s = np.ascontiguousarray(sel_bh, dtype=np.int32)
    NB = L if per_position else -(-L // block)
    assert s.shape == (NB, topk)
    M_lt = np.zeros((L, L), dtype=np.uint8)
    M_st = np.zeros((L, L), dtype=np.uint8)
    _check(lib().oracle_build_masks(L, block, 1 if per_position else block, topk, window, _stis(stis_block, block, bidir), int(n_valid), _p(s), _p(M_lt), _p(M_st)),
           "build_masks")
    return M_lt, M_st


def masked_attention(q, k, v, M, scale):
    """Eq. 1 for one head: q,k,v [L,d] float64, M uint8 [L,L].  Returns o [L,d], lse [L]."""
    q = _in(q, True)
    k = _in(k, True)
    v = _in(v, True)
    M = np.ascontiguousarray(M, dtype=np.uint8)
    L, d = q.shape
    o = np.zeros((L, d), dtype=np.float64)
    lse = np.zeros(L, dtype=np.float64)
    _check(lib().oracle_masked_attention(L, d, _p(q), _p(k), _p(v), _p(M), float(scale), _p(o), _p(lse)),
           "masked_attention")
    return o, lse


@dataclass
class Fwd:
    O: np.ndarray        # [n_bh,L,d] float64
    o_lt: np.ndarray
    o_st: np.ndarray
    lse_lt: np.ndarray   # [n_bh,L]
    lse_st: np.ndarray
    alpha: np.ndarray
    nnz_lt: int
    nnz_st: int


def attn_fwd(Q, K, V, valid_len, sel, gate_w, gate_b, block, topk, window, scale=None,
             bh_list=None, f64=False, stis_block=0, bidir=False, per_position=False) -> Fwd:
    Q = _in(Q, f64)
    K = _in(K, f64)
    V = _in(V, f64)
    B, H, L, d = Q.shape
    if scale is None or scale == 0.0:
        scale = 1.0 / np.sqrt(d)
    vl = np.ascontiguousarray(valid_len, dtype=np.int32)
    sel = np.ascontiguousarray(sel, dtype=np.int32)
    NB = L if per_position else -(-L // block)
    assert sel.shape == (B, H, NB, topk)
    gw = _in(gate_w, f64)
    assert gw.shape == (H, 2 * d)
    gb = None if gate_b is None else _in(gate_b, f64)
    bh, n_bh = _bh(bh_list, B, H)
    z = lambda *s: np.zeros(s, dtype=np.float64)
    out = Fwd(z(n_bh, L, d), z(n_bh, L, d), z(n_bh, L, d), z(n_bh, L), z(n_bh, L), z(n_bh, L), 0, 0)
    nnz = np.zeros(2, dtype=np.int64)
    rc = lib().oracle_attn_fwd(B, H, L, d, block, 1 if per_position else block, topk, window, _stis(stis_block, block, bidir), float(scale), int(f64),
                               _p(Q), _p(K), _p(V), _p(vl), _p(sel), _p(gw), _p(gb), _p(bh), n_bh,
                               _p(out.O), _p(out.o_lt), _p(out.o_st), _p(out.lse_lt), _p(out.lse_st),
                               _p(out.alpha), _p(nnz))
    _check(rc, "attn_fwd")
    out.nnz_lt, out.nnz_st = int(nnz[0]), int(nnz[1])
    return out


@dataclass
class Bwd:
    dQ: np.ndarray        # [n_bh,L,d] float64
    dK: np.ndarray
    dV: np.ndarray
    d_gate_w: np.ndarray  # [H,2d], summed over the listed pairs
    d_gate_b: np.ndarray  # [H]


def attn_bwd(Q, K, V, valid_len, sel, gate_w, gate_b, dO, block, topk, window, scale=None,
             bh_list=None, f64=False, stis_block=0, bidir=False, per_position=False) -> Bwd:
    Q = _in(Q, f64)
    K = _in(K, f64)
    V = _in(V, f64)
    dO = _in(dO, f64)
    B, H, L, d = Q.shape
    assert dO.shape == Q.shape
    if scale is None or scale == 0.0:
        scale = 1.0 / np.sqrt(d)
    vl = np.ascontiguousarray(valid_len, dtype=np.int32)
    sel = np.ascontiguousarray(sel, dtype=np.int32)
    gw = _in(gate_w, f64)
    gb = None if gate_b is None else _in(gate_b, f64)
    bh, n_bh = _bh(bh_list, B, H)
    z = lambda *s: np.zeros(s, dtype=np.float64)
    out = Bwd(z(n_bh, L, d), z(n_bh, L, d), z(n_bh, L, d), z(H, 2 * d), z(H))
    rc = lib().oracle_attn_bwd(B, H, L, d, block, 1 if per_position else block, topk, window, _stis(stis_block, block, bidir), float(scale), int(f64),
                               _p(Q), _p(K), _p(V), _p(vl), _p(sel), _p(gw), _p(gb), _p(dO),
                               _p(bh), n_bh, _p(out.dQ), _p(out.dK), _p(out.dV),
                               _p(out.d_gate_w), _p(out.d_gate_b))
    _check(rc, "attn_bwd")
    return out


def dense_causal_fwd(Q, K, V, valid_len, scale=None, bh_list=None, f64=False):
    Q = _in(Q, f64)
    K = _in(K, f64)
    V = _in(V, f64)
    B, H, L, d = Q.shape
    if scale is None or scale == 0.0:
        scale = 1.0 / np.sqrt(d)
    vl = np.ascontiguousarray(valid_len, dtype=np.int32)
    bh, n_bh = _bh(bh_list, B, H)
    O = np.zeros((n_bh, L, d), dtype=np.float64)
    lse = np.zeros((n_bh, L), dtype=np.float64)
    rc = lib().oracle_dense_causal_fwd(B, H, L, d, float(scale), int(f64), _p(Q), _p(K), _p(V),
                                       _p(vl), _p(bh), n_bh, _p(O), _p(lse))
    _check(rc, "dense_causal_fwd")
    return O, lse


def rope(x, cos, sin, to_bf16=False):
    """Step 0: rotary position embedding of x [..., L, d] (fp32 recipe of the C file's header) with the
    caller's tables cos, sin [L, d/2] float32.  to_bf16 rounds the result to bf16 values."""
    x = _in(x, False)
    L, d = x.shape[-2:]
    cos = _in(cos, False)
    sin = _in(sin, False)
    assert cos.shape == (L, d // 2) and sin.shape == (L, d // 2)
    out = np.empty_like(x)
    _check(lib().oracle_rope(int(x.size // (L * d)), L, d, _p(x), _p(cos), _p(sin), int(bool(to_bf16)), _p(out)), "rope")
    return out


def rope_bwd(g, cos, sin):
    """Gradient w.r.t. the unrotated rows from the gradient g [..., L, d] (float64) w.r.t. the rotated ones."""
    g = _in(g, True)
    L, d = g.shape[-2:]
    cos = _in(cos, False)
    sin = _in(sin, False)
    out = np.empty_like(g)
    _check(lib().oracle_rope_bwd(int(g.size // (L * d)), L, d, _p(g), _p(cos), _p(sin), _p(out)), "rope_bwd")
    return out


def canon_exp(x: float) -> float:
    """The canonical fp32 exponential of the printed selection rule (x <= 0)."""
    return float(lib().oracle_canon_exp(ctypes.c_float(x)))


def select_positions(Q, K, valid_len, cmp_block, stride, sel_block, topk, score_scale=1.0, want_scores=False):
    """The selection rule of Sec. 3.4 as printed (Eq. 8-13): Q [B,H,L,d], K [B,G,L,d] float32 (G key/value
    groups, H = G*Hg).  Returns sel [B,G,L,k] int32 (one ascending, -1 padded row per position and group) and,
    if asked, the group scores [B,G,L,ceil(L/sel_block)] float32."""
    Q = _in(Q, False)
    K = _in(K, False)
    B, H, L, d = Q.shape
    G = K.shape[1]
    assert K.shape == (B, G, L, d) and H % G == 0
    vl = np.ascontiguousarray(valid_len, dtype=np.int32)
    NBs = -(-L // sel_block)
    sel = np.full((B, G, L, topk), -2, dtype=np.int32)
    scores = np.zeros((B, G, L, NBs), dtype=np.float32) if want_scores else None
    rc = lib().oracle_select_positions(B, H, G, L, d, cmp_block, stride, sel_block, topk, float(score_scale),
                                       _p(Q), _p(K), _p(vl), _p(sel), _p(scores))
    _check(rc, "select_positions")
    return (sel, scores) if want_scores else sel


def out_proj_ln(O, Wt, H_prev, gamma, beta, eps, bias=None, want_stats=False):
    """The layer around the attention (Eq. 4 and the equation after Eq. 19, dropout = identity):
    S = LayerNorm(H_prev + Concat_h(O[:, h]) W^O (+ bias)).  O [B,H,L,d], Wt [Dm, H*d] (W^O transposed),
    H_prev [B,L,Dm], gamma, beta [Dm]; float64 throughout.  Returns S [B,L,Dm] (and mean, rstd [B,L])."""
    O = _in(O, True)
    B, H, L, d = O.shape
    Wt = _in(Wt, True)
    Dm = Wt.shape[0]
    assert Wt.shape == (Dm, H * d)
    H_prev = _in(H_prev, True)
    assert H_prev.shape == (B, L, Dm)
    gamma, beta = _in(gamma, True), _in(beta, True)
    assert gamma.shape == (Dm,) and beta.shape == (Dm,)
    bias = None if bias is None else _in(bias, True)
    S = np.empty((B, L, Dm), dtype=np.float64)
    mean = np.empty((B, L), dtype=np.float64)
    rstd = np.empty((B, L), dtype=np.float64)
    _check(lib().oracle_out_proj_ln(B, H, L, d, Dm, _p(O), _p(Wt), _p(bias), _p(H_prev), _p(gamma), _p(beta),
                                    float(eps), _p(S), _p(mean), _p(rstd)), "out_proj_ln")
    return (S, mean, rstd) if want_stats else S
