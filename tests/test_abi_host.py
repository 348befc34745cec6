"""Host-only checks of the C ABI: the library loads, exports what include/blossom.h declares,
and rejects bad arguments before touching the GPU (no kernel is launched here)."""
import ctypes
import os
import re

import pytest

from paper_2512_13368_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    return B.lib()


def test_exports_match_header(lib):
    hdr = open(os.path.join(ROOT, "include", "blossom.h")).read()
    declared = set(re.findall(r"\b(blossom_[a-z_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert B.version().startswith("blossom-gfx950")


def _p(**kw):
    base = dict(B=2, H=2, L=50, d=32, block=8, topk=2, window=8, dtype=B.F32)
    base.update(kw)
    return B.Params(**base)


def test_workspace_sizes(lib):
    p = _p()
    NB = 7
    assert B.workspace_bytes(p, B.WS_SELECT) == 2 * 2 * 2 * NB * 32 * 4
    assert B.workspace_bytes(p, B.WS_FWD) == 0
    assert B.workspace_bytes(p, B.WS_BWD) >= 2 * 2 * 50 * 16
    assert B.workspace_bytes(_p(d=48), B.WS_SELECT) == 0          # invalid params -> 0
    assert B.workspace_bytes(p, 99) == 0


def _select(lib, p, Q=16, K=16, vl=16, sel=16, ws=16, ws_bytes=1 << 30):
    cp = p.c()
    vp = ctypes.c_void_p
    return lib.blossom_select_blocks(ctypes.byref(cp), vp(Q), vp(K), vp(vl), vp(sel), vp(ws), ws_bytes, None)


def test_validation_codes_select(lib):
    # Pointers below are fake non-NULL addresses: every call must fail before they are used.
    assert _select(lib, _p(d=48)) == -3
    assert _select(lib, _p(block=12)) == -3
    assert _select(lib, _p(dtype=7)) == -3
    assert _select(lib, _p(stis_mode=3)) == -3                      # 0, 1 and 2 are the defined masks
    assert _select(lib, _p(stis_mode=1, stis_block=-1)) == -4
    assert _select(lib, _p(B=0)) == -2
    assert _select(lib, _p(L=0)) == -2
    assert _select(lib, _p(L=8 * 4097)) == -2                       # more than 4096 blocks
    assert _select(lib, _p(topk=0)) == -4
    assert _select(lib, _p(window=0)) == -4
    assert _select(lib, _p(softmax_scale=-1.0)) == -4
    assert _select(lib, _p(softmax_scale=float("nan"))) == -4
    assert _select(lib, _p(), Q=0) == -1
    assert _select(lib, _p(), sel=0) == -1
    assert _select(lib, _p(), Q=24) == -5                           # misaligned
    assert _select(lib, _p(), ws=0) == -6
    assert _select(lib, _p(), ws_bytes=16) == -6
    assert _select(lib, _p(), ws=24) == -5
    assert lib.blossom_select_blocks(None, None, None, None, None, None, 0, None) == -1
    assert lib.blossom_select_blocks_cmp(None, None, None, None, None, None, 0, None) == -1


def test_validation_codes_fwd_bwd_dense(lib):
    vp = ctypes.c_void_p
    a = vp(4096)
    cp = _p().c()
    fwd = lambda **k: lib.blossom_attn_fwd(ctypes.byref(k.get("p", cp)), k.get("Q", a), a, a, a, a,
                                           k.get("gw", a), None, k.get("O", a), k.get("o_lt", None), None,
                                           None, None, None, 0, None)
    assert fwd(Q=None) == -1
    assert fwd(gw=None) == -1
    assert fwd(O=vp(4100)) == -5
    assert fwd(p=_p(save_for_bwd=1).c()) == -1                      # saved outputs required
    assert fwd(p=_p(d=24).c()) == -3
    bwd = lambda **k: lib.blossom_attn_bwd(ctypes.byref(k.get("p", cp)), a, a, a, a, a, a, None, a, a, a, a,
                                           k.get("dO", a), a, a, a, k.get("dgw", a), None,
                                           k.get("ws", a), k.get("n", 1 << 30), None)
    assert bwd(dO=None) == -1
    assert bwd(dgw=None) == -1
    assert bwd(ws=None) == -6
    assert bwd(n=8) == -6
    assert bwd(p=_p(topk=0).c()) == -4
    assert bwd(p=_p(last_block_only=1).c()) == -3                   # serving mode has no backward
    dense = lambda **k: lib.blossom_dense_causal_fwd(ctypes.byref(k.get("p", cp)), k.get("Q", a), a, a, a,
                                                     k.get("O", a), None, None, 0, None)
    assert dense(Q=None) == -1
    assert dense(O=vp(4104)) == -5
    assert dense(p=_p(block=5).c()) == -3
    assert dense(p=_p(topk=0, window=0).c(), Q=None) == -1          # ignored fields never reject


def test_validation_codes_rope_and_probe(lib):
    vp = ctypes.c_void_p
    a = vp(4096)
    cp = _p().c()
    rs = lambda **k: lib.blossom_rope_select_blocks(ctypes.byref(k.get("p", cp)), a, a, k.get("cos", a), k.get("sin", a), a,
                                                    k.get("Qr", a), a, a, k.get("ws", a), 1 << 30, None)
    assert rs(cos=None) == -1 and rs(sin=None) == -1 and rs(Qr=None) == -1
    assert rs(cos=vp(4100)) == -5
    assert rs(ws=None) == -6
    assert rs(p=_p(d=12).c()) == -3
    br = lambda **k: lib.blossom_attn_bwd_rope(ctypes.byref(cp), a, a, a, a, a, a, None, a, a, a, a, a, k.get("cos", a),
                                               k.get("sin", a), a, a, a, a, None, k.get("ws", a), 1 << 30, None)
    assert br(cos=None) == -1 and br(sin=None) == -1
    assert br(sin=vp(4104)) == -5
    assert br(ws=None) == -6
    assert lib.blossom_probe(0, None, a, a, 4, None) == -1
    assert lib.blossom_probe(9, a, a, a, 4, None) == -4 and lib.blossom_probe(0, a, a, a, 3, None) == -4
    assert B.probe_bytes(0) == 8 * 128 * 64 * 64 * 2 and B.probe_bytes(1) == 4096 * 128 * 4 and B.probe_bytes(2) == 0
    # the selection entry point with its scratch inside the library: same checks as blossom_select_blocks
    st = lambda **k: lib.blossom_select_blocks_static(ctypes.byref(k.get("p", cp)), k.get("Q", a), a, a, a, None)
    assert st(Q=None) == -1 and st(Q=vp(4100)) == -5 and st(p=_p(topk=0).c()) == -4


def test_validation_codes_select_positions(lib):
    vp = ctypes.c_void_p
    a = vp(4096)
    f32 = ctypes.c_float
    call = lambda p, G=2, l=32, s=16, sc=0.0, Q=a, ws=a, n=1 << 30: lib.blossom_select_positions(
        ctypes.byref(p.c()), G, l, s, f32(sc), Q, a, a, a, ws, n, None)
    ok = _p(H=4, L=200, d=8, block=16, topk=4)
    assert call(ok, Q=None) == -1
    assert call(ok, G=3) == -4                       # heads not divisible by the groups
    assert call(ok, s=5) == -4                       # the stride divides neither block size
    assert call(ok, l=24, s=16) == -4
    assert call(ok, sc=-1.0) == -4
    assert call(_p(H=4, L=200, d=12, block=16, topk=4)) == -3
    assert call(_p(H=4, L=16 * 600, d=8, block=16, topk=4)) == -2   # more than 512 selection blocks
    assert call(ok, ws=None) == -6 and call(ok, n=8) == -6
    assert call(ok, Q=vp(4100)) == -5
    need = lib.blossom_select_positions_workspace_bytes(ctypes.byref(ok.c()), 2, 32, 16)
    assert need == 2 * 2 * 8 * ((200 - 32) // 16 + 1) * 4
    assert lib.blossom_select_positions_workspace_bytes(ctypes.byref(ok.c()), 3, 32, 16) == 0


def test_validation_codes_attn_fwd_positions(lib):
    vp = ctypes.c_void_p
    a = vp(4096)
    call = lambda p, G=2, Q=a, O=a, sel=a, o_lt=None: lib.blossom_attn_fwd_positions(
        ctypes.byref(p.c()), G, Q, a, a, a, sel, a, None, O, o_lt, None, None, None, None)
    ok = _p(H=4, L=200, d=8, block=16, topk=4, window=8)
    assert call(ok, Q=None) == -1 and call(ok, sel=None) == -1 and call(ok, O=None) == -1
    assert call(ok, G=3) == -4 and call(ok, G=0) == -4       # the groups must divide the heads
    assert call(ok, Q=vp(4100)) == -5 and call(ok, o_lt=vp(4100)) == -5
    assert call(_p(H=4, L=200, d=8, block=32, topk=4, window=8)) == -3    # selection block outside {8, 16}
    assert call(_p(H=4, L=200, d=64, block=16, topk=4, window=8)) == -3   # head size outside {8, 16, 32}
    assert call(_p(H=4, L=16 * 65, d=8, block=16, topk=4, window=8)) == -3  # more than 64 selection blocks
    assert call(_p(H=4, L=200, d=8, block=16, topk=4, window=8, stis_mode=2, stis_block=1)) == -3
    assert call(_p(H=4, L=200, d=8, block=16, topk=4, window=8, last_block_only=1)) == -3
    assert call(_p(H=4, L=200, d=8, block=16, topk=0, window=8)) == -4


def test_validation_codes_attn_bwd_positions(lib):
    vp = ctypes.c_void_p
    a = vp(4096)
    call = lambda p, G=2, Q=a, dK=a, sel=a, lse=a, ws=a, n=1 << 40: lib.blossom_attn_bwd_positions(
        ctypes.byref(p.c()), G, Q, a, a, a, sel, a, None, a, a, lse, a, a, a, dK, a, a, None, ws, n, None)
    ok = _p(H=4, L=200, d=8, block=16, topk=4, window=8)
    assert call(ok, Q=None) == -1 and call(ok, sel=None) == -1 and call(ok, dK=None) == -1 and call(ok, lse=None) == -1
    assert call(ok, G=3) == -4 and call(ok, G=0) == -4
    assert call(ok, Q=vp(4100)) == -5 and call(ok, dK=vp(4100)) == -5
    assert call(ok, ws=None) == -6 and call(ok, n=16) == -6 and call(ok, ws=vp(4100)) == -5
    assert call(_p(H=4, L=200, d=8, block=32, topk=4, window=8)) == -3
    assert call(_p(H=4, L=480, d=32, block=16, topk=4, window=8)) == -3   # the forward's limit, beyond the backward's
    assert call(_p(H=4, L=432, d=32, block=16, topk=4, window=8), ws=None) == -6   # the longest the backward takes
    assert call(_p(H=4, L=200, d=8, block=16, topk=4, window=8, stis_mode=2, stis_block=1)) == -3


def test_validation_codes_out_proj_ln(lib):
    vp = ctypes.c_void_p
    a = vp(4096)
    call = lambda p, Dm=64, O=a, W=a, S=a, g=a, bias=None, eps=1e-5: lib.blossom_out_proj_ln(
        ctypes.byref(p.c()), Dm, O, W, bias, a, g, a, ctypes.c_float(eps), S, None, None, None)
    ok = _p(H=2, L=200, d=32, block=16, topk=4)
    assert call(ok, O=None) == -1 and call(ok, W=None) == -1 and call(ok, S=None) == -1 and call(ok, g=None) == -1
    assert call(ok, Dm=0) == -4 and call(ok, eps=-1.0) == -4 and call(ok, eps=float("nan")) == -4
    assert call(ok, O=vp(4100)) == -5 and call(ok, bias=vp(4100)) == -5
    assert call(ok, Dm=2048) == -3 and call(ok, Dm=60) == -3          # beyond 1024; no multiple of 8
    assert call(_p(H=32, L=200, d=64, block=16, topk=4)) == -3          # H*d beyond 1024 on the scalar kernel


def test_strerror(lib):
    seen = set()
    for code in range(0, -9, -1):
        s = B.strerror(code)
        assert s and s != "unknown error code"
        seen.add(s)
    assert len(seen) == 9
    assert B.strerror(-99) == "unknown error code"
