"""Python binding of libblossom.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI of
``include/blossom.h``; this module turns torch device tensors into pointers,
allocates outputs and workspaces with torch, and raises on error codes.  There
is no CPU fallback: a missing library is an ImportError-like failure.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libblossom.so")

F32, BF16 = 0, 1
WS_SELECT, WS_FWD, WS_BWD, WS_DENSE = 0, 1, 2, 3

EXPORTS = ("blossom_workspace_bytes", "blossom_select_blocks", "blossom_select_blocks_static", "blossom_select_blocks_cmp",
           "blossom_rope_select_blocks", "blossom_attn_bwd_rope", "blossom_select_positions_workspace_bytes",
           "blossom_select_positions", "blossom_attn_fwd_positions", "blossom_attn_bwd_positions", "blossom_out_proj_ln", "blossom_attn_fwd", "blossom_attn_bwd",
           "blossom_attn_bwd_stages", "blossom_dense_causal_fwd", "blossom_probe_bytes", "blossom_probe", "blossom_strerror", "blossom_version")
PROBE_WORKGROUPS = 4096
BWD_GATE, BWD_INVERSE, BWD_DQ, BWD_DKV, BWD_ALL = 1, 2, 4, 8, 15


class BlossomParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("L", ctypes.c_int32), ("d", ctypes.c_int32),
                ("block", ctypes.c_int32), ("topk", ctypes.c_int32), ("window", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
                ("stis_mode", ctypes.c_int32), ("save_for_bwd", ctypes.c_int32),
                ("stis_block", ctypes.c_int32), ("last_block_only", ctypes.c_int32)]


class BlossomError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} (code {code})")


_lib = None


def lib() -> ctypes.CDLL:
    """Open libblossom.so (after torch, so that both use one HIP runtime instance)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`"
                " (there is no fallback path)")
        import torch  # noqa: F401  (loads torch's HIP runtime first)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32p, fp = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
        pp = ctypes.POINTER(BlossomParams)
        L.blossom_workspace_bytes.restype = ctypes.c_size_t
        L.blossom_workspace_bytes.argtypes = [pp, ctypes.c_int]
        L.blossom_select_blocks.restype = ctypes.c_int
        L.blossom_select_blocks.argtypes = [pp, vp, vp, i32p, i32p, vp, ctypes.c_size_t, vp]
        L.blossom_select_blocks_static.restype = ctypes.c_int
        L.blossom_select_blocks_static.argtypes = [pp, vp, vp, i32p, i32p, vp]
        L.blossom_rope_select_blocks.restype = ctypes.c_int
        L.blossom_rope_select_blocks.argtypes = [pp, vp, vp, fp, fp, i32p, vp, vp, i32p, vp, ctypes.c_size_t, vp]
        L.blossom_select_positions_workspace_bytes.restype = ctypes.c_size_t
        L.blossom_select_positions_workspace_bytes.argtypes = [pp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
        L.blossom_select_positions.restype = ctypes.c_int
        L.blossom_select_positions.argtypes = [pp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_float,
                                               vp, vp, i32p, i32p, vp, ctypes.c_size_t, vp]
        L.blossom_attn_fwd_positions.restype = ctypes.c_int
        L.blossom_attn_fwd_positions.argtypes = [pp, ctypes.c_int32] + [vp] * 12 + [vp]
        L.blossom_attn_bwd_positions.restype = ctypes.c_int
        L.blossom_attn_bwd_positions.argtypes = [pp, ctypes.c_int32, vp, vp, vp, i32p, i32p, fp, fp, vp, vp, fp, fp, vp, vp,
                                                 vp, vp, fp, fp, vp, ctypes.c_size_t, vp]
        L.blossom_out_proj_ln.restype = ctypes.c_int
        L.blossom_out_proj_ln.argtypes = [pp, ctypes.c_int32, vp, vp, fp, vp, fp, fp, ctypes.c_float, vp, fp, fp, vp]
        L.blossom_select_blocks_cmp.restype = ctypes.c_int
        L.blossom_select_blocks_cmp.argtypes = [pp, vp, vp, i32p, i32p, vp, ctypes.c_size_t, vp]
        L.blossom_attn_fwd.restype = ctypes.c_int
        L.blossom_attn_fwd.argtypes = [pp, vp, vp, vp, i32p, i32p, fp, fp, vp, vp, vp, fp, fp, vp,
                                       ctypes.c_size_t, vp]
        L.blossom_attn_bwd.restype = ctypes.c_int
        L.blossom_attn_bwd.argtypes = [pp, vp, vp, vp, i32p, i32p, fp, fp, vp, vp, fp, fp, vp, vp, vp, vp,
                                       fp, fp, vp, ctypes.c_size_t, vp]
        L.blossom_attn_bwd_rope.restype = ctypes.c_int
        L.blossom_attn_bwd_rope.argtypes = [pp, vp, vp, vp, i32p, i32p, fp, fp, vp, vp, fp, fp, vp, fp, fp, vp, vp, vp,
                                            fp, fp, vp, ctypes.c_size_t, vp]
        L.blossom_attn_bwd_stages.restype = ctypes.c_int
        L.blossom_attn_bwd_stages.argtypes = L.blossom_attn_bwd.argtypes + [ctypes.c_uint]
        L.blossom_dense_causal_fwd.restype = ctypes.c_int
        L.blossom_dense_causal_fwd.argtypes = [pp, vp, vp, vp, i32p, vp, fp, vp, ctypes.c_size_t, vp]
        L.blossom_probe_bytes.restype = ctypes.c_size_t
        L.blossom_probe_bytes.argtypes = [ctypes.c_int]
        L.blossom_probe.restype = ctypes.c_int
        L.blossom_probe.argtypes = [ctypes.c_int, vp, vp, fp, ctypes.c_int, vp]
        L.blossom_strerror.restype = ctypes.c_char_p
        L.blossom_strerror.argtypes = [ctypes.c_int]
        L.blossom_version.restype = ctypes.c_char_p
        L.blossom_version.argtypes = []
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().blossom_strerror(int(code)).decode()


def version() -> str:
    return lib().blossom_version().decode()


@dataclass
class Params:
    B: int
    H: int
    L: int
    d: int
    block: int
    topk: int
    window: int
    dtype: int = F32
    softmax_scale: float = 0.0
    stis_mode: int = 0
    save_for_bwd: int = 0
    stis_block: int = 0
    last_block_only: int = 0

    @property
    def NB(self) -> int:
        return -(-self.L // self.block)

    def c(self) -> BlossomParams:
        return BlossomParams(self.B, self.H, self.L, self.d, self.block, self.topk, self.window,
                             self.dtype, self.softmax_scale, self.stis_mode, self.save_for_bwd, self.stis_block,
                             self.last_block_only)


def workspace_bytes(p: Params, which: int) -> int:
    cp = p.c()
    return int(lib().blossom_workspace_bytes(ctypes.byref(cp), which))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _torch_dtype(p: Params):
    import torch
    return torch.float32 if p.dtype == F32 else torch.bfloat16


def _check_tensor(t, shape, dtype, name):
    if t is None:
        return
    if tuple(t.shape) != tuple(shape) or t.dtype != dtype or not t.is_contiguous() or not t.is_cuda:
        raise ValueError(f"{name}: expected contiguous cuda tensor {tuple(shape)} {dtype}, got "
                         f"{tuple(t.shape)} {t.dtype} contiguous={t.is_contiguous()} cuda={t.is_cuda}")


def _workspace(p: Params, which: int, ws, device):
    import torch
    need = workspace_bytes(p, which)
    if ws is None and need > 0:
        ws = torch.empty(need, dtype=torch.uint8, device=device)
    nbytes = 0 if ws is None else ws.numel() * ws.element_size()
    return ws, nbytes


def select_blocks(p: Params, Q, K, valid_len, sel=None, ws=None, stream=None):
    import torch
    shp = (p.B, p.H, p.L, p.d)
    _check_tensor(Q, shp, _torch_dtype(p), "Q")
    _check_tensor(K, shp, _torch_dtype(p), "K")
    _check_tensor(valid_len, (p.B,), torch.int32, "valid_len")
    if sel is None:
        sel = torch.empty((p.B, p.H, p.NB, p.topk), dtype=torch.int32, device=Q.device)
    _check_tensor(sel, (p.B, p.H, p.NB, p.topk), torch.int32, "sel")
    ws, nbytes = _workspace(p, WS_SELECT, ws, Q.device)
    cp = p.c()
    rc = lib().blossom_select_blocks(ctypes.byref(cp), _ptr(Q), _ptr(K), _ptr(valid_len), _ptr(sel),
                                     _ptr(ws), nbytes, _stream(stream))
    if rc:
        raise BlossomError(rc, "blossom_select_blocks")
    return sel


def select_blocks_static(p: Params, Q, K, valid_len, sel, stream=None):
    """blossom_select_blocks_static: no workspace, nothing allocated (the caller passes `sel`)."""
    import torch
    shp = (p.B, p.H, p.L, p.d)
    _check_tensor(Q, shp, _torch_dtype(p), "Q")
    _check_tensor(K, shp, _torch_dtype(p), "K")
    _check_tensor(valid_len, (p.B,), torch.int32, "valid_len")
    if sel is None:
        raise ValueError("sel is required: this entry point allocates nothing")
    _check_tensor(sel, (p.B, p.H, p.NB, p.topk), torch.int32, "sel")
    cp = p.c()
    rc = lib().blossom_select_blocks_static(ctypes.byref(cp), _ptr(Q), _ptr(K), _ptr(valid_len), _ptr(sel),
                                            _stream(stream))
    if rc:
        raise BlossomError(rc, "blossom_select_blocks_static")
    return sel


def rope_select_blocks(p: Params, Q, K, rope_cos, rope_sin, valid_len, Q_rot=None, K_rot=None, sel=None, ws=None,
                       stream=None):
    """blossom_rope_select_blocks: returns (Q_rot, K_rot, sel)."""
    import torch
    shp = (p.B, p.H, p.L, p.d)
    dt = _torch_dtype(p)
    _check_tensor(Q, shp, dt, "Q")
    _check_tensor(K, shp, dt, "K")
    _check_tensor(rope_cos, (p.L, p.d // 2), torch.float32, "rope_cos")
    _check_tensor(rope_sin, (p.L, p.d // 2), torch.float32, "rope_sin")
    _check_tensor(valid_len, (p.B,), torch.int32, "valid_len")
    if Q_rot is None:
        Q_rot = torch.empty(shp, dtype=dt, device=Q.device)
    if K_rot is None:
        K_rot = torch.empty(shp, dtype=dt, device=Q.device)
    _check_tensor(Q_rot, shp, dt, "Q_rot")
    _check_tensor(K_rot, shp, dt, "K_rot")
    if sel is None:
        sel = torch.empty((p.B, p.H, p.NB, p.topk), dtype=torch.int32, device=Q.device)
    _check_tensor(sel, (p.B, p.H, p.NB, p.topk), torch.int32, "sel")
    ws, nbytes = _workspace(p, WS_SELECT, ws, Q.device)
    cp = p.c()
    rc = lib().blossom_rope_select_blocks(ctypes.byref(cp), _ptr(Q), _ptr(K), _ptr(rope_cos), _ptr(rope_sin),
                                          _ptr(valid_len), _ptr(Q_rot), _ptr(K_rot), _ptr(sel), _ptr(ws), nbytes,
                                          _stream(stream))
    if rc:
        raise BlossomError(rc, "blossom_rope_select_blocks")
    return Q_rot, K_rot, sel


def select_blocks_cmp(p: Params, Q, Kcmp, valid_len, sel=None, ws=None, stream=None):
    """blossom_select_blocks_cmp: Kcmp [B,H,NB,d] holds the caller's compressed keys."""
    import torch
    _check_tensor(Q, (p.B, p.H, p.L, p.d), _torch_dtype(p), "Q")
    _check_tensor(Kcmp, (p.B, p.H, p.NB, p.d), _torch_dtype(p), "Kcmp")
    _check_tensor(valid_len, (p.B,), torch.int32, "valid_len")
    if sel is None:
        sel = torch.empty((p.B, p.H, p.NB, p.topk), dtype=torch.int32, device=Q.device)
    _check_tensor(sel, (p.B, p.H, p.NB, p.topk), torch.int32, "sel")
    ws, nbytes = _workspace(p, WS_SELECT, ws, Q.device)
    cp = p.c()
    rc = lib().blossom_select_blocks_cmp(ctypes.byref(cp), _ptr(Q), _ptr(Kcmp), _ptr(valid_len), _ptr(sel),
                                         _ptr(ws), nbytes, _stream(stream))
    if rc:
        raise BlossomError(rc, "blossom_select_blocks_cmp")
    return sel


@dataclass
class FwdOut:
    O: object
    o_lt: object = None
    o_st: object = None
    lse_lt: object = None
    lse_st: object = None


def attn_fwd(p: Params, Q, K, V, valid_len, sel, gate_w, gate_b=None, out: FwdOut | None = None,
             ws=None, stream=None) -> FwdOut:
    import torch
    shp = (p.B, p.H, p.L, p.d)
    dt = _torch_dtype(p)
    for t, nm in ((Q, "Q"), (K, "K"), (V, "V")):
        _check_tensor(t, shp, dt, nm)
    _check_tensor(valid_len, (p.B,), torch.int32, "valid_len")
    _check_tensor(sel, (p.B, p.H, p.NB, p.topk), torch.int32, "sel")
    _check_tensor(gate_w, (p.H, 2 * p.d), torch.float32, "gate_w")
    _check_tensor(gate_b, (p.H,), torch.float32, "gate_b")
    if out is None:
        out = FwdOut(torch.empty(shp, dtype=dt, device=Q.device))
        if p.save_for_bwd:
            out.o_lt = torch.empty(shp, dtype=torch.float32, device=Q.device)
            out.o_st = torch.empty(shp, dtype=torch.float32, device=Q.device)
            out.lse_lt = torch.empty(shp[:3], dtype=torch.float32, device=Q.device)
            out.lse_st = torch.empty(shp[:3], dtype=torch.float32, device=Q.device)
    _check_tensor(out.O, shp, dt, "O")
    _check_tensor(out.o_lt, shp, torch.float32, "o_lt")
    _check_tensor(out.o_st, shp, torch.float32, "o_st")
    _check_tensor(out.lse_lt, shp[:3], torch.float32, "lse_lt")
    _check_tensor(out.lse_st, shp[:3], torch.float32, "lse_st")
    ws, nbytes = _workspace(p, WS_FWD, ws, Q.device)
    cp = p.c()
    rc = lib().blossom_attn_fwd(ctypes.byref(cp), _ptr(Q), _ptr(K), _ptr(V), _ptr(valid_len), _ptr(sel),
                                _ptr(gate_w), _ptr(gate_b), _ptr(out.O), _ptr(out.o_lt), _ptr(out.o_st),
                                _ptr(out.lse_lt), _ptr(out.lse_st), _ptr(ws), nbytes, _stream(stream))
    if rc:
        raise BlossomError(rc, "blossom_attn_fwd")
    return out


@dataclass
class BwdOut:
    dQ: object
    dK: object
    dV: object
    d_gate_w: object
    d_gate_b: object


def attn_bwd(p: Params, Q, K, V, valid_len, sel, gate_w, gate_b, fwd: FwdOut, dO,
             out: BwdOut | None = None, ws=None, stream=None, stages: int = BWD_ALL, rope=None) -> BwdOut:
    """blossom_attn_bwd (or _stages); rope=(cos, sin) calls blossom_attn_bwd_rope instead."""
    import torch
    shp = (p.B, p.H, p.L, p.d)
    dt = _torch_dtype(p)
    for t, nm in ((Q, "Q"), (K, "K"), (V, "V"), (dO, "dO")):
        if t is None:
            raise ValueError(f"{nm} is required")
        _check_tensor(t, shp, dt, nm)
    for t, nm in ((fwd.o_lt, "o_lt"), (fwd.o_st, "o_st")):
        if t is None:
            raise ValueError(f"{nm} is required")
        _check_tensor(t, shp, torch.float32, nm)
    for t, nm in ((fwd.lse_lt, "lse_lt"), (fwd.lse_st, "lse_st")):
        if t is None:
            raise ValueError(f"{nm} is required")
        _check_tensor(t, shp[:3], torch.float32, nm)
    _check_tensor(valid_len, (p.B,), torch.int32, "valid_len")
    _check_tensor(sel, (p.B, p.H, p.NB, p.topk), torch.int32, "sel")
    _check_tensor(gate_w, (p.H, 2 * p.d), torch.float32, "gate_w")
    _check_tensor(gate_b, (p.H,), torch.float32, "gate_b")
    if out is None:
        out = BwdOut(torch.empty(shp, dtype=dt, device=Q.device), torch.empty(shp, dtype=dt, device=Q.device),
                     torch.empty(shp, dtype=dt, device=Q.device),
                     torch.empty((p.H, 2 * p.d), dtype=torch.float32, device=Q.device),
                     torch.empty((p.H,), dtype=torch.float32, device=Q.device))
    for t, nm in ((out.dQ, "dQ"), (out.dK, "dK"), (out.dV, "dV")):
        _check_tensor(t, shp, dt, nm)
    _check_tensor(out.d_gate_w, (p.H, 2 * p.d), torch.float32, "d_gate_w")
    _check_tensor(out.d_gate_b, (p.H,), torch.float32, "d_gate_b")
    ws, nbytes = _workspace(p, WS_BWD, ws, Q.device)
    cp = p.c()
    args = (ctypes.byref(cp), _ptr(Q), _ptr(K), _ptr(V), _ptr(valid_len), _ptr(sel), _ptr(gate_w), _ptr(gate_b),
            _ptr(fwd.o_lt), _ptr(fwd.o_st), _ptr(fwd.lse_lt), _ptr(fwd.lse_st), _ptr(dO), _ptr(out.dQ),
            _ptr(out.dK), _ptr(out.dV), _ptr(out.d_gate_w), _ptr(out.d_gate_b), _ptr(ws), nbytes, _stream(stream))
    if rope is not None:
        _check_tensor(rope[0], (p.L, p.d // 2), torch.float32, "rope_cos")
        _check_tensor(rope[1], (p.L, p.d // 2), torch.float32, "rope_sin")
        if stages != BWD_ALL:
            raise ValueError("blossom_attn_bwd_rope runs all passes")
        rc = lib().blossom_attn_bwd_rope(*args[:13], _ptr(rope[0]), _ptr(rope[1]), *args[13:])
    elif stages == BWD_ALL:
        rc = lib().blossom_attn_bwd(*args)
    else:
        rc = lib().blossom_attn_bwd_stages(*args, stages)
    if rc:
        raise BlossomError(rc, "blossom_attn_bwd")
    return out


def dense_causal_fwd(p: Params, Q, K, V, valid_len, O=None, lse=None, ws=None, stream=None):
    import torch
    shp = (p.B, p.H, p.L, p.d)
    dt = _torch_dtype(p)
    for t, nm in ((Q, "Q"), (K, "K"), (V, "V")):
        _check_tensor(t, shp, dt, nm)
    _check_tensor(valid_len, (p.B,), torch.int32, "valid_len")
    if O is None:
        O = torch.empty(shp, dtype=dt, device=Q.device)
    _check_tensor(O, shp, dt, "O")
    _check_tensor(lse, shp[:3], torch.float32, "lse")
    ws, nbytes = _workspace(p, WS_DENSE, ws, Q.device)
    cp = p.c()
    rc = lib().blossom_dense_causal_fwd(ctypes.byref(cp), _ptr(Q), _ptr(K), _ptr(V), _ptr(valid_len),
                                        _ptr(O), _ptr(lse), _ptr(ws), nbytes, _stream(stream))
    if rc:
        raise BlossomError(rc, "blossom_dense_causal_fwd")
    return O, lse


def probe_bytes(which: int) -> int:
    return int(lib().blossom_probe_bytes(which))


def probe(kind: int, K, V, sink, iters: int, stream=None):
    """blossom_probe: one launch of the stripped tile loop (the caller times it)."""
    rc = lib().blossom_probe(int(kind), _ptr(K), _ptr(V), _ptr(sink), int(iters), _stream(stream))
    if rc:
        raise BlossomError(rc, "blossom_probe")


def select_positions_workspace_bytes(p: Params, kv_groups: int, cmp_block: int, cmp_stride: int) -> int:
    cp = p.c()
    return int(lib().blossom_select_positions_workspace_bytes(ctypes.byref(cp), kv_groups, cmp_block, cmp_stride))


def select_positions(p: Params, kv_groups: int, cmp_block: int, cmp_stride: int, Q, K, valid_len, score_scale: float = 0.0,
                     sel_pos=None, ws=None, stream=None):
    """blossom_select_positions: the printed selection rule, one row per position and key/value group.
    p.block is the selection block size, p.topk is k.  Returns sel_pos int32 [B,G,L,topk]."""
    import torch
    dt = _torch_dtype(p)
    _check_tensor(Q, (p.B, p.H, p.L, p.d), dt, "Q")
    _check_tensor(K, (p.B, kv_groups, p.L, p.d), dt, "K")
    _check_tensor(valid_len, (p.B,), torch.int32, "valid_len")
    if sel_pos is None:
        sel_pos = torch.empty((p.B, kv_groups, p.L, p.topk), dtype=torch.int32, device=Q.device)
    _check_tensor(sel_pos, (p.B, kv_groups, p.L, p.topk), torch.int32, "sel_pos")
    cp = p.c()
    need = select_positions_workspace_bytes(p, kv_groups, cmp_block, cmp_stride)
    if ws is None:
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=Q.device)
    rc = lib().blossom_select_positions(ctypes.byref(cp), kv_groups, cmp_block, cmp_stride, float(score_scale), _ptr(Q),
                                        _ptr(K), _ptr(valid_len), _ptr(sel_pos), _ptr(ws), ws.numel(), _stream(stream))
    if rc:
        raise BlossomError(rc, "blossom_select_positions")
    return sel_pos


def attn_fwd_positions(p: Params, kv_groups: int, Q, K, V, valid_len, sel_pos, gate_w, gate_b=None, out: FwdOut | None = None,
                       want_branches: bool = False, stream=None) -> FwdOut:
    """blossom_attn_fwd_positions: forward under one selection row per query position and key/value group
    (K, V [B,G,L,d], sel_pos [B,G,L,topk]).  `want_branches` also returns o_lt, o_st, lse_lt, lse_st."""
    import torch
    shp = (p.B, p.H, p.L, p.d)
    dt = _torch_dtype(p)
    _check_tensor(Q, shp, dt, "Q")
    for t, nm in ((K, "K"), (V, "V")):
        _check_tensor(t, (p.B, kv_groups, p.L, p.d), dt, nm)
    _check_tensor(valid_len, (p.B,), torch.int32, "valid_len")
    _check_tensor(sel_pos, (p.B, kv_groups, p.L, p.topk), torch.int32, "sel_pos")
    _check_tensor(gate_w, (p.H, 2 * p.d), torch.float32, "gate_w")
    _check_tensor(gate_b, (p.H,), torch.float32, "gate_b")
    if out is None:
        out = FwdOut(torch.empty(shp, dtype=dt, device=Q.device))
        if want_branches:
            out.o_lt = torch.empty(shp, dtype=torch.float32, device=Q.device)
            out.o_st = torch.empty(shp, dtype=torch.float32, device=Q.device)
            out.lse_lt = torch.empty(shp[:3], dtype=torch.float32, device=Q.device)
            out.lse_st = torch.empty(shp[:3], dtype=torch.float32, device=Q.device)
    cp = p.c()
    rc = lib().blossom_attn_fwd_positions(ctypes.byref(cp), kv_groups, _ptr(Q), _ptr(K), _ptr(V), _ptr(valid_len), _ptr(sel_pos),
                                          _ptr(gate_w), _ptr(gate_b), _ptr(out.O), _ptr(out.o_lt), _ptr(out.o_st),
                                          _ptr(out.lse_lt), _ptr(out.lse_st), _stream(stream))
    if rc:
        raise BlossomError(rc, "blossom_attn_fwd_positions")
    return out


def attn_bwd_positions(p: Params, kv_groups: int, Q, K, V, valid_len, sel_pos, gate_w, gate_b, fwd: FwdOut, dO,
                       out: BwdOut | None = None, ws=None, stream=None) -> BwdOut:
    """blossom_attn_bwd_positions: backward of attn_fwd_positions (dQ [B,H,L,d]; dK, dV [B,G,L,d]: the
    gradients of the query heads of a group added up)."""
    import torch
    shp = (p.B, p.H, p.L, p.d)
    kv_shp = (p.B, kv_groups, p.L, p.d)
    dt = _torch_dtype(p)
    for t, nm, sh in ((Q, "Q", shp), (K, "K", kv_shp), (V, "V", kv_shp), (dO, "dO", shp)):
        if t is None:
            raise ValueError(f"{nm} is required")
        _check_tensor(t, sh, dt, nm)
    for t, nm in ((fwd.o_lt, "o_lt"), (fwd.o_st, "o_st")):
        if t is None:
            raise ValueError(f"{nm} is required")
        _check_tensor(t, shp, torch.float32, nm)
    for t, nm in ((fwd.lse_lt, "lse_lt"), (fwd.lse_st, "lse_st")):
        if t is None:
            raise ValueError(f"{nm} is required")
        _check_tensor(t, shp[:3], torch.float32, nm)
    _check_tensor(valid_len, (p.B,), torch.int32, "valid_len")
    _check_tensor(sel_pos, (p.B, kv_groups, p.L, p.topk), torch.int32, "sel_pos")
    _check_tensor(gate_w, (p.H, 2 * p.d), torch.float32, "gate_w")
    _check_tensor(gate_b, (p.H,), torch.float32, "gate_b")
    if out is None:
        out = BwdOut(torch.empty(shp, dtype=dt, device=Q.device), torch.empty(kv_shp, dtype=dt, device=Q.device),
                     torch.empty(kv_shp, dtype=dt, device=Q.device),
                     torch.empty((p.H, 2 * p.d), dtype=torch.float32, device=Q.device),
                     torch.empty((p.H,), dtype=torch.float32, device=Q.device))
    _check_tensor(out.dQ, shp, dt, "dQ")
    _check_tensor(out.dK, kv_shp, dt, "dK")
    _check_tensor(out.dV, kv_shp, dt, "dV")
    _check_tensor(out.d_gate_w, (p.H, 2 * p.d), torch.float32, "d_gate_w")
    _check_tensor(out.d_gate_b, (p.H,), torch.float32, "d_gate_b")
    ws, nbytes = _workspace(p, WS_BWD, ws, Q.device)
    cp = p.c()
    rc = lib().blossom_attn_bwd_positions(ctypes.byref(cp), kv_groups, _ptr(Q), _ptr(K), _ptr(V), _ptr(valid_len),
                                          _ptr(sel_pos), _ptr(gate_w), _ptr(gate_b), _ptr(fwd.o_lt), _ptr(fwd.o_st),
                                          _ptr(fwd.lse_lt), _ptr(fwd.lse_st), _ptr(dO), _ptr(out.dQ), _ptr(out.dK),
                                          _ptr(out.dV), _ptr(out.d_gate_w), _ptr(out.d_gate_b), _ptr(ws), nbytes,
                                          _stream(stream))
    if rc:
        raise BlossomError(rc, "blossom_attn_bwd_positions")
    return out


def out_proj_ln(p: Params, d_model: int, O, W_O_t, H_prev, ln_gamma, ln_beta, ln_eps: float, bias=None, S=None,
                want_stats: bool = False, stream=None):
    """blossom_out_proj_ln: S = LayerNorm(H_prev + Concat_h(O[:, h]) W^O (+ bias)); W_O_t is [d_model, H*d].
    Returns S, or (S, mean, rstd) with want_stats."""
    import torch
    dt = _torch_dtype(p)
    _check_tensor(O, (p.B, p.H, p.L, p.d), dt, "O")
    _check_tensor(W_O_t, (d_model, p.H * p.d), dt, "W_O_t")
    _check_tensor(H_prev, (p.B, p.L, d_model), dt, "H_prev")
    _check_tensor(ln_gamma, (d_model,), torch.float32, "ln_gamma")
    _check_tensor(ln_beta, (d_model,), torch.float32, "ln_beta")
    _check_tensor(bias, (d_model,), torch.float32, "bias")
    if S is None:
        S = torch.empty((p.B, p.L, d_model), dtype=dt, device=O.device)
    _check_tensor(S, (p.B, p.L, d_model), dt, "S")
    mean = rstd = None
    if want_stats:
        mean = torch.empty((p.B, p.L), dtype=torch.float32, device=O.device)
        rstd = torch.empty((p.B, p.L), dtype=torch.float32, device=O.device)
    cp = p.c()
    rc = lib().blossom_out_proj_ln(ctypes.byref(cp), d_model, _ptr(O), _ptr(W_O_t), _ptr(bias), _ptr(H_prev), _ptr(ln_gamma),
                                   _ptr(ln_beta), float(ln_eps), _ptr(S), _ptr(mean), _ptr(rstd), _stream(stream))
    if rc:
        raise BlossomError(rc, "blossom_out_proj_ln")
    return (S, mean, rstd) if want_stats else S
