"""ctypes binding of liba2d.so: the same four calls as include/a2d.h, on torch tensors.

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  torch supplies device memory and the current stream.  If the library
has not been built (python -m paper_2503_15758_amd.build) every call raises.
"""
import ctypes
import math
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "liba2d.so")

A2D_F32, A2D_BF16 = 0, 1
OP_PARTIAL_FWD, OP_FIX, OP_PARTIAL_BWD, OP_FIX_BWD, OP_PARTIAL_BWD_DS, OP_PARTIAL_BWD_SPLIT = 0, 1, 2, 3, 4, 5
MAX_PARTS = 32

EXPORTS = ("a2d_workspace_bytes", "a2d_partial_fwd", "a2d_fix", "a2d_attnfix", "a2d_partial_bwd", "a2d_fix_bwd",
           "a2d_partial_bwd_static",
           "a2d_partial_fwd_seg", "a2d_partial_bwd_seg", "a2d_partial_fwd_acc", "a2d_partial_bwd_acc",
           "a2d_partial_fwd_norm", "a2d_fix_norm", "a2d_partial_fwd_gqa", "a2d_partial_bwd_gqa",
           "a2d_fix_strided", "a2d_fix_bwd_strided", "a2d_fix_norm_strided",
           "a2d_mfma_ceiling_scratch_bytes", "a2d_mfma_ceiling", "a2d_forward_mix_ceiling", "a2d_backward_mix_ceiling", "a2d_lds_read_ceiling", "a2d_debug_force_generic",
           "a2d_debug_trace", "a2d_debug_trace_count", "a2d_copy_probe",
           "a2d_status_str", "a2d_last_error", "a2d_version")


class Layout(ctypes.Structure):
    """a2d_layout: element strides of a [heads][rows][H] tensor; (0, 0) = plain."""
    _fields_ = [("head", ctypes.c_int64), ("row", ctypes.c_int64)]


class TileDesc(ctypes.Structure):
    _fields_ = [("heads", ctypes.c_int32), ("nq", ctypes.c_int32), ("nkv", ctypes.c_int32),
                ("hdim", ctypes.c_int32), ("q_off", ctypes.c_int64), ("kv_off", ctypes.c_int64),
                ("causal", ctypes.c_int32), ("scale", ctypes.c_float), ("dtype", ctypes.c_int32),
                ("flags", ctypes.c_int32), ("lq", Layout), ("lk", Layout), ("lv", Layout), ("lo", Layout),
                ("ldo", Layout)]


class KvSegment(ctypes.Structure):
    _fields_ = [("kv_off", ctypes.c_int64), ("rows", ctypes.c_int32), ("pad", ctypes.c_int32)]


MAX_SEGMENTS = 32
TILE_ACCUMULATE, TILE_NORMALISED, TILE_SPLIT_GROUPS = 1, 2, 4
DESC_KEEP_DS = 1


class A2DError(RuntimeError):
    def __init__(self, status, detail):
        super().__init__("a2d status %d: %s" % (status, detail))
        self.status = status


_lib = None


def lib():
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("liba2d.so is missing at %s: build it with "
                               "`python -m paper_2503_15758_amd.build`" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, fp = ctypes.c_void_p, ctypes.c_void_p
        L.a2d_workspace_bytes.restype = ctypes.c_size_t
        L.a2d_workspace_bytes.argtypes = [ctypes.POINTER(TileDesc), ctypes.c_int, ctypes.c_int]
        L.a2d_partial_fwd.restype = ctypes.c_int
        L.a2d_partial_fwd.argtypes = [ctypes.POINTER(TileDesc), vp, vp, vp, fp, fp, fp, vp,
                                      ctypes.c_size_t, vp]
        L.a2d_partial_fwd_seg.restype = ctypes.c_int
        L.a2d_partial_fwd_seg.argtypes = [ctypes.POINTER(TileDesc), ctypes.c_int, ctypes.POINTER(KvSegment),
                                          vp, vp, vp, fp, fp, fp, vp, ctypes.c_size_t, vp]
        L.a2d_partial_bwd_seg.restype = ctypes.c_int
        L.a2d_partial_bwd_seg.argtypes = [ctypes.POINTER(TileDesc), ctypes.c_int, ctypes.POINTER(KvSegment),
                                          vp, vp, vp, vp, vp, fp, fp, fp, fp, vp, ctypes.c_size_t, vp]
        L.a2d_partial_fwd_acc.restype = ctypes.c_int
        L.a2d_partial_fwd_acc.argtypes = L.a2d_partial_fwd_seg.argtypes
        L.a2d_partial_bwd_acc.restype = ctypes.c_int
        L.a2d_partial_bwd_acc.argtypes = L.a2d_partial_bwd_seg.argtypes
        L.a2d_partial_fwd_norm.restype = ctypes.c_int
        L.a2d_partial_fwd_norm.argtypes = [ctypes.POINTER(TileDesc), ctypes.c_int, ctypes.POINTER(KvSegment),
                                           vp, vp, vp, vp, fp, vp, ctypes.c_size_t, vp]
        # (every argument is typed: an untyped Python int travels as a 32-bit C int, and one that lands
        # on the stack - these calls have more arguments than registers - reaches a size_t parameter
        # with undefined upper bits)
        L.a2d_partial_fwd_gqa.restype = ctypes.c_int
        L.a2d_partial_fwd_gqa.argtypes = [ctypes.POINTER(TileDesc), ctypes.c_int32, ctypes.c_int,
                                          ctypes.POINTER(KvSegment), ctypes.c_int, vp, vp, vp, vp, fp, fp, vp,
                                          ctypes.c_size_t, vp]
        L.a2d_partial_bwd_gqa.restype = ctypes.c_int
        L.a2d_partial_bwd_gqa.argtypes = [ctypes.POINTER(TileDesc), ctypes.c_int32, ctypes.c_int,
                                          ctypes.POINTER(KvSegment), ctypes.c_int, vp, vp, vp, vp, vp, fp,
                                          fp, fp, fp, vp, ctypes.c_size_t, vp]
        L.a2d_fix_norm.restype = ctypes.c_int
        L.a2d_fix_norm.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                   ctypes.POINTER(vp), ctypes.POINTER(vp), vp, fp, vp]
        L.a2d_fix.restype = ctypes.c_int
        L.a2d_fix.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                              ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), vp, fp, vp]
        L.a2d_attnfix.restype = ctypes.c_int
        L.a2d_attnfix.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int32,
                                  ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), fp, fp, fp, vp]
        L.a2d_partial_bwd.restype = ctypes.c_int
        L.a2d_partial_bwd.argtypes = [ctypes.POINTER(TileDesc), vp, vp, vp, vp, vp, fp, fp, fp, fp,
                                      vp, ctypes.c_size_t, vp]
        L.a2d_partial_bwd_static.restype = ctypes.c_int
        L.a2d_partial_bwd_static.argtypes = [ctypes.POINTER(TileDesc), vp, vp, vp, vp, vp, fp, fp, fp, fp, vp]
        L.a2d_fix_bwd.restype = ctypes.c_int
        L.a2d_fix_bwd.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int32, ctypes.POINTER(vp),
                                  vp, vp]
        L.a2d_fix_strided.restype = ctypes.c_int
        L.a2d_fix_strided.argtypes = [ctypes.c_int, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                      ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), vp,
                                      ctypes.POINTER(Layout), vp, vp]
        L.a2d_fix_norm_strided.restype = ctypes.c_int
        L.a2d_fix_norm_strided.argtypes = [ctypes.c_int, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                           ctypes.c_int32, ctypes.POINTER(vp), ctypes.POINTER(vp), vp,
                                           ctypes.POINTER(Layout), vp, vp]
        L.a2d_fix_bwd_strided.restype = ctypes.c_int
        L.a2d_fix_bwd_strided.argtypes = [ctypes.c_int, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                          ctypes.POINTER(vp), vp, ctypes.POINTER(Layout), vp]
        L.a2d_mfma_ceiling_scratch_bytes.restype = ctypes.c_size_t
        L.a2d_mfma_ceiling_scratch_bytes.argtypes = []
        L.a2d_mfma_ceiling.restype = ctypes.c_int
        L.a2d_mfma_ceiling.argtypes = [ctypes.c_int, ctypes.c_int, vp, ctypes.c_size_t,
                                       ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        L.a2d_backward_mix_ceiling.restype = ctypes.c_int
        L.a2d_backward_mix_ceiling.argtypes = [ctypes.c_int, ctypes.c_int, vp, ctypes.c_size_t,
                                               ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        L.a2d_lds_read_ceiling.restype = ctypes.c_int
        L.a2d_lds_read_ceiling.argtypes = [ctypes.c_int, ctypes.c_int, vp, ctypes.c_size_t,
                                           ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        L.a2d_forward_mix_ceiling.restype = ctypes.c_int
        L.a2d_forward_mix_ceiling.argtypes = [ctypes.c_int, vp, ctypes.c_size_t,
                                              ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        L.a2d_debug_force_generic.restype = None
        L.a2d_debug_force_generic.argtypes = [ctypes.c_int]
        L.a2d_debug_trace.restype = None
        L.a2d_debug_trace.argtypes = [ctypes.POINTER(vp), ctypes.c_int]
        L.a2d_debug_trace_count.restype = ctypes.c_int
        L.a2d_debug_trace_count.argtypes = []
        L.a2d_copy_probe.restype = ctypes.c_int
        L.a2d_copy_probe.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.a2d_status_str.restype = ctypes.c_char_p
        L.a2d_status_str.argtypes = [ctypes.c_int]
        L.a2d_last_error.restype = ctypes.c_char_p
        L.a2d_last_error.argtypes = []
        L.a2d_version.restype = ctypes.c_char_p
        L.a2d_version.argtypes = []
        _lib = L
    return _lib


def _check(status):
    if status != 0:
        raise A2DError(status, lib().a2d_last_error().decode())


def _dtype_code(t):
    if t == torch.float32:
        return A2D_F32
    if t == torch.bfloat16:
        return A2D_BF16
    raise A2DError(-2, "dtype %s not supported" % t)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def _ptr_array(ts):
    return (ctypes.c_void_p * len(ts))(*[t.data_ptr() for t in ts])


def _dev3(t, name):
    """The tile calls' inputs: [heads][rows][H] device tensors (or views) whose rows of H elements are
    contiguous; the head and row strides travel in the descriptor."""
    if not (t.is_cuda and t.dim() == 3 and (t.stride(2) == 1 or t.shape[2] == 1)):
        raise A2DError(-1, "%s must be a [heads][rows][H] device tensor with contiguous rows" % name)


def _plain(ts, name):
    """What the library writes is always in the plain layout."""
    for t in ts:
        if not (t.is_cuda and t.is_contiguous()):
            raise A2DError(-1, "%s must be contiguous device tensors" % name)


def _layout(t):
    """a2d_layout of a tensor or view accepted by _dev3 ((0, 0) for the plain layout)."""
    if t is None or t.is_contiguous():
        return Layout(0, 0)
    heads, rows, H = t.shape
    row = t.stride(1) if rows > 1 else H             # a stride over a dimension of extent 1 is arbitrary
    head = t.stride(0) if heads > 1 else rows * row
    return Layout(int(head), int(row))


def tile_desc(Q, K, q_off, kv_off, causal, scale, V=None, O=None, dO=None, flags=0):
    """Descriptor of the tile; the strides of Q, K (and V, O, dO when given) are taken from the tensors."""
    heads, nq, H = Q.shape
    return TileDesc(heads, nq, K.shape[1], H, int(q_off), int(kv_off), int(bool(causal)),
                    float(scale if scale is not None else 1.0 / math.sqrt(H)), _dtype_code(Q.dtype), int(flags),
                    _layout(Q), _layout(K), _layout(V if V is not None else K), _layout(O), _layout(dO))


def workspace_bytes(desc, op, k=0):
    return int(lib().a2d_workspace_bytes(ctypes.byref(desc), op, k))


def _segments(segments):
    arr = (KvSegment * len(segments))()
    for i, (off, rows) in enumerate(segments):
        arr[i].kv_off, arr[i].rows, arr[i].pad = int(off), int(rows), 0
    return arr


def partial_fwd(Q, K, V, q_off=0, kv_off=0, causal=False, scale=None, out=None, segments=None,
                accumulate=False):
    """a2d_partial_fwd. Returns (O_part fp32 [heads][nq][H], m, l fp32 [heads][nq])."""
    for t, n in ((Q, "Q"), (K, "K"), (V, "V")):
        _dev3(t, n)
    if K.shape != V.shape or K.shape[2] != Q.shape[2] or K.dtype != Q.dtype or V.dtype != Q.dtype:
        raise A2DError(-1, "Q, K, V shapes / dtypes do not match")
    d = tile_desc(Q, K, q_off, kv_off, causal, scale, V)
    if out is None:
        O_part = torch.empty(Q.shape, dtype=torch.float32, device=Q.device)
        m = torch.empty(Q.shape[:2], dtype=torch.float32, device=Q.device)
        l = torch.empty(Q.shape[:2], dtype=torch.float32, device=Q.device)
    else:
        O_part, m, l = out
        _plain(out, "out=(O_part, m, l)")
    if accumulate and out is None:
        raise A2DError(-1, "accumulate needs out=(O_part, m, l)")
    if K.shape[0] != Q.shape[0]:   # grouped queries: K, V hold fewer heads than Q
        n = len(segments) if segments is not None else 0
        _check(lib().a2d_partial_fwd_gqa(ctypes.byref(d), int(K.shape[0]), n, _segments(segments) if n else None,
                                         TILE_ACCUMULATE if accumulate else 0, _ptr(Q), _ptr(K), _ptr(V),
                                         _ptr(O_part), _ptr(m), _ptr(l), None, 0, _stream()))
        return O_part, m, l
    if accumulate:                 # out holds a partial triple of the same query block: merged in place
        if out is None:
            raise A2DError(-1, "accumulate needs out=(O_part, m, l)")
        n = len(segments) if segments is not None else 0
        _check(lib().a2d_partial_fwd_acc(ctypes.byref(d), n, _segments(segments) if n else None, _ptr(Q),
                                         _ptr(K), _ptr(V), _ptr(O_part), _ptr(m), _ptr(l), None, 0,
                                         _stream()))
        return O_part, m, l
    if segments is not None:       # gathered tile: list of (kv_off, rows) sub-blocks, kv_off unused
        _check(lib().a2d_partial_fwd_seg(ctypes.byref(d), len(segments), _segments(segments), _ptr(Q),
                                         _ptr(K), _ptr(V), _ptr(O_part), _ptr(m), _ptr(l), None, 0,
                                         _stream()))
        return O_part, m, l
    _check(lib().a2d_partial_fwd(ctypes.byref(d), _ptr(Q), _ptr(K), _ptr(V), _ptr(O_part), _ptr(m),
                                 _ptr(l), None, 0, _stream()))
    return O_part, m, l


def partial_fwd_norm(Q, K, V, q_off=0, kv_off=0, causal=False, scale=None, out=None, segments=None):
    """a2d_partial_fwd_norm: the normalised partial (O' in Q's dtype, lse' fp32) of a plain or gathered tile."""
    for t, n in ((Q, "Q"), (K, "K"), (V, "V")):
        _dev3(t, n)
    if K.shape != V.shape or K.shape[2] != Q.shape[2] or K.dtype != Q.dtype or V.dtype != Q.dtype:
        raise A2DError(-1, "Q, K, V shapes / dtypes do not match")
    d = tile_desc(Q, K, q_off, kv_off, causal, scale, V)
    if out is None:
        O_norm = torch.empty(Q.shape, dtype=Q.dtype, device=Q.device)
        lse = torch.empty(Q.shape[:2], dtype=torch.float32, device=Q.device)
    else:
        O_norm, lse = out
        _plain(out, "out=(O_norm, lse)")
    n = len(segments) if segments is not None else 0
    if K.shape[0] != Q.shape[0]:   # grouped queries
        _check(lib().a2d_partial_fwd_gqa(ctypes.byref(d), int(K.shape[0]), n, _segments(segments) if n else None,
                                         TILE_NORMALISED, _ptr(Q), _ptr(K), _ptr(V), _ptr(O_norm), _ptr(lse),
                                         None, None, 0, _stream()))
        return O_norm, lse
    _check(lib().a2d_partial_fwd_norm(ctypes.byref(d), n, _segments(segments) if n else None, _ptr(Q),
                                      _ptr(K), _ptr(V), _ptr(O_norm), _ptr(lse), None, 0, _stream()))
    return O_norm, lse


def fix_norm(O_norms, lses, out_dtype=torch.bfloat16, out=None):
    """a2d_fix_norm over k normalised partials. Returns (O in out_dtype, lse fp32)."""
    k = len(O_norms)
    if k < 1 or len(lses) != k:
        raise A2DError(-1, "need k >= 1 normalised partials")
    shape = O_norms[0].shape
    rows = 1
    for s in shape[:-1]:
        rows *= s
    if out is None:
        O = torch.empty(shape, dtype=out_dtype, device=O_norms[0].device)
        lse = torch.empty(shape[:-1], dtype=torch.float32, device=O_norms[0].device)
    else:
        O, lse = out
    _plain(list(O_norms) + list(lses) + [lse], "the partials and lse")
    if not O.is_contiguous():      # a [heads][nq][H] view: written in place through its strides
        _dev3(O, "O")
        lo = _layout(O)
        _check(lib().a2d_fix_norm_strided(k, O.shape[0], O.shape[1], shape[-1], _dtype_code(O_norms[0].dtype),
                                          _dtype_code(O.dtype), _ptr_array(O_norms), _ptr_array(lses), _ptr(O),
                                          ctypes.byref(lo), _ptr(lse), _stream()))
        return O, lse
    _check(lib().a2d_fix_norm(k, rows, shape[-1], _dtype_code(O_norms[0].dtype), _dtype_code(O.dtype),
                              _ptr_array(O_norms), _ptr_array(lses), _ptr(O), _ptr(lse), _stream()))
    return O, lse


def fix(O_parts, ms, ls, out_dtype=torch.bfloat16, out=None):
    """a2d_fix over k partial triples. Returns (O [heads][nq][H] in out_dtype, lse fp32)."""
    k = len(O_parts)
    if k < 1 or len(ms) != k or len(ls) != k:
        raise A2DError(-1, "need k >= 1 partial triples")
    shape = O_parts[0].shape
    rows = 1
    for s in shape[:-1]:
        rows *= s
    if out is None:
        O = torch.empty(shape, dtype=out_dtype, device=O_parts[0].device)
        lse = torch.empty(shape[:-1], dtype=torch.float32, device=O_parts[0].device)
    else:
        O, lse = out
    _plain(list(O_parts) + list(ms) + list(ls) + [lse], "the partials and lse")
    if not O.is_contiguous():      # a [heads][nq][H] view: written in place through its strides
        _dev3(O, "O")
        lo = _layout(O)
        _check(lib().a2d_fix_strided(k, O.shape[0], O.shape[1], shape[-1], _dtype_code(O.dtype),
                                     _ptr_array(O_parts), _ptr_array(ms), _ptr_array(ls), _ptr(O),
                                     ctypes.byref(lo), _ptr(lse), _stream()))
        return O, lse
    _check(lib().a2d_fix(k, rows, shape[-1], _dtype_code(O.dtype), _ptr_array(O_parts),
                         _ptr_array(ms), _ptr_array(ls), _ptr(O), _ptr(lse), _stream()))
    return O, lse


def attnfix(O_parts, ms, ls, out=None):
    """a2d_attnfix: AttnFix alone over k partial triples. Returns one partial (N, m, l), fp32, not normalised."""
    k = len(O_parts)
    if k < 1 or len(ms) != k or len(ls) != k:
        raise A2DError(-1, "need k >= 1 partial triples")
    shape = O_parts[0].shape
    rows = 1
    for s in shape[:-1]:
        rows *= s
    if out is None:
        N = torch.empty(shape, dtype=torch.float32, device=O_parts[0].device)
        m = torch.empty(shape[:-1], dtype=torch.float32, device=O_parts[0].device)
        l = torch.empty(shape[:-1], dtype=torch.float32, device=O_parts[0].device)
    else:
        N, m, l = out
    _plain(list(O_parts) + list(ms) + list(ls) + [N, m, l], "the partials")
    _check(lib().a2d_attnfix(k, rows, shape[-1], _ptr_array(O_parts), _ptr_array(ms), _ptr_array(ls),
                             _ptr(N), _ptr(m), _ptr(l), _stream()))
    return N, m, l


def partial_bwd(Q, K, V, O, dO, lse, q_off=0, kv_off=0, causal=False, scale=None, out=None,
                workspace=None, segments=None, accumulate=False, ds_handover=False, split_groups=False):
    """a2d_partial_bwd. Returns (dQ_part, dK_part, dV_part), all fp32.  ds_handover=True sets
    A2D_DESC_KEEP_DS in the descriptor: the library keeps dS for the dQ contraction instead of
    recomputing it, and the workspace (allocated here when none is given) must then hold
    a2d_workspace_bytes(A2D_OP_PARTIAL_BWD_DS) bytes.  split_groups=True
    (grouped heads only) passes A2D_TILE_SPLIT_GROUPS: a key block may go to several workgroups,
    each summing over a share of the group's query heads (workspace of A2D_OP_PARTIAL_BWD_SPLIT
    size, which includes the dS area)."""
    for t, n in ((Q, "Q"), (K, "K"), (V, "V"), (O, "O"), (dO, "dO")):
        _dev3(t, n)
    if O.shape != Q.shape or dO.shape != Q.shape or O.dtype != Q.dtype or dO.dtype != Q.dtype or \
            lse.shape != Q.shape[:2] or lse.dtype != torch.float32 or K.shape != V.shape or \
            not lse.is_contiguous():
        raise A2DError(-1, "O, dO, lse do not match Q (lse: plain fp32 [heads][nq])")
    d = tile_desc(Q, K, q_off, kv_off, causal, scale, V, O, dO, flags=DESC_KEEP_DS if ds_handover else 0)
    need = workspace_bytes(d, OP_PARTIAL_BWD_DS if ds_handover else OP_PARTIAL_BWD)
    split_groups = bool(split_groups) and K.shape[0] != Q.shape[0]
    if split_groups:
        need = workspace_bytes(d, OP_PARTIAL_BWD_SPLIT, int(K.shape[0]))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
    if out is None:
        dQ = torch.empty(Q.shape, dtype=torch.float32, device=Q.device)
        dK = torch.empty(K.shape, dtype=torch.float32, device=Q.device)
        dV = torch.empty(K.shape, dtype=torch.float32, device=Q.device)
    else:
        dQ, dK, dV = out
        _plain(out, "out=(dQ_part, dK_part, dV_part)")
    if accumulate and out is None:
        raise A2DError(-1, "accumulate needs out=(dQ_part, dK_part, dV_part)")
    if K.shape[0] != Q.shape[0]:   # grouped queries: dK_part, dV_part have K's heads
        n = len(segments) if segments is not None else 0
        _check(lib().a2d_partial_bwd_gqa(ctypes.byref(d), int(K.shape[0]), n, _segments(segments) if n else None,
                                         (TILE_ACCUMULATE if accumulate else 0) |
                                         (TILE_SPLIT_GROUPS if split_groups else 0), _ptr(Q), _ptr(K), _ptr(V),
                                         _ptr(O), _ptr(dO), _ptr(lse), _ptr(dQ), _ptr(dK), _ptr(dV),
                                         _ptr(workspace), workspace.numel() * workspace.element_size(),
                                         _stream()))
        return dQ, dK, dV
    if accumulate:                 # out[0] (dQ_part) is added to
        n = len(segments) if segments is not None else 0
        _check(lib().a2d_partial_bwd_acc(ctypes.byref(d), n, _segments(segments) if n else None, _ptr(Q),
                                         _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(lse), _ptr(dQ),
                                         _ptr(dK), _ptr(dV), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream()))
        return dQ, dK, dV
    if segments is not None:
        _check(lib().a2d_partial_bwd_seg(ctypes.byref(d), len(segments), _segments(segments), _ptr(Q),
                                         _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(lse), _ptr(dQ),
                                         _ptr(dK), _ptr(dV), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream()))
        return dQ, dK, dV
    _check(lib().a2d_partial_bwd(ctypes.byref(d), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO),
                                 _ptr(lse), _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream()))
    return dQ, dK, dV


STATIC_MAX_ROWS = 1 << 20


def partial_bwd_static(Q, K, V, O, dO, lse, q_off=0, kv_off=0, causal=False, scale=None, out=None):
    """a2d_partial_bwd_static: a2d_partial_bwd without a workspace argument (the library's own static
    scratch holds delta; heads * nq <= STATIC_MAX_ROWS).  `out` = (dQ_part, dK_part, dV_part) fp32;
    with out given this function allocates nothing either."""
    for t, n in ((Q, "Q"), (K, "K"), (V, "V"), (O, "O"), (dO, "dO")):
        _dev3(t, n)
    if O.shape != Q.shape or dO.shape != Q.shape or O.dtype != Q.dtype or dO.dtype != Q.dtype or \
            lse.shape != Q.shape[:2] or lse.dtype != torch.float32 or K.shape != V.shape or \
            K.shape[0] != Q.shape[0] or not lse.is_contiguous():
        raise A2DError(-1, "O, dO, lse do not match Q (lse: plain fp32 [heads][nq]); K, V need Q's head count")
    d = tile_desc(Q, K, q_off, kv_off, causal, scale, V, O, dO)
    if out is None:
        out = (torch.empty(Q.shape, dtype=torch.float32, device=Q.device),
               torch.empty(K.shape, dtype=torch.float32, device=Q.device),
               torch.empty(K.shape, dtype=torch.float32, device=Q.device))
    _plain(out, "out=(dQ_part, dK_part, dV_part)")
    dQ, dK, dV = out
    _check(lib().a2d_partial_bwd_static(ctypes.byref(d), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(lse),
                                        _ptr(dQ), _ptr(dK), _ptr(dV), _stream()))
    return dQ, dK, dV


def fix_bwd(parts, out_dtype=torch.bfloat16, out=None):
    """a2d_fix_bwd: sum of k fp32 partials, rounded once to out_dtype."""
    k = len(parts)
    if k < 1:
        raise A2DError(-1, "need k >= 1 partials")
    if out is None:
        out = torch.empty(parts[0].shape, dtype=out_dtype, device=parts[0].device)
    _plain(parts, "the partials")
    if not out.is_contiguous():    # a [heads][rows][H] view: written in place through its strides
        _dev3(out, "out")
        lo = _layout(out)
        _check(lib().a2d_fix_bwd_strided(k, out.shape[0], out.shape[1], out.shape[2], _dtype_code(out.dtype),
                                         _ptr_array(parts), _ptr(out), ctypes.byref(lo), _stream()))
        return out
    _check(lib().a2d_fix_bwd(k, parts[0].numel(), _dtype_code(out.dtype), _ptr_array(parts), _ptr(out),
                             _stream()))
    return out


def mfma_ceiling(iters=20000, random_data=True):
    """Diagnostic (a2d_mfma_ceiling): (dense bf16 TFLOP/s of the MFMA units alone, shader MHz)."""
    n = int(lib().a2d_mfma_ceiling_scratch_bytes())
    scratch = torch.empty(max(n, 16), dtype=torch.uint8, device="cuda")
    tf, mhz = ctypes.c_double(0.0), ctypes.c_double(0.0)
    _check(lib().a2d_mfma_ceiling(int(iters), int(bool(random_data)), _ptr(scratch), scratch.numel(),
                                  ctypes.byref(tf), ctypes.byref(mhz)))
    return tf.value, mhz.value


def forward_mix_ceiling(iters=6000):
    """Diagnostic (a2d_forward_mix_ceiling): (TFLOP/s of the forward loop's model - MFMA + LDS fragment +
    softmax arithmetic per MFMA -, shader MHz)."""
    n = int(lib().a2d_mfma_ceiling_scratch_bytes())
    scratch = torch.empty(max(n, 16), dtype=torch.uint8, device="cuda")
    tf, mhz = ctypes.c_double(0.0), ctypes.c_double(0.0)
    _check(lib().a2d_forward_mix_ceiling(int(iters), _ptr(scratch), scratch.numel(), ctypes.byref(tf), ctypes.byref(mhz)))
    return tf.value, mhz.value


LEAVE_MAILBOX, LEAVE_ARITHMETIC, LEAVE_BARRIER = 1, 2, 4


def backward_mix_ceiling(iters=6000, leave_out=0):
    """Diagnostic (a2d_backward_mix_ceiling): (TFLOP/s of the dK/dV loop's model - paired roles, natural and
    transposing LDS fragments, mailbox, one barrier per step -, shader MHz); leave_out: LEAVE_* bits."""
    n = int(lib().a2d_mfma_ceiling_scratch_bytes())
    scratch = torch.empty(max(n, 16), dtype=torch.uint8, device="cuda")
    tf, mhz = ctypes.c_double(0.0), ctypes.c_double(0.0)
    _check(lib().a2d_backward_mix_ceiling(int(iters), int(leave_out), _ptr(scratch), scratch.numel(),
                                          ctypes.byref(tf), ctypes.byref(mhz)))
    return tf.value, mhz.value


def lds_read_ceiling(iters=20000, transposing=False):
    """Diagnostic (a2d_lds_read_ceiling): (10^12 bytes per second the chip's LDS delivers to wavefronts that
    only read it, shader MHz)."""
    n = int(lib().a2d_mfma_ceiling_scratch_bytes())
    scratch = torch.empty(max(n, 16), dtype=torch.uint8, device="cuda")
    tb, mhz = ctypes.c_double(0.0), ctypes.c_double(0.0)
    _check(lib().a2d_lds_read_ceiling(int(iters), int(bool(transposing)), _ptr(scratch), scratch.numel(),
                                      ctypes.byref(tb), ctypes.byref(mhz)))
    return tb.value, mhz.value


def force_generic(on):
    """a2d_debug_force_generic: route every tile call to the vector-ALU kernels (debugging aid)."""
    lib().a2d_debug_force_generic(int(bool(on)))


def copy_probe(dst, src):
    """a2d_copy_probe: plain device copy of src into dst (contiguous device tensors of equal byte size)."""
    _plain([dst, src], "dst, src")
    n = src.numel() * src.element_size()
    if n != dst.numel() * dst.element_size():
        raise A2DError(-1, "dst and src differ in size")
    _check(lib().a2d_copy_probe(_ptr(dst), _ptr(src), n, _stream()))
    return dst


def _loaded_hip_runtime():
    """Path of the HIP runtime ALREADY mapped into this process (the one liba2d.so and torch use):
    events must come from that copy, not from a second one a search by name might load."""
    with open("/proc/self/maps") as f:
        for line in f:
            if "libamdhip64.so" in line:
                return line.split()[-1]
    raise RuntimeError("no HIP runtime is loaded in this process")


class KernelTrace:
    """a2d_debug_trace on the calling thread: `with KernelTrace(n) as tr:` records up to n HIP events
    (created here through the HIP runtime the library is linked against); after a device
    synchronisation tr.intervals_ms() gives the time between consecutive recorded events."""

    def __init__(self, n):
        self.n = int(n)
        lib()
        self._hip = ctypes.CDLL(_loaded_hip_runtime())
        self._hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self._hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self._hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self._ev = (ctypes.c_void_p * self.n)()
        for i in range(self.n):
            e = ctypes.c_void_p()
            if self._hip.hipEventCreate(ctypes.byref(e)) != 0:
                raise A2DError(-5, "hipEventCreate failed")
            self._ev[i] = e
        self.count = 0

    def __enter__(self):
        lib().a2d_debug_trace(self._ev, self.n)
        return self

    def __exit__(self, *exc):
        self.count = int(lib().a2d_debug_trace_count())
        lib().a2d_debug_trace(None, 0)
        return False

    def intervals_ms(self):
        """[t(event i+1) - t(event i)] for the recorded events; call after the device has finished them."""
        out = []
        for i in range(self.count - 1):
            ms = ctypes.c_float()
            if self._hip.hipEventElapsedTime(ctypes.byref(ms), self._ev[i], self._ev[i + 1]) != 0:
                raise A2DError(-5, "hipEventElapsedTime failed")
            out.append(ms.value)
        return out

    def close(self):
        for i in range(self.n):
            if self._ev[i]:
                self._hip.hipEventDestroy(self._ev[i])
                self._ev[i] = None


def version():
    return lib().a2d_version().decode()
