"""fp64 CPU oracle for the Attention2D tile kernels and AttnFix (arXiv 2503.15758).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the GPU library never does, and
this package never imports the GPU library.

The arithmetic lives in ``a2d_oracle.c`` (plain C, fp64, OpenMP over rows).
This module only compiles it with gcc, loads it with ctypes and marshals numpy
arrays.  Every array is fp64, C-contiguous, laid out ``[heads][rows][H]``
(matrices) or ``[heads][rows]`` (per-row statistics).

Functions and the passage each follows:
  attention_fwd   Sec. 2.1, Eq. (1)-(2)
  attention_bwd   gradient of Eq. (1)-(2) (textbook softmax-attention gradient)
  partial_fwd     Sec. 3.1, Eq. (3)
  attnfix_pair    Alg. 2 (AttnFix)
  fix             Alg. 2 folded over k partials + Alg. 1 line 6 + L = M + log D
  partial_bwd     Alg. 3 line 3 on one tile (final O / lse as inputs)
  fix_bwd         Alg. 3 lines 4-5 (sum of gradient partials)
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "a2d_oracle.c")
_SO = os.path.join(_HERE, "liba2d_oracle.so")
_lib = None


def build(force=False):
    """Compile a2d_oracle.c into liba2d_oracle.so (gcc, -O2, OpenMP, no -march)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall",
               "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_SO)
        _lib.a2d_oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads():
    return int(_load().a2d_oracle_num_threads())


_dp = ctypes.POINTER(ctypes.c_double)


def _c(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a


def _p(a):
    return a.ctypes.data_as(_dp)


def _pp(arrs):
    arr_t = _dp * len(arrs)
    return arr_t(*[_p(a) for a in arrs])


def attention_fwd(Q, K, V, scale, causal, return_p=False):
    """Full attention of [heads][n][H] inputs. Returns (O, lse[, P])."""
    Q, K, V = _c(Q), _c(K), _c(V)
    heads, n, H = Q.shape
    assert K.shape == Q.shape and V.shape == Q.shape
    O = np.empty_like(Q)
    lse = np.empty((heads, n))
    P = np.empty((heads, n, n)) if return_p else None
    _load().a2d_oracle_attention_fwd(
        ctypes.c_int(heads), ctypes.c_int(n), ctypes.c_int(H), _p(Q), _p(K), _p(V),
        ctypes.c_double(scale), ctypes.c_int(int(causal)), _p(O), _p(lse),
        _p(P) if return_p else None)
    return (O, lse, P) if return_p else (O, lse)


def attention_bwd(Q, K, V, dO, scale, causal):
    """Gradient of full attention. Returns (dQ, dK, dV)."""
    Q, K, V, dO = _c(Q), _c(K), _c(V), _c(dO)
    heads, n, H = Q.shape
    dQ, dK, dV = np.empty_like(Q), np.empty_like(Q), np.empty_like(Q)
    _load().a2d_oracle_attention_bwd(
        ctypes.c_int(heads), ctypes.c_int(n), ctypes.c_int(H), _p(Q), _p(K), _p(V),
        _p(dO), ctypes.c_double(scale), ctypes.c_int(int(causal)), _p(dQ), _p(dK), _p(dV))
    return dQ, dK, dV


def partial_fwd(Q, K, V, q_off, kv_off, causal, scale):
    """Eq. (3) on one tile. Q [heads][nq][H], K,V [heads][nkv][H]. Returns (N, m, d)."""
    Q, K, V = _c(Q), _c(K), _c(V)
    heads, nq, H = Q.shape
    nkv = K.shape[1]
    assert K.shape == (heads, nkv, H) and V.shape == K.shape
    N = np.empty((heads, nq, H))
    m = np.empty((heads, nq))
    d = np.empty((heads, nq))
    _load().a2d_oracle_partial_fwd(
        ctypes.c_int(heads), ctypes.c_int(nq), ctypes.c_int(nkv), ctypes.c_int(H),
        _p(Q), _p(K), _p(V), ctypes.c_int64(q_off), ctypes.c_int64(kv_off),
        ctypes.c_int(int(causal)), ctypes.c_double(scale), _p(N), _p(m), _p(d))
    return N, m, d


def segment_positions(segments):
    """Global key indices of a gathered KV tile: the concatenation of sub-blocks, sub-block s
    being `rows` consecutive tokens starting at token `kv_off` (list of (kv_off, rows))."""
    pos = [np.arange(off, off + rows, dtype=np.int64) for off, rows in segments]
    return np.ascontiguousarray(np.concatenate(pos) if pos else np.zeros(0, dtype=np.int64))


def partial_fwd_pos(Q, K, V, q_off, kpos, causal, scale):
    """Eq. (3) on one tile whose key r is token kpos[r]. Returns (N, m, d)."""
    Q, K, V = _c(Q), _c(K), _c(V)
    kpos = np.ascontiguousarray(kpos, dtype=np.int64)
    heads, nq, H = Q.shape
    nkv = K.shape[1]
    assert K.shape == (heads, nkv, H) and V.shape == K.shape and kpos.shape == (nkv,)
    N = np.empty((heads, nq, H))
    m = np.empty((heads, nq))
    d = np.empty((heads, nq))
    _load().a2d_oracle_partial_fwd_pos(
        ctypes.c_int(heads), ctypes.c_int(nq), ctypes.c_int(nkv), ctypes.c_int(H),
        _p(Q), _p(K), _p(V), ctypes.c_int64(q_off), kpos.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
        ctypes.c_int(int(causal)), ctypes.c_double(scale), _p(N), _p(m), _p(d))
    return N, m, d


def partial_bwd_pos(Q, K, V, O, dO, lse, q_off, kpos, causal, scale):
    """Per-tile gradients for a tile whose key r is token kpos[r]. Returns (dQ, dK, dV) partials."""
    Q, K, V, O, dO, lse = map(_c, (Q, K, V, O, dO, lse))
    kpos = np.ascontiguousarray(kpos, dtype=np.int64)
    heads, nq, H = Q.shape
    nkv = K.shape[1]
    assert O.shape == Q.shape and dO.shape == Q.shape and lse.shape == (heads, nq) and kpos.shape == (nkv,)
    dQ = np.empty((heads, nq, H))
    dK = np.empty((heads, nkv, H))
    dV = np.empty((heads, nkv, H))
    _load().a2d_oracle_partial_bwd_pos(
        ctypes.c_int(heads), ctypes.c_int(nq), ctypes.c_int(nkv), ctypes.c_int(H),
        _p(Q), _p(K), _p(V), _p(O), _p(dO), _p(lse), ctypes.c_int64(q_off),
        kpos.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), ctypes.c_int(int(causal)),
        ctypes.c_double(scale), _p(dQ), _p(dK), _p(dV))
    return dQ, dK, dV


def attnfix_pair(M1, N1, D1, M2, N2, D2):
    """Alg. 2 on two partial triples. Returns (M, N, D)."""
    M1, N1, D1, M2, N2, D2 = map(_c, (M1, N1, D1, M2, N2, D2))
    H = N1.shape[-1]
    rows = M1.size
    M, N, D = np.empty_like(M1), np.empty_like(N1), np.empty_like(D1)
    _load().a2d_oracle_attnfix_pair(
        ctypes.c_int64(rows), ctypes.c_int(H), _p(M1), _p(N1), _p(D1), _p(M2), _p(N2),
        _p(D2), _p(M), _p(N), _p(D))
    return M, N, D


def partial_fwd_acc(N_in, m_in, d_in, Q, K, V, q_off, kpos, causal, scale):
    """The compute-then-reduce pair of the overlapped algorithms (Alg. GatherCompute /
    GatherComputeScatter, lines Compute and Reduce): the tile's partial (Eq. (3)) merged by
    AttnFix (Alg. 2) into an existing partial triple of the same query block.  Returns (N, m, d)."""
    N, m, d = partial_fwd_pos(Q, K, V, q_off, kpos, causal, scale)
    M, Nn, D = attnfix_pair(m_in, N_in, d_in, m, N, d)
    return Nn, M, D


def normalised_partial(N, m, d):
    """The FlashAttention-style form of a partial triple (footnote of Sec. 3.2): O' = Diag(d^-1) N,
    lse' = m + log d; a row with no visible key gives O' = 0, lse' = -inf."""
    N, m, d = _c(N), _c(m), _c(d)
    with np.errstate(divide="ignore", invalid="ignore"):
        On = np.where(d[..., None] > 0, N / d[..., None], 0.0)
        lse = np.where(d > 0, m + np.log(d), -np.inf)
    return np.ascontiguousarray(On), np.ascontiguousarray(lse)


def fix_norm(Onorms, lses):
    """Merge of k normalised partials of one query block: with L = log sum_k exp(lse_k),
    O = sum_k exp(lse_k - L) O'_k (AttnFix, Alg. 2, and the final division of Alg. 1 line 6 written
    for the normalised form; sums in index order).  Returns (O, L)."""
    Onorms = [_c(a) for a in Onorms]
    lses = [_c(a) for a in lses]
    M = np.max(np.stack(lses), axis=0)
    Ms = np.where(np.isinf(M), 0.0, M)
    D = np.zeros_like(M)
    acc = np.zeros_like(Onorms[0])
    for On, l in zip(Onorms, lses):
        with np.errstate(invalid="ignore"):
            w = np.where(np.isinf(l), 0.0, np.exp(l - Ms))
        D += w
        acc += w[..., None] * On
    with np.errstate(divide="ignore", invalid="ignore"):
        O = np.where(D[..., None] > 0, acc / D[..., None], 0.0)
        L = np.where(D > 0, Ms + np.log(D), -np.inf)
    return O, L


def fix(Nparts, Mparts, Dparts):
    """k-way AttnFix + normalisation. Returns (O, lse)."""
    Nparts = [_c(a) for a in Nparts]
    Mparts = [_c(a) for a in Mparts]
    Dparts = [_c(a) for a in Dparts]
    k = len(Nparts)
    assert k >= 1 and len(Mparts) == k and len(Dparts) == k
    H = Nparts[0].shape[-1]
    rows = Mparts[0].size
    O = np.empty_like(Nparts[0])
    lse = np.empty_like(Mparts[0])
    _load().a2d_oracle_fix(
        ctypes.c_int(k), ctypes.c_int64(rows), ctypes.c_int(H), _pp(Nparts), _pp(Mparts),
        _pp(Dparts), _p(O), _p(lse))
    return O, lse


def partial_bwd(Q, K, V, O, dO, lse, q_off, kv_off, causal, scale):
    """Per-tile gradients from the final O / lse. Returns (dQ_part, dK_part, dV_part)."""
    Q, K, V, O, dO, lse = map(_c, (Q, K, V, O, dO, lse))
    heads, nq, H = Q.shape
    nkv = K.shape[1]
    assert O.shape == Q.shape and dO.shape == Q.shape and lse.shape == (heads, nq)
    dQ = np.empty((heads, nq, H))
    dK = np.empty((heads, nkv, H))
    dV = np.empty((heads, nkv, H))
    _load().a2d_oracle_partial_bwd(
        ctypes.c_int(heads), ctypes.c_int(nq), ctypes.c_int(nkv), ctypes.c_int(H),
        _p(Q), _p(K), _p(V), _p(O), _p(dO), _p(lse), ctypes.c_int64(q_off),
        ctypes.c_int64(kv_off), ctypes.c_int(int(causal)), ctypes.c_double(scale),
        _p(dQ), _p(dK), _p(dV))
    return dQ, dK, dV


def fix_bwd(parts):
    """Sum of k gradient partials (index order)."""
    parts = [_c(a) for a in parts]
    out = np.empty_like(parts[0])
    _load().a2d_oracle_fix_bwd(ctypes.c_int(len(parts)), ctypes.c_int64(parts[0].size),
                               _pp(parts), _p(out))
    return out
