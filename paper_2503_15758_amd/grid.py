"""The non-overlapped Attention2D forward and backward (Alg. 1 and Alg. 3) over an emulated
sqrt(P) x sqrt(P) device grid on ONE GPU.

Every "device" (r, c) of the paper becomes one tile call of the library; the collectives become
plain data movement on the one GPU (the row / column all-gathers are index gathers of the blocks,
the reduce-scatters are the library's merge calls).  Tiles are independent (Sec. 3.2), so they are
issued round-robin on several HIP streams of default priority.  This module only marshals: all
arithmetic of the method runs in the library's kernels.

Layouts of the sequence over the grid (Sec. 3.2):
  "cyclic"      Q block r = tokens {r + i sqrtP}, K/V block c = tokens {c + j sqrtP}: under the causal
                mask every tile does the same work; tile (r, c) masks i >= j (r >= c) or i >= j + 1.
  "contiguous"  block b = tokens [b T, (b + 1) T): tiles above the diagonal are empty and skipped.
"""
import math

import torch

from . import binding as a2d


def block_indices(n, grid, layout, device):
    """Token indices of block b = 0 .. grid - 1 (the same sets serve queries and keys)."""
    if n % grid:
        raise ValueError("sequence length %d is not a multiple of the grid side %d" % (n, grid))
    T = n // grid
    if layout == "cyclic":
        return [torch.arange(b, n, grid, device=device) for b in range(grid)]
    if layout == "contiguous":
        return [torch.arange(b * T, (b + 1) * T, device=device) for b in range(grid)]
    raise ValueError("layout must be 'cyclic' or 'contiguous'")


def tile_offsets(r, c, T, layout):
    """(q_off, kv_off) that express the causal mask of tile (r, c) in local indices."""
    if layout == "cyclic":
        return 0, (0 if r >= c else 1)
    return r * T, c * T


def _tiles(grid, causal, layout):
    """Tiles that hold any visible score, row by row."""
    skip_upper = causal and layout == "contiguous"
    return [(r, c) for r in range(grid) for c in range(grid) if not (skip_upper and c > r)]


class _Streams:
    """A few side streams (default priority) that start after the caller's stream and are joined
    back into it."""

    def __init__(self, count):
        self.main = torch.cuda.current_stream()
        self.side = [torch.cuda.Stream() for _ in range(max(1, count))]
        start = torch.cuda.Event()
        start.record(self.main)
        for s in self.side:
            s.wait_event(start)

    def of(self, i):
        return self.side[i % len(self.side)]

    def join(self):
        for s in self.side:
            e = torch.cuda.Event()
            e.record(s)
            self.main.wait_event(e)


def forward(Q, K, V, grid, causal=True, layout="cyclic", scale=None, streams=4, merge="kway"):
    """Alg. 1: O [heads][n][H] in the input dtype and lse [heads][n] (what the forward saves).
    merge: "kway" - the partials of a grid row in one a2d_fix pass; "ring" - folded pairwise by
    a2d_attnfix, one hop per partial as a ring reduce-scatter with AttnFix as its operator does
    (Alg. 1 line 5), then the division of line 6 (a2d_fix of the one remaining partial)."""
    heads, n, H = Q.shape
    scale = float(scale if scale is not None else 1.0 / math.sqrt(H))
    idx = block_indices(n, grid, layout, Q.device)
    T = n // grid
    Qb = [Q.index_select(1, i) for i in idx]           # row all-gather of the query blocks
    Kb = [K.index_select(1, i) for i in idx]           # column all-gather of the key / value blocks
    Vb = [V.index_select(1, i) for i in idx]
    f32 = dict(dtype=torch.float32, device=Q.device)
    tiles = _tiles(grid, causal, layout)
    parts = {t: (torch.empty(heads, T, H, **f32), torch.empty(heads, T, **f32), torch.empty(heads, T, **f32))
             for t in tiles}
    O = torch.empty_like(Q)
    lse = torch.empty(heads, n, **f32)
    st = _Streams(streams)
    for i, (r, c) in enumerate(tiles):                 # Alg. 1 line 4 on every device of the grid
        qo, ko = tile_offsets(r, c, T, layout)
        with torch.cuda.stream(st.of(i)):
            a2d.partial_fwd(Qb[r], Kb[c], Vb[c], qo, ko, causal, scale, out=parts[(r, c)])
    st.join()
    for r in range(grid):                              # Alg. 1 lines 5-6: AttnFix over the grid row, then 1 / D
        row = [parts[t] for t in tiles if t[0] == r]
        if merge == "ring":
            acc = row[0]
            for p in row[1:]:
                acc = a2d.attnfix([acc[0], p[0]], [acc[1], p[1]], [acc[2], p[2]])
            row = [acc]
        elif merge != "kway":
            raise ValueError("merge must be 'kway' or 'ring'")
        Or, lr = a2d.fix([p[0] for p in row], [p[1] for p in row], [p[2] for p in row], Q.dtype)
        O.index_copy_(1, idx[r], Or)
        lse.index_copy_(1, idx[r], lr)
    return O, lse


def backward(Q, K, V, O, dO, lse, grid, causal=True, layout="cyclic", scale=None, streams=4,
             ds_handover=True):
    """Alg. 3: dQ, dK, dV [heads][n][H] in the input dtype from the saved O and lse.
    ds_handover: give every stream the larger workspace with which the tile call keeps dS for its dQ
    contraction instead of recomputing the scores (about 2 T^2 bytes per head and stream more)."""
    heads, n, H = Q.shape
    scale = float(scale if scale is not None else 1.0 / math.sqrt(H))
    idx = block_indices(n, grid, layout, Q.device)
    T = n // grid
    gather = lambda X: [X.index_select(1, i) for i in idx]
    Qb, Kb, Vb, Ob, dOb, lb = gather(Q), gather(K), gather(V), gather(O), gather(dO), gather(lse)
    f32 = dict(dtype=torch.float32, device=Q.device)
    tiles = _tiles(grid, causal, layout)
    kvh = K.shape[0]                                   # fewer than `heads` with grouped-query heads
    parts = {t: (torch.empty(heads, T, H, **f32), torch.empty(kvh, T, H, **f32), torch.empty(kvh, T, H, **f32))
             for t in tiles}
    st = _Streams(streams)
    # one workspace per stream: calls that share a workspace must be ordered on one stream
    need = a2d.workspace_bytes(a2d.tile_desc(Qb[0], Kb[0], 0, 0, causal, scale),
                               a2d.OP_PARTIAL_BWD_DS if ds_handover else a2d.OP_PARTIAL_BWD)
    ws = [torch.empty(need, dtype=torch.uint8, device=Q.device) for _ in st.side]
    for i, (r, c) in enumerate(tiles):                 # Alg. 3 line 3
        qo, ko = tile_offsets(r, c, T, layout)
        with torch.cuda.stream(st.of(i)):
            a2d.partial_bwd(Qb[r], Kb[c], Vb[c], Ob[r], dOb[r], lb[r], qo, ko, causal, scale,
                            out=parts[(r, c)], workspace=ws[i % len(ws)], ds_handover=ds_handover)
    st.join()
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    for b in range(grid):                              # Alg. 3 lines 4-5: sums over the grid row / column
        dQ.index_copy_(1, idx[b], a2d.fix_bwd([parts[t][0] for t in tiles if t[0] == b], Q.dtype))
        dK.index_copy_(1, idx[b], a2d.fix_bwd([parts[t][1] for t in tiles if t[1] == b], Q.dtype))
        dV.index_copy_(1, idx[b], a2d.fix_bwd([parts[t][2] for t in tiles if t[1] == b], Q.dtype))
    return dQ, dK, dV
