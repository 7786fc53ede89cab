"""Shared helpers of the GPU parity tests (no arithmetic of the method lives here)."""
import numpy as np
import torch

# spec tolerances: max abs error against the fp64 oracle
TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}
# relative Frobenius bound used beside the absolute one so that small-magnitude
# outputs (gradients of long rows) are still checked meaningfully:
# fp32: accumulated rounding of H..Nkv-term sums; bf16: P / dS are rounded to 8 bits
REL = {torch.float32: 2e-5, torch.bfloat16: 1.5e-2}


def np64(t):
    return t.detach().to("cpu", torch.float64).numpy()


def max_abs(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    both_inf = np.isinf(a) & np.isinf(b) & (np.sign(a) == np.sign(b))
    with np.errstate(invalid="ignore"):
        diff = np.where(both_inf, 0.0, a - b)
    d = np.abs(diff)
    return (float(np.nanmax(d)) if d.size else 0.0), bool(np.isnan(diff).any())


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a))


def assert_close(got, ref, dtype, what, rel=True, scale_rows=False):
    """max-abs within the benchmark spec's tolerance (optionally per row relative to max(1, |ref|_inf of the
    row) for unnormalised quantities) and a relative Frobenius bound."""
    g = np64(got) if isinstance(got, torch.Tensor) else np.asarray(got, dtype=np.float64)
    r = np.asarray(ref, dtype=np.float64)
    assert g.shape == r.shape, (what, g.shape, r.shape)
    tol = TOL[dtype]
    if scale_rows:
        den = np.maximum(1.0, np.abs(r).max(axis=-1, keepdims=True))
        err, nan = max_abs(g / den, r / den)
    else:
        err, nan = max_abs(g, r)
    assert not nan, "%s: NaN in result" % what
    assert err <= tol, "%s: max abs err %.3e > %.1e" % (what, err, tol)
    if rel:
        finite = np.isfinite(r)
        rf = rel_fro(np.where(finite, g, 0.0), np.where(finite, r, 0.0))
        assert rf <= REL[dtype], "%s: relative Frobenius err %.3e > %.1e" % (what, rf, REL[dtype])
    return err


def grid_forward(a2d, Qb, Kb, Vb, T, causal, scale, out_dtype):
    """Emulates the sqrt(P) x sqrt(P) grid on one GPU with contiguous blocks: every (r, c) tile through
    a2d_partial_fwd, then a2d_fix across the partials of each query block (Alg. 1 lines 4-6)."""
    grid = len(Qb)
    parts = [[a2d.partial_fwd(Qb[r], Kb[c], Vb[c], r * T, c * T, causal, scale) for c in range(grid)]
             for r in range(grid)]
    fixed = [a2d.fix([p[0] for p in parts[r]], [p[1] for p in parts[r]], [p[2] for p in parts[r]], out_dtype)
             for r in range(grid)]
    return parts, fixed


def grid_backward(a2d, Qb, Kb, Vb, Ob, dOb, lseb, T, causal, scale, out_dtype):
    """Alg. 3 lines 3-5 on the emulated grid: per-tile gradient shares, then row / column sums."""
    grid = len(Qb)
    parts = [[a2d.partial_bwd(Qb[r], Kb[c], Vb[c], Ob[r], dOb[r], lseb[r], r * T, c * T, causal, scale)
              for c in range(grid)] for r in range(grid)]
    dQ = [a2d.fix_bwd([parts[r][c][0] for c in range(grid)], out_dtype) for r in range(grid)]
    dK = [a2d.fix_bwd([parts[r][c][1] for r in range(grid)], out_dtype) for c in range(grid)]
    dV = [a2d.fix_bwd([parts[r][c][2] for r in range(grid)], out_dtype) for c in range(grid)]
    return parts, dQ, dK, dV
