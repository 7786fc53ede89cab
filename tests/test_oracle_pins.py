"""Pins for the fp64 oracle: everything here is fixed by the paper or by mathematics,
and none of it is computed by the oracle's own code.

  - brute force straight from Sec. 2.1 Eq. (2) in pure Python (math.fsum),
  - closed forms (uniform scores, single key, two keys, dominant key),
  - torch's fp64 CPU softmax/matmul + autograd as an independent library route,
  - central finite differences for the gradient,
  - the partition identity of Sec. 3.1 (any disjoint split of the keys merges
    back to full attention), associativity/commutativity of Alg. 2,
  - the block recurrence of Sec. 2.2,
  - the grid index sets of Sec. 3.2 (exactly-once coverage of the score matrix).
"""
import itertools
import math
import os

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


# ----------------------------------------------------------------------------
# brute force, pure Python (Sec. 2.1, element form and Eq. (2))
# ----------------------------------------------------------------------------
def brute_attention(Q, K, V, scale, causal, q_off=0, kv_off=0):
    nq, H = len(Q), len(Q[0])
    nkv = len(K)
    O, LSE = [], []
    for i in range(nq):
        s = []
        for r in range(nkv):
            if causal and (q_off + i) < (kv_off + r):
                s.append(None)
            else:
                s.append(scale * math.fsum(Q[i][h] * K[r][h] for h in range(H)))
        vis = [x for x in s if x is not None]
        m = max(vis)
        d = math.fsum(math.exp(x - m) for x in vis)
        O.append([math.fsum(math.exp(s[r] - m) / d * V[r][j] for r in range(nkv) if s[r] is not None)
                  for j in range(H)])
        LSE.append(m + math.log(d))
    return O, LSE


@pytest.mark.parametrize("causal", [False, True])
def test_brute_force_4x4(causal):
    g = rng(7)
    Q, K, V = (g.standard_normal((1, 4, 4)) for _ in range(3))
    scale = 0.5
    O, lse = oracle.attention_fwd(Q, K, V, scale, causal)
    Ob, Lb = brute_attention(Q[0].tolist(), K[0].tolist(), V[0].tolist(), scale, causal)
    np.testing.assert_allclose(O[0], np.array(Ob), rtol=0, atol=1e-14)
    np.testing.assert_allclose(lse[0], np.array(Lb), rtol=0, atol=1e-14)


@pytest.mark.parametrize("q_off,kv_off", [(0, 0), (4, 0), (2, 4), (0, 1), (3, 5)])
def test_brute_force_partial_offsets(q_off, kv_off):
    """Eq. (3) normalised (n/d) and m + log d equal attention over the visible keys."""
    g = rng(11)
    nq, nkv, H = 5, 6, 3
    Q = g.standard_normal((1, nq, H)); K = g.standard_normal((1, nkv, H)); V = g.standard_normal((1, nkv, H))
    scale = 0.7
    N, m, d = oracle.partial_fwd(Q, K, V, q_off, kv_off, True, scale)
    for i in range(nq):
        nvis = sum(1 for r in range(nkv) if q_off + i >= kv_off + r)
        if nvis == 0:
            assert m[0, i] == -np.inf and d[0, i] == 0.0 and np.all(N[0, i] == 0.0)
            continue
        Ob, Lb = brute_attention([Q[0, i].tolist()], K[0, :nvis].tolist(), V[0, :nvis].tolist(), scale, False)
        np.testing.assert_allclose(N[0, i] / d[0, i], Ob[0], atol=1e-14)
        assert abs(m[0, i] + math.log(d[0, i]) - Lb[0]) < 1e-14
        # m is the true maximum of the visible scores
        smax = max(scale * float(Q[0, i] @ K[0, r]) for r in range(nvis))
        assert abs(m[0, i] - smax) < 1e-14
        assert d[0, i] >= 1.0 - 1e-15


# ----------------------------------------------------------------------------
# closed forms
# ----------------------------------------------------------------------------
def test_rows_of_p_sum_to_one():
    g = rng(1)
    Q, K, V = (g.standard_normal((2, 9, 5)) for _ in range(3))
    for causal in (False, True):
        _, _, P = oracle.attention_fwd(Q, K, V, 0.3, causal, return_p=True)
        np.testing.assert_allclose(P.sum(-1), 1.0, atol=1e-14)
        assert np.all(P >= 0)
        if causal:
            assert np.all(np.triu(P[0], 1) == 0.0)


def test_uniform_scores_closed_form():
    g = rng(2)
    n, H = 7, 4
    V = g.standard_normal((1, n, H))
    K = g.standard_normal((1, n, H))
    Q = np.zeros((1, n, H))
    O, lse = oracle.attention_fwd(Q, K, V, 0.5, False)
    np.testing.assert_allclose(O[0], np.broadcast_to(V[0].mean(0), (n, H)), atol=1e-14)
    np.testing.assert_allclose(lse[0], math.log(n), atol=1e-14)
    O, lse = oracle.attention_fwd(Q, K, V, 0.5, True)
    pref = np.cumsum(V[0], 0) / np.arange(1, n + 1)[:, None]
    np.testing.assert_allclose(O[0], pref, atol=1e-14)
    np.testing.assert_allclose(lse[0], np.log(np.arange(1, n + 1)), atol=1e-14)
    # identical keys give the same result whatever Q is
    Q2 = g.standard_normal((1, n, H))
    K2 = np.broadcast_to(K[0, :1], (1, n, H)).copy()
    O2, lse2 = oracle.attention_fwd(Q2, K2, V, 0.5, False)
    np.testing.assert_allclose(O2[0], np.broadcast_to(V[0].mean(0), (n, H)), atol=1e-13)
    np.testing.assert_allclose(lse2[0], 0.5 * (Q2[0] @ K[0, 0]) + math.log(n), atol=1e-13)


def test_single_key_and_two_keys():
    g = rng(3)
    q = g.standard_normal((1, 3, 2)); k = g.standard_normal((1, 1, 2)); v = g.standard_normal((1, 1, 2))
    N, m, d = oracle.partial_fwd(q, k, v, 0, 0, False, 1.0)
    np.testing.assert_allclose(N[0], np.broadcast_to(v[0, 0], (3, 2)), atol=0)
    np.testing.assert_allclose(d[0], 1.0, atol=0)
    np.testing.assert_allclose(m[0], q[0] @ k[0, 0], atol=1e-15)
    # two keys, H = 1: o = sigmoid(s0 - s1) v0 + sigmoid(s1 - s0) v1
    q = np.array([[[1.3]]]); k = np.array([[[0.4], [-0.9]]]); v = np.array([[[2.0], [-5.0]]])
    scale = 0.8
    s0, s1 = scale * 1.3 * 0.4, scale * 1.3 * -0.9
    sig = lambda x: 1.0 / (1.0 + math.exp(-x))
    N, m, d = oracle.partial_fwd(q, k, v, 0, 0, False, scale)
    assert abs(N[0, 0, 0] / d[0, 0] - (sig(s0 - s1) * 2.0 + sig(s1 - s0) * -5.0)) < 1e-15
    O, lse = oracle.attention_fwd(np.repeat(q, 2, 1), k, v, scale, False)
    assert abs(O[0, 0, 0] - (sig(s0 - s1) * 2.0 + sig(s1 - s0) * -5.0)) < 1e-15
    assert abs(lse[0, 0] - math.log(math.exp(s0) + math.exp(s1))) < 1e-15


def test_dominant_key_and_shift_invariance():
    g = rng(4)
    n, H = 6, 4
    Q, K, V = (g.standard_normal((1, n, H)) for _ in range(3))
    Kbig = K.copy()
    Q1 = np.abs(Q) + 0.1
    Kbig[0, 2] = 1000.0            # key 2 dominates every row (all q components > 0)
    O, _ = oracle.attention_fwd(Q1, Kbig, V, 1.0, False)
    np.testing.assert_allclose(O[0], np.broadcast_to(V[0, 2], (n, H)), atol=1e-12)
    # adding c * e_h to every key shifts each row's scores by c * q_{i,h}: O unchanged, lse shifted
    c = 3.25
    Kshift = K.copy(); Kshift[0, :, 1] += c
    O0, l0 = oracle.attention_fwd(Q, K, V, 0.5, False)
    O1, l1 = oracle.attention_fwd(Q, Kshift, V, 0.5, False)
    np.testing.assert_allclose(O1, O0, atol=1e-13)
    np.testing.assert_allclose(l1 - l0, 0.5 * c * Q[..., 1], atol=1e-13)


def test_key_permutation_invariance():
    g = rng(5)
    Q, K, V = (g.standard_normal((2, 8, 3)) for _ in range(3))
    perm = g.permutation(8)
    O0, l0 = oracle.attention_fwd(Q, K, V, 0.6, False)
    O1, l1 = oracle.attention_fwd(Q, K[:, perm], V[:, perm], 0.6, False)
    np.testing.assert_allclose(O1, O0, atol=1e-14)
    np.testing.assert_allclose(l1, l0, atol=1e-14)


# ----------------------------------------------------------------------------
# independent library route: torch fp64 CPU softmax + autograd
# ----------------------------------------------------------------------------
def torch_attention(Q, K, V, scale, causal, q_off=0, kv_off=0):
    S = scale * Q @ K.transpose(-1, -2)
    if causal:
        i = torch.arange(Q.shape[-2])[:, None] + q_off
        r = torch.arange(K.shape[-2])[None, :] + kv_off
        S = S.masked_fill(i < r, float("-inf"))
    return torch.softmax(S, -1) @ V, torch.logsumexp(S, -1)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("heads,n,H", [(2, 33, 8), (1, 64, 16)])
def test_fwd_bwd_vs_torch_autograd(causal, heads, n, H):
    g = rng(100 + n)
    Q, K, V, dO = (g.standard_normal((heads, n, H)) for _ in range(4))
    scale = 1.0 / math.sqrt(H)
    tq, tk, tv = (torch.tensor(x, requires_grad=True) for x in (Q, K, V))
    tO, tl = torch_attention(tq, tk, tv, scale, causal)
    (tO * torch.tensor(dO)).sum().backward()
    O, lse = oracle.attention_fwd(Q, K, V, scale, causal)
    np.testing.assert_allclose(O, tO.detach().numpy(), atol=1e-13)
    np.testing.assert_allclose(lse, tl.detach().numpy(), atol=1e-13)
    dQ, dK, dV = oracle.attention_bwd(Q, K, V, dO, scale, causal)
    np.testing.assert_allclose(dQ, tq.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dK, tk.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dV, tv.grad.numpy(), atol=1e-12)


def test_finite_difference_gradient():
    g = rng(9)
    heads, n, H = 1, 6, 3
    Q, K, V, G = (g.standard_normal((heads, n, H)) for _ in range(4))
    scale = 0.9
    for causal in (False, True):
        dQ, dK, dV = oracle.attention_bwd(Q, K, V, G, scale, causal)

        def f(q, k, v):
            return float((oracle.attention_fwd(q, k, v, scale, causal)[0] * G).sum())

        h = 1e-6
        for which, grad in ((0, dQ), (1, dK), (2, dV)):
            for idx in itertools.product(range(n), range(H)):
                args = [Q.copy(), K.copy(), V.copy()]
                args[which][0][idx] += h
                fp = f(*args)
                args[which][0][idx] -= 2 * h
                fm = f(*args)
                num = (fp - fm) / (2 * h)
                assert abs(num - grad[0][idx]) < 1e-7 * max(1.0, abs(num)), (causal, which, idx)


def test_gradient_invariants():
    g = rng(10)
    heads, n, H = 2, 12, 4
    Q, K, V, dO = (g.standard_normal((heads, n, H)) for _ in range(4))
    dQ, dK, dV = oracle.attention_bwd(Q, K, V, dO, 0.5, False)
    # rows of P sum to 1  =>  sum_r dV_r = sum_i dO_i
    np.testing.assert_allclose(dV.sum(1), dO.sum(1), atol=1e-13)
    # identical keys: scores do not depend on which key => dS = 0 => dQ = 0
    Kc = np.broadcast_to(K[:, :1], K.shape).copy()
    dQ, dK, dV = oracle.attention_bwd(Q, Kc, V, dO, 0.5, False)
    np.testing.assert_allclose(dQ, 0.0, atol=1e-14)
    # sum_r dS_{i,r} = 0  =>  sum_r dK_r = scale * sum_i (sum_r dS_ir) q_i = 0
    dQ, dK, dV = oracle.attention_bwd(Q, K, V, dO, 0.5, False)
    np.testing.assert_allclose(dK.sum(1), 0.0, atol=1e-13)


# ----------------------------------------------------------------------------
# Sec. 3.1: merging partials over any disjoint partition of the keys is exact
# ----------------------------------------------------------------------------
def _partitions(n, g):
    idx = np.arange(n)
    yield "contiguous", np.array_split(idx, 3)
    yield "cyclic", [idx[c::4] for c in range(4)]
    yield "random", np.array_split(g.permutation(n), 5)
    yield "uneven", [idx[:1], idx[1:2], idx[2:n - 3], idx[n - 3:]]
    yield "single", [idx]


def test_partition_identity_noncausal():
    g = rng(20)
    heads, n, H = 2, 29, 6
    Q, K, V = (g.standard_normal((heads, n, H)) * 2.0 for _ in range(3))
    scale = 0.4
    O, lse = oracle.attention_fwd(Q, K, V, scale, False)
    for name, parts in _partitions(n, g):
        trip = [oracle.partial_fwd(Q, K[:, p], V[:, p], 0, 0, False, scale) for p in parts]
        Of, lf = oracle.fix([t[0] for t in trip], [t[1] for t in trip], [t[2] for t in trip])
        np.testing.assert_allclose(Of, O, atol=1e-13, err_msg=name)
        np.testing.assert_allclose(lf, lse, atol=1e-13, err_msg=name)


@pytest.mark.parametrize("grid", [1, 2, 3, 4])
def test_partition_identity_causal_contiguous_grid(grid):
    """Contiguous blocks with global offsets, including tiles wholly above the diagonal."""
    g = rng(21)
    heads, T, H = 1, 5, 4
    n = grid * T
    Q, K, V = (g.standard_normal((heads, n, H)) for _ in range(3))
    scale = 0.5
    O, lse = oracle.attention_fwd(Q, K, V, scale, True)
    for r in range(grid):
        qs = slice(r * T, (r + 1) * T)
        trip = [oracle.partial_fwd(Q[:, qs], K[:, c * T:(c + 1) * T], V[:, c * T:(c + 1) * T],
                                   r * T, c * T, True, scale) for c in range(grid)]
        for c in range(r + 1, grid):     # above the diagonal: empty partials
            assert np.all(trip[c][1] == -np.inf) and np.all(trip[c][2] == 0) and np.all(trip[c][0] == 0)
        Of, lf = oracle.fix([t[0] for t in trip], [t[1] for t in trip], [t[2] for t in trip])
        np.testing.assert_allclose(Of, O[:, qs], atol=1e-13)
        np.testing.assert_allclose(lf, lse[:, qs], atol=1e-13)


@pytest.mark.parametrize("grid", [2, 3])
def test_partition_identity_causal_cyclic_grid(grid):
    """The paper's cyclic index sets (Sec. 3.2): Q_g(r) = {r + i sqrtP}, K_g(c) = {c + j sqrtP}.
    The mask of tile (r, c) is i >= j for r >= c and i >= j + 1 for r < c, i.e. offsets (0, 0) / (0, 1)."""
    g = rng(22)
    heads, T, H = 2, 6, 3
    n = grid * T
    Q, K, V = (g.standard_normal((heads, n, H)) for _ in range(3))
    scale = 0.7
    O, lse = oracle.attention_fwd(Q, K, V, scale, True)
    for r in range(grid):
        qi = np.arange(r, n, grid)
        trip = []
        for c in range(grid):
            ki = np.arange(c, n, grid)
            trip.append(oracle.partial_fwd(Q[:, qi], K[:, ki], V[:, ki], 0, 0 if r >= c else 1, True, scale))
        Of, lf = oracle.fix([t[0] for t in trip], [t[1] for t in trip], [t[2] for t in trip])
        np.testing.assert_allclose(Of, O[:, qi], atol=1e-13)
        np.testing.assert_allclose(lf, lse[:, qi], atol=1e-13)


def test_attnfix_pair_is_associative_and_commutative():
    g = rng(23)
    heads, n, H = 1, 10, 4
    Q, K, V = (g.standard_normal((heads, n, H)) * 3 for _ in range(3))
    parts = np.array_split(np.arange(n), 4)
    trip = [oracle.partial_fwd(Q, K[:, p], V[:, p], 0, 0, False, 1.0) for p in parts]
    Ok, lk = oracle.fix([t[0] for t in trip], [t[1] for t in trip], [t[2] for t in trip])
    for order in itertools.permutations(range(4)):
        N, m, d = trip[order[0]]
        for x in order[1:]:
            m, N, d = oracle.attnfix_pair(m, N, d, trip[x][1], trip[x][0], trip[x][2])
        np.testing.assert_allclose(N / d[..., None], Ok, atol=1e-13)
        np.testing.assert_allclose(m + np.log(d), lk, atol=1e-13)
    # tree order ((0,1),(2,3))
    a = oracle.attnfix_pair(trip[0][1], trip[0][0], trip[0][2], trip[1][1], trip[1][0], trip[1][2])
    b = oracle.attnfix_pair(trip[2][1], trip[2][0], trip[2][2], trip[3][1], trip[3][0], trip[3][2])
    m, N, d = oracle.attnfix_pair(*a, *b)
    np.testing.assert_allclose(N / d[..., None], Ok, atol=1e-13)


def test_attnfix_pair_hand_values():
    """Alg. 2 on numbers small enough to do by hand."""
    M1, D1, N1 = np.array([0.0]), np.array([2.0]), np.array([[4.0, -2.0]])
    M2, D2, N2 = np.array([math.log(2.0)]), np.array([1.5]), np.array([[1.0, 3.0]])
    M, N, D = oracle.attnfix_pair(M1, N1, D1, M2, N2, D2)
    # M = ln2, E1 = 1/2, E2 = 1
    assert M[0] == math.log(2.0)
    np.testing.assert_allclose(D, [0.5 * 2.0 + 1.5], atol=1e-15)
    np.testing.assert_allclose(N, [[0.5 * 4.0 + 1.0, 0.5 * -2.0 + 3.0]], atol=1e-15)
    O, lse = oracle.fix([N1, N2], [M1, M2], [D1, D2])
    np.testing.assert_allclose(O, [[3.0 / 2.5, 2.0 / 2.5]], atol=1e-15)
    np.testing.assert_allclose(lse, [math.log(2.0) + math.log(2.5)], atol=1e-15)
    # an empty partial is the identity of the merge
    Me, De, Ne = np.array([-np.inf]), np.array([0.0]), np.zeros((1, 2))
    M, N, D = oracle.attnfix_pair(M1, N1, D1, Me, Ne, De)
    assert M[0] == 0.0 and D[0] == 2.0 and np.all(N == N1)
    M, N, D = oracle.attnfix_pair(Me, Ne, De, Me, Ne, De)
    assert M[0] == -np.inf and D[0] == 0.0 and np.all(N == 0.0)
    O, lse = oracle.fix([Ne, Ne], [Me, Me], [De, De])
    assert np.all(O == 0.0) and lse[0] == -np.inf


def test_block_recurrence_matches_one_shot():
    """Sec. 2.2: folding blocks of B keys left to right gives the one-shot result."""
    g = rng(24)
    heads, nq, nkv, H, B = 1, 4, 20, 3, 4
    Q = g.standard_normal((heads, nq, H)); K = g.standard_normal((heads, nkv, H)) * 2
    V = g.standard_normal((heads, nkv, H))
    N1, m1, d1 = oracle.partial_fwd(Q, K, V, 0, 0, False, 1.0)
    N, m, d = oracle.partial_fwd(Q, K[:, :B], V[:, :B], 0, 0, False, 1.0)
    for b0 in range(B, nkv, B):
        Nb, mb, db = oracle.partial_fwd(Q, K[:, b0:b0 + B], V[:, b0:b0 + B], 0, 0, False, 1.0)
        m, N, d = oracle.attnfix_pair(m, N, d, mb, Nb, db)
    np.testing.assert_allclose(m, m1, atol=0)
    np.testing.assert_allclose(N, N1, atol=1e-13)
    np.testing.assert_allclose(d, d1, atol=1e-13)


# ----------------------------------------------------------------------------
# backward decomposition (Alg. 3): partial gradients sum to the full gradient
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("causal,layout", [(False, "contiguous"), (True, "contiguous"), (True, "cyclic")])
def test_partial_bwd_sums_to_full(causal, layout):
    g = rng(30)
    heads, grid, T, H = 2, 3, 4, 5
    n = grid * T
    Q, K, V, dO = (g.standard_normal((heads, n, H)) for _ in range(4))
    scale = 1 / math.sqrt(H)
    O, lse = oracle.attention_fwd(Q, K, V, scale, causal)
    dQ, dK, dV = oracle.attention_bwd(Q, K, V, dO, scale, causal)
    if layout == "contiguous":
        sets = [np.arange(b * T, (b + 1) * T) for b in range(grid)]
        offs = lambda r, c: (r * T, c * T)
    else:
        sets = [np.arange(b, n, grid) for b in range(grid)]
        offs = lambda r, c: (0, 0 if r >= c else 1)
    dq_parts = [[None] * grid for _ in range(grid)]
    dk_parts = [[None] * grid for _ in range(grid)]
    dv_parts = [[None] * grid for _ in range(grid)]
    for r in range(grid):
        for c in range(grid):
            qo, ko = offs(r, c)
            a, b, cc = oracle.partial_bwd(Q[:, sets[r]], K[:, sets[c]], V[:, sets[c]], O[:, sets[r]],
                                          dO[:, sets[r]], lse[:, sets[r]], qo, ko, causal, scale)
            dq_parts[r][c], dk_parts[r][c], dv_parts[r][c] = a, b, cc
    for r in range(grid):
        np.testing.assert_allclose(oracle.fix_bwd(dq_parts[r]), dQ[:, sets[r]], atol=1e-13)
    for c in range(grid):
        np.testing.assert_allclose(oracle.fix_bwd([dk_parts[r][c] for r in range(grid)]), dK[:, sets[c]], atol=1e-13)
        np.testing.assert_allclose(oracle.fix_bwd([dv_parts[r][c] for r in range(grid)]), dV[:, sets[c]], atol=1e-13)


def test_partial_bwd_vs_torch_autograd_of_tile():
    """A tile's gradient share equals autograd through exp(S_tile - lse) with lse, O held constant:
    d/dX sum_i [ sum_r exp(s_ir - lse_i) (dO_i . v_r) ] minus the delta term is what Alg. 3 line 3 returns.
    Checked through the equivalent statement: for a single tile covering all keys it is the full gradient."""
    g = rng(31)
    heads, nq, nkv, H = 1, 7, 9, 4
    Q = g.standard_normal((heads, nq, H)); K = g.standard_normal((heads, nkv, H))
    V = g.standard_normal((heads, nkv, H)); dO = g.standard_normal((heads, nq, H))
    scale = 0.5
    for causal, qo, ko in ((False, 0, 0), (True, 5, 0), (True, 3, 1)):
        tq, tk, tv = (torch.tensor(x, requires_grad=True) for x in (Q, K, V))
        tO, tl = torch_attention(tq, tk, tv, scale, causal, qo, ko)
        (tO * torch.tensor(dO)).sum().backward()
        dQ, dK, dV = oracle.partial_bwd(Q, K, V, tO.detach().numpy(), dO, tl.detach().numpy(), qo, ko, causal, scale)
        np.testing.assert_allclose(dQ, tq.grad.numpy(), atol=1e-13)
        np.testing.assert_allclose(dK, tk.grad.numpy(), atol=1e-13)
        np.testing.assert_allclose(dV, tv.grad.numpy(), atol=1e-13)


def test_fix_bwd_is_plain_sum():
    g = rng(32)
    parts = [g.standard_normal((2, 3, 4)) for _ in range(5)]
    np.testing.assert_allclose(oracle.fix_bwd(parts), sum(parts), atol=1e-15)
    np.testing.assert_array_equal(oracle.fix_bwd(parts[:1]), parts[0])


# ----------------------------------------------------------------------------
# Sec. 3.2 index sets and Fig. 2 (8 tokens on a 2 x 2 grid)
# ----------------------------------------------------------------------------
def _read_sets(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            key, vals = line.split(":")
            out[key.strip()] = [int(x) for x in vals.split()]
    return out


def test_fig2_index_sets_and_coverage():
    gold = _read_sets(os.path.join(GOLDEN, "fig2_grid_8tokens.txt"))
    N, P = 8, 4
    sp = 2
    count = np.zeros((N, N), dtype=int)
    unmasked = {}
    for r in range(sp):
        for c in range(sp):
            Qp = [r + sp * c + i * P for i in range(N // P)]
            Kt = [sp * r + c + i * P for i in range(N // P)]
            assert Qp == gold[f"Qp({r},{c})"] and Kt == gold[f"Kt({r},{c})"]
        Qg = sorted(set().union(*[gold[f"Qp({r},{j})"] for j in range(sp)]))
        assert Qg == [r + i * sp for i in range(N // sp)] == gold[f"Qg({r})"]
    for c in range(sp):
        Kg = sorted(set().union(*[gold[f"Kt({j},{c})"] for j in range(sp)]))
        assert Kg == [c + i * sp for i in range(N // sp)] == gold[f"Kg({c})"]
    for r in range(sp):
        for c in range(sp):
            u = 0
            for i in gold[f"Qg({r})"]:
                for j in gold[f"Kg({c})"]:
                    count[i, j] += 1
                    u += int(i >= j)
            unmasked[(r, c)] = u
    assert np.all(count == 1)                      # every score has exactly one owner (Fig. 2)
    T = N // sp
    assert unmasked == {(0, 0): T * (T + 1) // 2, (1, 0): T * (T + 1) // 2,
                        (1, 1): T * (T + 1) // 2, (0, 1): T * (T - 1) // 2}
    assert sum(unmasked.values()) == N * (N + 1) // 2
    # the local mask of tile (r, c) is lower triangular with offset 0 (r >= c) or 1 (r < c)
    for r in range(sp):
        for c in range(sp):
            for i, gi in enumerate(gold[f"Qg({r})"]):
                for j, gj in enumerate(gold[f"Kg({c})"]):
                    assert (gi >= gj) == (i >= j + (0 if r >= c else 1))


# ----------------------------------------------------------------------------
# gathered key/value tiles: sub-blocks with their own global offsets (the Compute line of
# Alg. GatherComputeScatter; Sec. 4.1 calls the resulting mask step-like)
# ----------------------------------------------------------------------------
def brute_positions(Q, K, V, scale, q_off, kpos):
    """Pure Python: attention of each query over the keys whose position does not exceed its own."""
    out = []
    for i in range(len(Q)):
        vis = [r for r in range(len(K)) if kpos[r] <= q_off + i]
        if not vis:
            out.append(None)
            continue
        s = [scale * math.fsum(Q[i][h] * K[r][h] for h in range(len(Q[0]))) for r in vis]
        m = max(s)
        d = math.fsum(math.exp(x - m) for x in s)
        o = [math.fsum(math.exp(s[t] - m) / d * V[r][j] for t, r in enumerate(vis)) for j in range(len(V[0]))]
        out.append((o, m + math.log(d), m))
    return out


def test_segment_positions():
    pos = oracle.segment_positions([(10, 3), (0, 2), (7, 1)])
    assert pos.tolist() == [10, 11, 12, 0, 1, 7]


def test_gathered_tile_brute_force():
    g = rng(40)
    nq, H = 6, 3
    segs = [(4, 3), (0, 4), (9, 2), (2, 1)]          # unordered, overlapping, different lengths
    kpos = oracle.segment_positions(segs)
    nkv = len(kpos)
    Q = g.standard_normal((1, nq, H)); K = g.standard_normal((1, nkv, H)); V = g.standard_normal((1, nkv, H))
    scale, q_off = 0.6, 3
    N, m, d = oracle.partial_fwd_pos(Q, K, V, q_off, kpos, True, scale)
    ref = brute_positions(Q[0].tolist(), K[0].tolist(), V[0].tolist(), scale, q_off, kpos.tolist())
    for i, r in enumerate(ref):
        if r is None:
            assert m[0, i] == -np.inf and d[0, i] == 0.0 and np.all(N[0, i] == 0.0)
            continue
        np.testing.assert_allclose(N[0, i] / d[0, i], r[0], atol=1e-14)
        assert abs(m[0, i] + math.log(d[0, i]) - r[1]) < 1e-14 and abs(m[0, i] - r[2]) < 1e-14
    # without the mask the positions do not matter
    a = oracle.partial_fwd_pos(Q, K, V, q_off, kpos, False, scale)
    b = oracle.partial_fwd(Q, K, V, 0, 0, False, scale)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)


def test_gathered_tile_equals_merge_of_its_segments():
    """One call on the gathered tile = AttnFix over one call per sub-block (the identity of Sec. 3.1);
    its gradients: dQ is the sum over the sub-blocks, dK / dV their concatenation (Alg. 3 lines 4-5)."""
    g = rng(41)
    heads, nq, H = 2, 9, 4
    segs = [(0, 5), (12, 4), (6, 7), (30, 3)]        # the last one is wholly invisible
    kpos = oracle.segment_positions(segs)
    nkv = len(kpos)
    Q = g.standard_normal((heads, nq, H)); K = g.standard_normal((heads, nkv, H))
    V = g.standard_normal((heads, nkv, H)); dO = g.standard_normal((heads, nq, H))
    scale, q_off = 0.5, 8
    N, m, d = oracle.partial_fwd_pos(Q, K, V, q_off, kpos, True, scale)
    trip, start = [], 0
    for off, rows in segs:
        trip.append(oracle.partial_fwd(Q, K[:, start:start + rows], V[:, start:start + rows], q_off, off, True, scale))
        start += rows
    O1, l1 = oracle.fix([N], [m], [d])
    O2, l2 = oracle.fix([t[0] for t in trip], [t[1] for t in trip], [t[2] for t in trip])
    np.testing.assert_allclose(O1, O2, atol=1e-14)
    np.testing.assert_allclose(l1, l2, atol=1e-14)
    assert np.array_equal(m, np.max(np.stack([t[1] for t in trip]), axis=0))
    dQ, dK, dV = oracle.partial_bwd_pos(Q, K, V, O1, dO, l1, q_off, kpos, True, scale)
    dq_sum, start = np.zeros_like(dQ), 0
    for off, rows in segs:
        a, b, c = oracle.partial_bwd(Q, K[:, start:start + rows], V[:, start:start + rows], O1, dO, l1,
                                     q_off, off, True, scale)
        dq_sum += a
        np.testing.assert_allclose(dK[:, start:start + rows], b, atol=1e-14)
        np.testing.assert_allclose(dV[:, start:start + rows], c, atol=1e-14)
        start += rows
    np.testing.assert_allclose(dQ, dq_sum, atol=1e-13)
    assert np.all(dK[:, -3:] == 0.0) and np.all(dV[:, -3:] == 0.0)


@pytest.mark.parametrize("grid", [2, 3])
def test_gathered_tile_cyclic_layout_reproduces_full_attention(grid):
    """Overlapped algorithm, cyclic 1D layout: device (r, c) holds query block Q_n = tokens
    {r' + sqrtP c' + i P} and the gathered K_g = tokens {c + j sqrtP}, made of sqrtP sub-blocks
    {c + sqrtP s + j P}.  Against sub-block s the mask is i >= j when the block's first token does
    not exceed the query block's, else i >= j + 1: segments (0 | 1, N / P).  Merging the sqrtP
    gathered-tile results of a query block over the grid columns gives rows of full attention."""
    g = rng(42)
    heads, t, H = 1, 3, 3                      # t = N / P tokens per block
    P = grid * grid
    n = P * t
    Q, K, V, dO = (g.standard_normal((heads, n, H)) for _ in range(4))
    scale = 0.8
    O, lse = oracle.attention_fwd(Q, K, V, scale, True)
    dQf, dKf, dVf = oracle.attention_bwd(Q, K, V, dO, scale, True)
    dK_acc, dV_acc = np.zeros_like(K), np.zeros_like(V)
    for qa in range(P):                        # query block: tokens qa + i P
        qi = np.arange(qa, n, P)
        trip, keysets, segsets = [], [], []
        for c in range(grid):                  # gathered keys of grid column c
            ki = np.concatenate([np.arange(c + grid * s, n, P) for s in range(grid)])
            segs = [(0 if c + grid * s <= qa else 1, t) for s in range(grid)]
            trip.append(oracle.partial_fwd_pos(Q[:, qi], K[:, ki], V[:, ki], 0, oracle.segment_positions(segs), True, scale))
            keysets.append(ki); segsets.append(segs)
        Of, lf = oracle.fix([x[0] for x in trip], [x[1] for x in trip], [x[2] for x in trip])
        np.testing.assert_allclose(Of, O[:, qi], atol=1e-13)
        np.testing.assert_allclose(lf, lse[:, qi], atol=1e-13)
        dq = np.zeros_like(Of)
        for ki, segs in zip(keysets, segsets):
            a, b, cc = oracle.partial_bwd_pos(Q[:, qi], K[:, ki], V[:, ki], Of, dO[:, qi], lf, 0,
                                              oracle.segment_positions(segs), True, scale)
            dq += a
            dK_acc[:, ki] += b
            dV_acc[:, ki] += cc
        np.testing.assert_allclose(dq, dQf[:, qi], atol=1e-13)
    np.testing.assert_allclose(dK_acc, dKf, atol=1e-13)
    np.testing.assert_allclose(dV_acc, dVf, atol=1e-13)


# ----------------------------------------------------------------------------
# accumulating tile call = FlashAttn followed by AttnFix (Compute and Reduce lines of the
# overlapped algorithms, Sec. 3.4)
# ----------------------------------------------------------------------------
def test_accumulating_partial_walks_to_full_attention():
    g = rng(50)
    heads, grid, T, H = 2, 3, 5, 4
    n = grid * T
    Q, K, V = (g.standard_normal((heads, n, H)) for _ in range(3))
    scale = 0.6
    O, lse = oracle.attention_fwd(Q, K, V, scale, True)
    for r in range(grid):
        qs = slice(r * T, (r + 1) * T)
        N = np.zeros((heads, T, H)); m = np.full((heads, T), -np.inf); d = np.zeros((heads, T))
        for c in (2, 0, 1):                                 # any order, including the empty tile above the diagonal
            ks = slice(c * T, (c + 1) * T)
            prev = (N.copy(), m.copy(), d.copy())
            N, m, d = oracle.partial_fwd_acc(N, m, d, Q[:, qs], K[:, ks], V[:, ks], r * T,
                                             oracle.segment_positions([(c * T, T)]), True, scale)
            assert np.all(m >= prev[1])                     # the maximum only grows
            if np.all(np.isinf(prev[1])):                   # from the empty triple: the tile's own partial, exactly
                P = oracle.partial_fwd(Q[:, qs], K[:, ks], V[:, ks], r * T, c * T, True, scale)
                for x, y in zip((N, m, d), P):
                    np.testing.assert_array_equal(x, y)
        Of, lf = oracle.fix([N], [m], [d])
        np.testing.assert_allclose(Of, O[:, qs], atol=1e-13)
        np.testing.assert_allclose(lf, lse[:, qs], atol=1e-13)


# ----------------------------------------------------------------------------
# normalised partial format (O' = N / d, lse' = m + log d)
# ----------------------------------------------------------------------------
def test_normalised_partials_merge_like_the_triples():
    g = rng(60)
    heads, T, H, grid = 2, 5, 3, 4
    n = grid * T
    Q, K, V = (g.standard_normal((heads, n, H)) for _ in range(3))
    scale = 0.9
    O, lse = oracle.attention_fwd(Q, K, V, scale, True)
    for r in (0, 2, 3):
        qs = slice(r * T, (r + 1) * T)
        trip = [oracle.partial_fwd(Q[:, qs], K[:, c * T:(c + 1) * T], V[:, c * T:(c + 1) * T], r * T, c * T, True, scale)
                for c in range(grid)]                       # includes empty tiles above the diagonal
        norm = [oracle.normalised_partial(*t) for t in trip]
        for (On, ln), (N, m, d) in zip(norm, trip):
            empty = d == 0
            assert np.all(np.isinf(ln[empty])) and np.all(On[empty] == 0)
            # a normalised partial alone is attention over the tile's visible keys: rows are convex combinations of V
            assert np.all(np.abs(On) <= np.abs(V).max() + 1e-12)
        O1, l1 = oracle.fix_norm([x[0] for x in norm], [x[1] for x in norm])
        O2, l2 = oracle.fix([t[0] for t in trip], [t[1] for t in trip], [t[2] for t in trip])
        np.testing.assert_allclose(O1, O2, atol=1e-14)
        np.testing.assert_allclose(l1, l2, atol=1e-14)
        np.testing.assert_allclose(O1, O[:, qs], atol=1e-13)
        np.testing.assert_allclose(l1, lse[:, qs], atol=1e-13)
    # closed form: two partials with equal lse average their outputs; an empty one is ignored
    a, b = g.standard_normal((1, 2, 3)), g.standard_normal((1, 2, 3))
    l = np.array([[0.3, -1.0]])
    Om, Lm = oracle.fix_norm([a, b, np.zeros_like(a)], [l, l, np.full_like(l, -np.inf)])
    np.testing.assert_allclose(Om, (a + b) / 2, atol=1e-15)
    np.testing.assert_allclose(Lm, l + math.log(2.0), atol=1e-15)
