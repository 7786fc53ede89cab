"""GPU parity at every launch shape of the tile kernels, on sizes the oracle still finishes.

The forward, dQ and dQ-from-dS kernels exist in several instantiations, chosen from the number of
query blocks against the number of compute units (256 on MI355X):
  * workgroups of eight wavefronts (256 query rows) once heads * ceil(nq / 256) reaches the number
    of compute units - the one every paper-sized workload runs;
  * workgroups of four wavefronts (128 rows) below that;
  * when even heads * ceil(nq / 128) is at most the number of compute units, 128-row workgroups of
    eight wavefronts in two key lanes whose partials (forward) or sums (dQ) are merged inside the
    kernel (the small cases of test_gpu_parity.py all take this one).
The cases here have many heads and short, RAGGED tiles, so that each regime is reached (with the
by-size workgroup order under a causal mask, and head counts that leave a partial last chunk of
heads per XCD) for every head size, in every form of the calls: plain, accumulating, normalised,
gathered, grouped heads, both backward paths.  The oracle checks whole heads: the first, the last,
and heads whose index is 1..6 modulo the 8 XCDs.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2503_15758_amd import synth
from helpers import assert_close, np64

pytestmark = pytest.mark.gpu

BF = torch.bfloat16
CUS = 256     # compute units of MI355X: the launchers' threshold for the eight-wavefront kernels


@pytest.fixture(scope="module")
def a2d():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2503_15758_amd import binding
    binding.lib()          # raises if the HIP library has not been built
    return binding


def dev(t):
    return t.to("cuda")


# heads, kv_heads, nq, nkv, H, causal, q_off, kv_off
CASES = [
    (64, 64, 1100, 700, 96, True, 200, 0),      # diagonal through the tile, ragged rows and keys
    (40, 40, 1700, 700, 80, True, 0, 300),      # 5 heads per XCD: last by-size chunk holds one; first rows see no key
    (72, 72, 1000, 900, 64, True, 500, 0),      # 9 heads per XCD: chunks of 4, 4, 1
    (33, 33, 2100, 300, 128, True, 0, 1500),    # head count not a multiple of 8; most rows see nothing
    (64, 64, 1100, 700, 128, False, 0, 0),      # no mask (head-by-head order), ragged
    (64, 16, 1100, 700, 96, True, 200, 0),      # grouped heads: 4 query heads per key/value head
    (96, 8, 700, 500, 128, True, 100, 0),       # 12 query heads per key/value head
    (264, 264, 250, 130, 80, True, 100, 0),     # one ragged query block per head, very many heads
]


def _ids(c):
    return "%dq%dkv_%dx%dxH%d_%s" % (c[0], c[1], c[2], c[3], c[4], "causal" if c[5] else "full")


def _heads_to_check(heads):
    """first, last, and one head of each residue 1..6 modulo 8 (spread over the head range)."""
    picks = {0, heads - 1}
    for res in range(1, 7):
        cand = [h for h in range(heads) if h % 8 == res]
        if cand:
            picks.add(cand[(res * len(cand)) // 7])
    return sorted(picks)


def _fwd_close(got, ref, what):
    Ng, mg, lg = (np64(x) for x in got)
    Nr, mr, lr = ref
    empty = np.isinf(mr)
    assert np.array_equal(np.isinf(mg) & (mg < 0), empty), what + ": set of empty rows differs"
    assert np.all(lg[empty] == 0.0) and np.all(Ng[empty] == 0.0), what + ": empty rows not zero"
    ok = ~empty
    if ok.any():
        assert_close(mg[ok], mr[ok], BF, what + " m", rel=False)
        assert_close(Ng[ok] / lg[ok][:, None], Nr[ok] / lr[ok][:, None], BF, what + " N/l")
        assert_close(mg[ok] + np.log(lg[ok]), mr[ok] + np.log(lr[ok]), BF, what + " m+ln l", rel=False)
        assert_close(Ng[ok], Nr[ok], BF, what + " N (per-row scaled)", rel=False, scale_rows=True)


# between the two thresholds: 128-row workgroups of four wavefronts, two per compute unit
CASES_FOUR = [
    (30, 30, 1100, 700, 96, True, 200, 0),      # 150 blocks of 256 rows, 270 of 128
    (36, 36, 1000, 400, 64, True, 300, 0),
    (24, 24, 1400, 500, 128, True, 0, 700),     # the first rows see no key
    (24, 6, 1400, 600, 80, False, 0, 0),        # grouped heads, no mask
]

# at most one 128-row block per compute unit: the forward and dQ kernels walk the keys in two lanes
CASES_LANES = [
    (8, 8, 700, 900, 128, True, 400, 0),        # diagonal through the tile: the lanes' shares differ
    (12, 12, 300, 1000, 80, True, 900, 0),      # an odd number of visible key blocks for most workgroups
    (16, 16, 130, 260, 64, False, 0, 0),        # a second, nearly empty query block per head
    (4, 2, 1000, 330, 96, True, 0, 0),          # grouped heads; short rows whose second lane has no block
    (3, 3, 200, 200, 128, True, 0, 150),        # most rows see nothing; the workgroup has at most one block
]


@pytest.mark.parametrize("case", CASES, ids=_ids)
def test_eight_wavefront_kernels_every_call_form(a2d, case):
    assert case[0] * ((case[2] + 255) // 256) >= CUS, "the case must take the eight-wavefront kernels"
    _every_call_form(a2d, case, "8w")


@pytest.mark.parametrize("case", CASES_FOUR, ids=_ids)
def test_four_wavefront_kernels_every_call_form(a2d, case):
    assert case[0] * ((case[2] + 255) // 256) < CUS < case[0] * ((case[2] + 127) // 128), \
        "the case must take the four-wavefront kernels with one key lane"
    _every_call_form(a2d, case, "4w")


@pytest.mark.parametrize("case", CASES_LANES, ids=_ids)
def test_two_key_lane_kernels_every_call_form(a2d, case):
    assert case[0] * ((case[2] + 127) // 128) <= CUS, "the case must take the kernels with two key lanes"
    _every_call_form(a2d, case, "2 lanes")


def _every_call_form(a2d, case, regime):
    heads, kvh, nq, nkv, H, causal, q_off, kv_off = case
    print("launch-variant case", regime, case, flush=True)
    grp = heads // kvh
    scale = 1.0 / math.sqrt(H)
    Q = synth.normal((heads, nq, H), 97, 0, 1.0, "bf16")
    K = synth.normal((kvh, nkv, H), 97, 1, 1.0, "bf16")
    V = synth.normal((kvh, nkv, H), 97, 2, 1.0, "bf16")
    dO = synth.normal((heads, nq, H), 97, 3, 1.0, "bf16")
    # a second, always visible key block of the same query block: makes the final lse finite on
    # every row and serves as the triple the accumulating call continues from
    K2 = synth.normal((kvh, 72, H), 97, 4, 1.0, "bf16")
    V2 = synth.normal((kvh, 72, H), 97, 5, 1.0, "bf16")
    hs = _heads_to_check(heads)
    if grp > 1:     # the gradients of a key/value head need every query head of its group
        hs = sorted(set(hs) | set(range(grp)) | set(range(heads - grp, heads)))
    kh = [h // grp for h in hs]
    Qh, dOh = np64(Q[hs]), np64(dO[hs])
    Kh, Vh, K2h, V2h = np64(K[kh]), np64(V[kh]), np64(K2[kh]), np64(V2[kh])
    what = "%s %s" % (regime, case)
    Qd, Kd, Vd, dOd = dev(Q), dev(K), dev(V), dev(dO)

    # ---- forward: plain, twice (bitwise), normalised
    ref = oracle.partial_fwd(Qh, Kh, Vh, q_off, kv_off, causal, scale)
    got = a2d.partial_fwd(Qd, Kd, Vd, q_off, kv_off, causal, scale)
    again = a2d.partial_fwd(Qd, Kd, Vd, q_off, kv_off, causal, scale)
    On, lsen = a2d.partial_fwd_norm(Qd, Kd, Vd, q_off, kv_off, causal, scale)
    torch.cuda.synchronize()
    _fwd_close([x[hs] for x in got], ref, what + " fwd")
    for x, y in zip(got, again):
        assert torch.equal(x, y), what + ": forward not reproducible"
    Onr, lsenr = oracle.normalised_partial(*ref)
    ok = ~np.isinf(ref[1])
    assert_close(np64(On[hs])[ok], Onr[ok], BF, what + " O'")
    assert_close(np64(lsen[hs])[ok], lsenr[ok], BF, what + " lse'", rel=False)
    assert np.all(np64(On[hs])[~ok] == 0.0) and np.all(np.isneginf(np64(lsen[hs])[~ok]))

    # ---- accumulating forward: continue from the triple of the second key block
    t2 = a2d.partial_fwd(Qd, dev(K2), dev(V2), 0, 0, False, scale)
    ref2 = oracle.partial_fwd(Qh, K2h, V2h, 0, 0, False, scale)
    trip = tuple(x.clone() for x in t2)
    a2d.partial_fwd(Qd, Kd, Vd, q_off, kv_off, causal, scale, out=trip, accumulate=True)
    torch.cuda.synchronize()
    kpos = np.arange(kv_off, kv_off + nkv, dtype=np.int64)
    refa = oracle.partial_fwd_acc(ref2[0], ref2[1], ref2[2], Qh, Kh, Vh, q_off, kpos, causal, scale)
    _fwd_close([x[hs] for x in trip], refa, what + " fwd acc")

    # ---- gathered tile: the same keys presented as three sub-blocks at different places
    a = max(64, (nkv // 3 // 64) * 64)
    b = max(a + 64, (2 * nkv // 3 // 64) * 64)
    assert b < nkv
    segs = [(kv_off + 7, a), (kv_off + 400, b - a), (kv_off, nkv - b)]
    spos = oracle.segment_positions(segs)
    refs = oracle.partial_fwd_pos(Qh, Kh, Vh, q_off, spos, causal, scale)
    gots = a2d.partial_fwd(Qd, Kd, Vd, q_off, 0, causal, scale, segments=segs)
    torch.cuda.synchronize()
    _fwd_close([x[hs] for x in gots], refs, what + " fwd seg")

    # ---- backward from the final O / lse over both key blocks, both paths, plain and gathered
    Of, lsef = oracle.fix([ref[0], ref2[0]], [ref[1], ref2[1]], [ref[2], ref2[2]])
    O_all, lse_all = a2d.fix([got[0], t2[0]], [got[1], t2[1]], [got[2], t2[2]], BF)
    torch.cuda.synchronize()
    assert_close(np64(O_all[hs]), Of, BF, what + " merged O")
    assert_close(np64(lse_all[hs]), lsef, BF, what + " merged lse", rel=False)
    # what the backward is given: on the checked heads the ORACLE's final O / lse, rounded to the
    # storage types (the other heads keep the merged values; nothing is compared there)
    O_all, lse_all = O_all.clone(), lse_all.clone()
    O_all[hs] = dev(torch.from_numpy(Of).to(BF))
    lse_all[hs] = dev(torch.from_numpy(lsef).to(torch.float32))
    torch.cuda.synchronize()
    O_h, lse_h = np64(torch.from_numpy(Of).to(BF)), np64(torch.from_numpy(lsef).to(torch.float32))

    def grads_ref(pos):
        return oracle.partial_bwd_pos(Qh, Kh, Vh, O_h, dOh, lse_h, q_off, pos, causal, scale)

    d = a2d.tile_desc(Qd, Kd, q_off, kv_off, causal, scale)
    assert a2d.workspace_bytes(d, a2d.OP_PARTIAL_BWD_DS) > a2d.workspace_bytes(d, a2d.OP_PARTIAL_BWD)
    for pos, kw, tag in ((kpos, {}, "plain"), (spos, dict(segments=segs), "seg")):
        rq, rk, rv = grads_ref(pos)
        for handover in (False, True):
            dQ, dK, dV = a2d.partial_bwd(Qd, Kd, Vd, O_all, dOd, lse_all, q_off, 0 if kw else kv_off, causal, scale,
                                         ds_handover=handover, **kw)
            torch.cuda.synchronize()
            w2 = "%s bwd %s handover=%s" % (what, tag, handover)
            assert_close(np64(dQ[hs]), rq, BF, w2 + " dQ", rel=bool(np.abs(rq).max() > 1e-3))
            if grp == 1:
                assert_close(np64(dK[kh]), rk, BF, w2 + " dK", rel=bool(np.abs(rk).max() > 1e-3))
                assert_close(np64(dV[kh]), rv, BF, w2 + " dV", rel=bool(np.abs(rv).max() > 1e-3))
            if handover and not kw:
                # accumulating backward: dQ += on top of a known buffer
                acc = (torch.full_like(dQ, 0.25), torch.empty_like(dK), torch.empty_like(dV))
                a2d.partial_bwd(Qd, Kd, Vd, O_all, dOd, lse_all, q_off, kv_off, causal, scale, out=acc,
                                accumulate=True, ds_handover=True)
                torch.cuda.synchronize()
                assert_close(np64(acc[0][hs]), rq + 0.25, BF, w2 + " dQ +=", rel=False)
                assert torch.equal(acc[1], dK) and torch.equal(acc[2], dV)
            del dQ
    if grp > 1:
        # grouped heads: dK, dV of a key/value head are sums over ALL its query heads - oracle on
        # the whole group of the first and the last key/value head
        for kv in (0, kvh - 1):
            ix = [hs.index(h) for h in range(kv * grp, (kv + 1) * grp)]
            _, rk, rv = oracle.partial_bwd_pos(Qh[ix], Kh[ix], Vh[ix], O_h[ix], dOh[ix], lse_h[ix], q_off, kpos,
                                               causal, scale)
            for handover, split in ((False, False), (True, False), (True, True)):
                _, dK, dV = a2d.partial_bwd(Qd, Kd, Vd, O_all, dOd, lse_all, q_off, kv_off, causal, scale,
                                            ds_handover=handover, split_groups=split)
                torch.cuda.synchronize()
                w2 = "%s gqa bwd kv head %d handover=%s split=%s" % (what, kv, handover, split)
                assert_close(np64(dK[kv]), rk.sum(axis=0), BF, w2 + " dK")
                assert_close(np64(dV[kv]), rv.sum(axis=0), BF, w2 + " dV")


def test_strided_inputs_eight_wavefront_kernels(a2d):
    """Q, K, V, O, dO as views of a packed [rows][..][heads][H] buffer at a launch shape of the
    eight-wavefront kernels: bit for bit the results on plain copies."""
    heads, n, H = 72, 900, 96
    scale = 1.0 / math.sqrt(H)
    packed = dev(synth.normal((n, 3, heads, H), 98, 0, 1.0, "bf16"))
    Qv, Kv, Vv = (packed[:, i].permute(1, 0, 2) for i in range(3))
    Qc, Kc, Vc = Qv.contiguous(), Kv.contiguous(), Vv.contiguous()
    got = a2d.partial_fwd(Qv, Kv, Vv, 0, 0, True, scale)
    ref = a2d.partial_fwd(Qc, Kc, Vc, 0, 0, True, scale)
    torch.cuda.synchronize()
    for x, y in zip(got, ref):
        assert torch.equal(x, y)
    O, lse = a2d.fix([ref[0]], [ref[1]], [ref[2]], BF)
    odo = dev(synth.normal((n, 2, heads, H), 98, 1, 1.0, "bf16"))
    odo[:, 0] = O.permute(1, 0, 2)
    Ov, dOv = odo[:, 0].permute(1, 0, 2), odo[:, 1].permute(1, 0, 2)
    for handover in (False, True):
        g3 = a2d.partial_bwd(Qv, Kv, Vv, Ov, dOv, lse, 0, 0, True, scale, ds_handover=handover)
        r3 = a2d.partial_bwd(Qc, Kc, Vc, Ov.contiguous(), dOv.contiguous(), lse, 0, 0, True, scale, ds_handover=handover)
        torch.cuda.synchronize()
        for x, y in zip(g3, r3):
            assert torch.equal(x, y)


@pytest.mark.parametrize("name", ["c3", "c5"])
def test_partial_formats_accuracy_side_by_side(a2d, name):
    """The two partial formats at full size, merged over all sqrt(P) partials of a query block and
    compared with the oracle on sampled rows: the fp32 unnormalised triple (N, m, l) merged by
    a2d_fix, and the normalised pair (O' in bf16, lse') merged by a2d_fix_norm (footnote of
    Sec. 3.2).  Both merges write fp32 here, so that the figures show the formats themselves and not
    the final rounding of O.  Prints max-abs and relative-Frobenius errors side by side (the numbers
    quoted in the design notes) and holds both to the bf16 bar."""
    from helpers import max_abs, rel_fro
    w = synth.WORKLOADS[name]
    T, scale, G = w.tile, 1.0 / math.sqrt(w.hdim), w.grid
    r = G - 1 if w.causal else 0
    Qr = synth.q_block(w, r)
    Qd = dev(Qr)
    step = max(1, T // 96)
    rows = np.array(sorted(set(list(range(0, T, step)) + [T - 1])))
    hs = [0, w.heads // 2 - 1 if w.heads > 2 else w.heads - 1]
    trip, norm, ref = [], [], []
    for c in range(G):
        Kc, Vc = synth.k_block(w, c), synth.v_block(w, c)
        trip.append(a2d.partial_fwd(Qd, dev(Kc), dev(Vc), r * T, c * T, w.causal, scale))
        norm.append(a2d.partial_fwd_norm(Qd, dev(Kc), dev(Vc), r * T, c * T, w.causal, scale))
        if w.causal and c == r:
            # the diagonal block needs the rows' own offsets: one row at a time
            N = np.empty((len(hs), len(rows), w.hdim)); m = np.empty((len(hs), len(rows))); l = np.empty((len(hs), len(rows)))
            for i, row in enumerate(rows):
                a, b, c_ = oracle.partial_fwd(np64(Qr[hs][:, row:row + 1]), np64(Kc[hs]), np64(Vc[hs]), r * T + row, c * T,
                                              True, scale)
                N[:, i], m[:, i], l[:, i] = a[:, 0], b[:, 0], c_[:, 0]
            ref.append((N, m, l))
        else:
            ref.append(oracle.partial_fwd(np64(Qr[hs][:, rows]), np64(Kc[hs]), np64(Vc[hs]), 0, 0, False, scale))
    O_t, lse_t = a2d.fix([p[0] for p in trip], [p[1] for p in trip], [p[2] for p in trip], torch.float32)
    O_n, lse_n = a2d.fix_norm([p[0] for p in norm], [p[1] for p in norm], torch.float32)
    torch.cuda.synchronize()
    Or, lr = oracle.fix([t[0] for t in ref], [t[1] for t in ref], [t[2] for t in ref])
    print("\n%s: %d partials, %d sampled rows of heads %s, merged O in fp32" % (name, G, len(rows), hs))
    print("%-34s %12s %12s %12s" % ("partial format", "max|dO|", "relFro(O)", "max|dlse|"))
    res = {}
    for tag, O, lse in (("fp32 triple (N, m, l) + a2d_fix", O_t, lse_t), ("bf16 O' + lse' + a2d_fix_norm", O_n, lse_n)):
        eo, _ = max_abs(np64(O[hs][:, rows]), Or)
        el, _ = max_abs(np64(lse[hs][:, rows]), lr)
        rf = rel_fro(np64(O[hs][:, rows]), Or)
        res[tag] = (eo, rf, el)
        print("%-34s %12.3e %12.3e %12.3e" % (tag, eo, rf, el), flush=True)
        assert eo <= 2e-2 and el <= 2e-2 and rf <= 1.5e-2, (name, tag, eo, rf, el)
