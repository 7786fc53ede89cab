"""a2d_partial_bwd_static (the entry point that allocates nothing: delta lives in the library's
static device array) against a2d_partial_bwd with its minimum workspace, through the C ABI: two
calls in a row, the second on a smaller tile, bit for bit; plus the size limit."""
import ctypes
import math

import pytest
import torch

from paper_2503_15758_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def a2d():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2503_15758_amd import binding
    binding.lib()
    return binding


def _inputs(heads, nq, nkv, H, seed):
    mk = lambda shape, s: synth.normal(shape, seed, s, 1.0, "bf16").to("cuda")
    Q, dO, O = mk((heads, nq, H), 0), mk((heads, nq, H), 1), mk((heads, nq, H), 2) * 0.1
    K, V = mk((heads, nkv, H), 3), mk((heads, nkv, H), 4)
    # a finite statistic of the right size for every row (the call only needs O / lse to be given)
    lse = (synth.normal((heads, nq), seed, 5, 0.3, "f32") + math.log(nkv)).to("cuda")
    return Q, K, V, O, dO, lse


@pytest.mark.parametrize("dt_case", ["bf16_mfma", "f32_generic"])
def test_static_scratch_backward_matches_workspace_backward(a2d, dt_case):
    shapes = [(6, 700, 500, 128, True, 300, 0), (3, 130, 200, 128, True, 60, 0)]   # the second is smaller
    for i, (heads, nq, nkv, H, causal, q_off, kv_off) in enumerate(shapes):
        print("no-alloc case", dt_case, shapes[i], flush=True)
        Q, K, V, O, dO, lse = _inputs(heads, nq, nkv, H, 77 + i)
        if dt_case == "f32_generic":
            Q, K, V, O, dO = (t.float() for t in (Q, K, V, O, dO))
        scale = 1.0 / math.sqrt(H)
        ref = a2d.partial_bwd(Q, K, V, O, dO, lse, q_off, kv_off, causal, scale)
        out = tuple(torch.full_like(t, float("nan")) for t in ref)
        torch.cuda.synchronize()
        allocs = lambda: torch.cuda.memory_stats()["allocation.all.allocated"]    # allocation events so far
        before = allocs()
        got = a2d.partial_bwd_static(Q, K, V, O, dO, lse, q_off, kv_off, causal, scale, out=out)
        assert allocs() == before, "the call went through torch's allocator"
        torch.cuda.synchronize()
        for x, y, name in zip(got, ref, ("dQ", "dK", "dV")):
            assert torch.equal(x, y), "%s differs from a2d_partial_bwd (%s, call %d)" % (name, dt_case, i)


def test_static_scratch_limits(a2d):
    L = a2d.lib()
    P = ctypes.c_void_p(0x10000)                   # aligned, never dereferenced: both calls fail validation
    d = a2d.TileDesc(heads=1 << 12, nq=(1 << 8) + 1, nkv=64, hdim=128, q_off=0, kv_off=0, causal=0, scale=0.1,
                     dtype=a2d.A2D_BF16)
    assert d.heads * d.nq > a2d.STATIC_MAX_ROWS
    assert L.a2d_partial_bwd_static(ctypes.byref(d), P, P, P, P, P, P, P, P, P, None) == -4
    assert b"static scratch" in L.a2d_last_error()
    d = a2d.TileDesc(heads=2, nq=64, nkv=64, hdim=128, q_off=0, kv_off=0, causal=0, scale=0.1,
                     dtype=a2d.A2D_BF16, flags=a2d.DESC_KEEP_DS)
    assert L.a2d_partial_bwd_static(ctypes.byref(d), P, P, P, P, P, P, P, P, P, None) == -2
