"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments before anything is enqueued."""
import ctypes
import os
import subprocess
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    from paper_2503_15758_amd import binding as b
    if not os.path.exists(b.LIB_PATH):
        from paper_2503_15758_amd import build
        build.build(verbose=False)
    b.lib()
    return b


def test_header_symbols_are_exported(binding):
    text = open(os.path.join(ROOT, "include", "a2d.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(a2d_[a-z_]+)\s*\(", text))
    assert declared == set(binding.EXPORTS), declared ^ set(binding.EXPORTS)
    L = ctypes.CDLL(binding.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name
    assert binding.version() == "0.1"


def test_descriptor_layout(binding, tmp_path):
    """The ctypes mirror of a2d_tile_desc against what the C compiler makes of include/a2d.h."""
    T = binding.TileDesc
    assert ctypes.sizeof(T) == 128
    assert T.q_off.offset == 16 and T.dtype.offset == 40 and T.flags.offset == 44
    assert T.lq.offset == 48 and T.ldo.offset == 112 and ctypes.sizeof(binding.Layout) == 16
    fields = ["heads", "nq", "nkv", "hdim", "q_off", "kv_off", "causal", "scale", "dtype", "flags",
              "lq", "lk", "lv", "lo", "ldo"]
    src = tmp_path / "layout.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "a2d.h"\nint main(void) {\n'
                   '  printf("%zu", sizeof(a2d_tile_desc));\n' +
                   "".join('  printf(" %%zu", offsetof(a2d_tile_desc, %s));\n' % f for f in fields) +
                   '  printf(" %zu %zu", sizeof(a2d_kv_segment), sizeof(a2d_layout));\n  return 0;\n}\n')
    exe = tmp_path / "layout"
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    subprocess.run(["gcc", "-I", inc, str(src), "-o", str(exe)], check=True)
    got = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    want = [ctypes.sizeof(T)] + [getattr(T, f).offset for f in fields] + \
           [ctypes.sizeof(binding.KvSegment), ctypes.sizeof(binding.Layout)]
    assert got == want


def _desc(b, **kw):
    d = dict(heads=2, nq=128, nkv=128, hdim=128, q_off=0, kv_off=0, causal=0, scale=0.1, dtype=b.A2D_BF16)
    d.update(kw)
    return b.TileDesc(**d)


def test_workspace_bytes(binding):
    b = binding
    assert b.workspace_bytes(_desc(b), b.OP_PARTIAL_FWD) == 0
    assert b.workspace_bytes(_desc(b), b.OP_FIX, 8) == 0
    assert b.workspace_bytes(_desc(b), b.OP_PARTIAL_BWD) == 2 * 128 * 4
    assert b.workspace_bytes(_desc(b, heads=3, nq=5), b.OP_PARTIAL_BWD) == 256
    assert b.lib().a2d_workspace_bytes(None, b.OP_PARTIAL_BWD, 0) == 0
    # with the dS hand-over: + one 4 KiB tile per head, 32-row tile and 64-key block (bf16 MFMA path only)
    assert b.workspace_bytes(_desc(b), b.OP_PARTIAL_BWD_DS) == 2 * 128 * 4 + 2 * 4 * 2 * 4096
    assert b.workspace_bytes(_desc(b, nq=33, nkv=65), b.OP_PARTIAL_BWD_DS) == 512 + 2 * 2 * 2 * 4096
    assert b.workspace_bytes(_desc(b, dtype=b.A2D_F32), b.OP_PARTIAL_BWD_DS) == 2 * 128 * 4
    # split over the group's query heads: + 2 x min(group, 32) partial buffers of [kv heads][nkv][H] floats
    ds = b.workspace_bytes(_desc(b, heads=8), b.OP_PARTIAL_BWD_DS)
    assert b.workspace_bytes(_desc(b, heads=8), b.OP_PARTIAL_BWD_SPLIT, 2) == ds + 2 * 4 * 2 * 128 * 128 * 4
    assert b.workspace_bytes(_desc(b, heads=8), b.OP_PARTIAL_BWD_SPLIT, 8) == ds + 2 * 1 * 8 * 128 * 128 * 4
    assert b.workspace_bytes(_desc(b, heads=64), b.OP_PARTIAL_BWD_SPLIT, 1) == \
        b.workspace_bytes(_desc(b, heads=64), b.OP_PARTIAL_BWD_DS) + 2 * 32 * 1 * 128 * 128 * 4


def test_argument_errors_enqueue_nothing(binding):
    """Every call below fails validation, so no pointer is dereferenced and no kernel is launched."""
    b, L = binding, binding.lib()
    P = ctypes.c_void_p(0x10000)       # aligned, never dereferenced
    odd = ctypes.c_void_p(0x10004)
    fwd = lambda d, q=P, o=P: L.a2d_partial_fwd(ctypes.byref(d) if d else None, q, P, P, o, P, P, None, 0, None)
    assert fwd(None) == -1 and b"NULL" in L.a2d_last_error()
    assert fwd(_desc(b, hdim=72)) == -2
    assert fwd(_desc(b, dtype=7)) == -2
    assert fwd(_desc(b, nq=0)) == -1
    assert fwd(_desc(b, scale=0.0)) == -1
    assert fwd(_desc(b, scale=float("nan"))) == -1
    assert fwd(_desc(b, causal=2)) == -1
    assert fwd(_desc(b), q=None) == -1
    assert fwd(_desc(b), q=odd) == -3 and b"aligned" in L.a2d_last_error()
    assert fwd(_desc(b), o=odd) == -3
    # layouts: pad, row stride below H, misaligned strides, more than 4 GiB through one base pointer
    assert fwd(_desc(b, flags=2)) == -1 and b"flags" in L.a2d_last_error()      # an undefined flag bit
    assert fwd(_desc(b, lq=b.Layout(128 * 128, 64))) == -1 and b"layout of Q" in L.a2d_last_error()
    assert fwd(_desc(b, lk=b.Layout(0, 128))) == -1 and b"layout of K" in L.a2d_last_error()
    assert fwd(_desc(b, lv=b.Layout(-128, 256))) == -1
    assert fwd(_desc(b, lv=b.Layout(128 * 132, 132))) == -3 and b"layout of V" in L.a2d_last_error()
    assert fwd(_desc(b, lq=b.Layout(132, 256))) == -3
    assert fwd(_desc(b, dtype=b.A2D_F32, lq=b.Layout(130, 256))) == -3      # fp32: multiples of 4 elements
    assert fwd(_desc(b, lk=b.Layout(128, 1 << 25))) == -2 and b"16 MiB" in L.a2d_last_error()
    assert fwd(_desc(b, nkv=1 << 12, lk=b.Layout(128, 1 << 20))) == -2 and b"4 GiB" in L.a2d_last_error()
    # backward: workspace missing / too small
    d = _desc(b)
    bwd = lambda ws, n: L.a2d_partial_bwd(ctypes.byref(d), P, P, P, P, P, P, P, P, P, ws, n, None)
    assert bwd(None, 0) == -4
    assert bwd(P, 16) == -4 and b"1024" in L.a2d_last_error()
    # the dS hand-over is asked for by flag and then needs its full workspace: the minimum is refused,
    # and a large workspace without the flag does not select it (nothing to observe here: the call
    # would launch; the GPU tests compare the two paths)
    d = _desc(b, flags=b.DESC_KEEP_DS)
    assert bwd(P, 1024) == -4 and str(b.workspace_bytes(d, b.OP_PARTIAL_BWD_DS)).encode() in L.a2d_last_error()
    d = _desc(b)
    d = _desc(b, ldo=b.Layout(128, 120))
    assert bwd(P, 1 << 20) == -1 and b"layout of dO" in L.a2d_last_error()
    d = _desc(b, lo=b.Layout(4, 256))
    assert bwd(P, 1 << 20) == -3 and b"layout of O" in L.a2d_last_error()
    d = _desc(b)
    # fix / fix_bwd
    arr = (ctypes.c_void_p * 2)(0x10000, 0x20000)
    assert L.a2d_fix(0, 10, 128, b.A2D_BF16, arr, arr, arr, P, P, None) == -1
    assert L.a2d_fix(33, 10, 128, b.A2D_BF16, arr, arr, arr, P, P, None) == -1
    assert L.a2d_fix(2, 0, 128, b.A2D_BF16, arr, arr, arr, P, P, None) == -1
    assert L.a2d_fix(2, 10, 126, b.A2D_BF16, arr, arr, arr, P, P, None) == -2
    assert L.a2d_fix(2, 10, 128, 9, arr, arr, arr, P, P, None) == -2
    assert L.a2d_fix(2, 10, 128, b.A2D_BF16, None, arr, arr, P, P, None) == -1
    bad = (ctypes.c_void_p * 2)(0x10000, 0x20002)
    assert L.a2d_fix(2, 10, 128, b.A2D_BF16, bad, arr, arr, P, P, None) == -3
    assert L.a2d_fix_bwd(2, 10, b.A2D_BF16, arr, P, None) == -1          # n not a multiple of 4
    assert L.a2d_fix_bwd(2, 16, b.A2D_BF16, arr, None, None) == -1
    assert L.a2d_fix_bwd(40, 16, b.A2D_BF16, arr, P, None) == -1
    # the merges with a strided output
    lay = lambda h, r: ctypes.byref(b.Layout(h, r))
    assert L.a2d_fix_strided(2, 0, 10, 128, b.A2D_BF16, arr, arr, arr, P, lay(128, 256), P, None) == -1
    assert L.a2d_fix_strided(2, 2, 10, 128, b.A2D_BF16, arr, arr, arr, P, lay(128, 64), P, None) == -1
    assert L.a2d_fix_strided(2, 2, 10, 128, b.A2D_BF16, arr, arr, arr, P, lay(132, 256), P, None) == -3
    assert L.a2d_fix_strided(40, 2, 10, 128, b.A2D_BF16, arr, arr, arr, P, lay(128, 256), P, None) == -1
    assert L.a2d_fix_strided(2, 2, 10, 128, b.A2D_BF16, arr, arr, arr, None, lay(128, 256), P, None) == -1
    assert L.a2d_fix_norm_strided(2, 2, 10, 128, b.A2D_BF16, b.A2D_BF16, arr, arr, P, lay(128, 100), P, None) == -1
    assert L.a2d_fix_norm_strided(2, 2, 0, 128, b.A2D_BF16, b.A2D_BF16, arr, arr, P, lay(128, 256), P, None) == -1
    assert L.a2d_fix_norm_strided(2, 2, 10, 128, b.A2D_BF16, b.A2D_F32, arr, arr, P, lay(130, 256), P, None) == -3
    assert L.a2d_fix_bwd_strided(2, 2, 0, 128, b.A2D_BF16, arr, P, lay(128, 256), None) == -1
    assert L.a2d_fix_bwd_strided(2, 2, 10, 126, b.A2D_BF16, arr, P, lay(128, 256), None) == -2
    assert L.a2d_fix_bwd_strided(2, 2, 10, 128, b.A2D_F32, arr, P, lay(130, 256), None) == -3
    assert L.a2d_fix_bwd_strided(2, 2, 10, 128, b.A2D_BF16, arr, odd, lay(128, 256), None) == -3
    assert L.a2d_status_str(-4) == b"workspace missing or too small"
    assert L.a2d_status_str(0) == b"ok"


def test_binding_fails_loudly_without_library(binding, monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/liba2d.so")
    with pytest.raises(RuntimeError, match="liba2d.so is missing"):
        binding.lib()


def test_binding_rejects_cpu_tensors(binding):
    import torch
    x = torch.zeros(1, 4, 128, dtype=torch.bfloat16)
    with pytest.raises(binding.A2DError):
        binding.partial_fwd(x, x, x)


def test_mfma_ceiling_argument_errors(binding):
    """The diagnostic probe validates before it touches the device."""
    L = binding.lib()
    P = ctypes.c_void_p(0x10000)
    tf, mhz = ctypes.c_double(), ctypes.c_double()
    assert L.a2d_mfma_ceiling(0, 1, P, 1 << 20, ctypes.byref(tf), ctypes.byref(mhz)) == -1
    assert L.a2d_mfma_ceiling(1 << 23, 1, P, 1 << 20, ctypes.byref(tf), ctypes.byref(mhz)) == -1
    assert L.a2d_mfma_ceiling(10, 1, P, 1 << 20, None, ctypes.byref(mhz)) == -1
    assert L.a2d_mfma_ceiling(10, 1, None, 1 << 20, ctypes.byref(tf), ctypes.byref(mhz)) == -1
    assert L.a2d_mfma_ceiling(10, 1, ctypes.c_void_p(0x10004), 1 << 20, ctypes.byref(tf), ctypes.byref(mhz)) == -3


def test_gathered_tile_argument_errors(binding):
    b, L = binding, binding.lib()
    P = ctypes.c_void_p(0x10000)
    d = _desc(b, nkv=128)
    def fwd(segs, n=None):
        arr = (b.KvSegment * max(len(segs), 1))()
        for i, (o, r, pad) in enumerate(segs):
            arr[i].kv_off, arr[i].rows, arr[i].pad = o, r, pad
        return L.a2d_partial_fwd_seg(ctypes.byref(d), len(segs) if n is None else n, arr, P, P, P, P, P, P, None, 0, None)
    assert fwd([(0, 64, 0), (5, 63, 0)]) == -1 and b"128" in L.a2d_last_error()     # rows do not add up
    assert fwd([(0, 128, 0), (5, 1, 0)]) == -1
    assert fwd([(0, 0, 0), (5, 128, 0)]) == -1
    assert fwd([(0, 128, 1)]) == -1
    assert fwd([(0, 128, 0)], n=0) == -1
    assert fwd([(0, 128, 0)], n=33) == -1
    assert L.a2d_partial_fwd_seg(ctypes.byref(d), 1, None, P, P, P, P, P, P, None, 0, None) == -1
    arr = (b.KvSegment * 1)(); arr[0].kv_off, arr[0].rows = 0, 128
    assert L.a2d_partial_bwd_seg(ctypes.byref(d), 1, arr, P, P, P, P, P, P, P, P, P, None, 0, None) == -4


def test_accumulating_calls_argument_errors(binding):
    b, L = binding, binding.lib()
    P = ctypes.c_void_p(0x10000)
    d = _desc(b, nkv=128)
    arr = (b.KvSegment * 1)(); arr[0].kv_off, arr[0].rows = 0, 100
    # nseg = 0: plain tile, segs ignored; the first failing check is then the NULL output pointer
    assert L.a2d_partial_fwd_acc(ctypes.byref(d), 0, None, P, P, P, None, P, P, None, 0, None) == -1
    assert L.a2d_partial_fwd_acc(ctypes.byref(d), 1, arr, P, P, P, P, P, P, None, 0, None) == -1      # 100 != 128 keys
    assert L.a2d_partial_fwd_acc(ctypes.byref(d), -1, arr, P, P, P, P, P, P, None, 0, None) == -1
    assert L.a2d_partial_bwd_acc(ctypes.byref(d), 0, None, P, P, P, P, P, P, P, P, P, None, 0, None) == -4


def test_normalised_format_argument_errors(binding):
    b, L = binding, binding.lib()
    P = ctypes.c_void_p(0x10000)
    d = _desc(b)
    assert L.a2d_partial_fwd_norm(ctypes.byref(d), 0, None, P, P, P, None, P, None, 0, None) == -1
    assert L.a2d_partial_fwd_norm(ctypes.byref(d), 0, None, P, P, P, ctypes.c_void_p(0x10002), P, None, 0, None) == -3
    arr = (ctypes.c_void_p * 2)(0x10000, 0x20000)
    fix = lambda k, rows, h, i, o, a=arr: L.a2d_fix_norm(k, rows, h, i, o, a, arr, P, P, None)
    assert fix(0, 10, 128, b.A2D_BF16, b.A2D_BF16) == -1
    assert fix(33, 10, 128, b.A2D_BF16, b.A2D_BF16) == -1
    assert fix(2, 0, 128, b.A2D_BF16, b.A2D_BF16) == -1
    assert fix(2, 10, 126, b.A2D_BF16, b.A2D_BF16) == -2
    assert fix(2, 10, 128, 5, b.A2D_BF16) == -2
    assert fix(2, 10, 128, b.A2D_BF16, 5) == -2
    assert fix(2, 10, 128, b.A2D_BF16, b.A2D_BF16, None) == -1


def test_grouped_query_argument_errors(binding):
    b, L = binding, binding.lib()
    P = ctypes.c_void_p(0x10000)
    d = _desc(b)                      # heads as _desc sets them
    heads = d.heads
    fwd = lambda kvh, flags, o0=P, o2=P: L.a2d_partial_fwd_gqa(ctypes.byref(d), kvh, 0, None, flags, P, P, P, o0, P, o2,
                                                               None, 0, None)
    assert fwd(0, 0) == -1 and fwd(heads + 1, 0) == -1           # kv_heads must divide heads
    if heads % 3:
        assert fwd(3, 0) == -1 and b"divide" in L.a2d_last_error()
    assert fwd(heads, 4) == -1 and fwd(heads, 3) == -1            # unknown / combined flags
    assert fwd(heads, 0, None) == -1                              # NULL output
    assert fwd(1, b.TILE_NORMALISED, ctypes.c_void_p(0x10002), None) == -3
    bwd = lambda kvh, flags: L.a2d_partial_bwd_gqa(ctypes.byref(d), kvh, 0, None, flags, P, P, P, P, P, P, P, P, P,
                                                   None, 0, None)
    assert bwd(heads + 1, 0) == -1
    assert bwd(1, b.TILE_NORMALISED) == -1                        # the backward has no normalised form
    assert bwd(1, 0) == -4                                        # first failing check: the workspace
    assert bwd(1, 8) == -1 and b"flags" in L.a2d_last_error()     # an unknown flag bit
    # A2D_TILE_SPLIT_GROUPS with a workspace that only covers the dS hand-over: refused before any launch
    small = b.workspace_bytes(d, b.OP_PARTIAL_BWD_DS)
    assert L.a2d_partial_bwd_gqa(ctypes.byref(d), 1, 0, None, b.TILE_SPLIT_GROUPS, P, P, P, P, P, P, P, P, P, P,
                                 small, None) == -4
    assert b"SPLIT_GROUPS" in L.a2d_last_error()
    assert L.a2d_partial_bwd_gqa(ctypes.byref(d), 1, 0, None, 0, P, P, P, P, P, P, P, P, P, P, 1 << 50, None) == -1
    assert b"plausible" in L.a2d_last_error()                    # a size no allocation can have
    big = _desc(b, nq=1 << 22)
    big.heads = 4
    assert L.a2d_partial_fwd_gqa(ctypes.byref(big), 2, 0, None, 0, P, P, P, P, P, P, None, 0, None) == -1
    assert b"2^22" in L.a2d_last_error()
    too = _desc(b, nq=(1 << 22) + 1)
    assert L.a2d_partial_fwd(ctypes.byref(too), P, P, P, P, P, P, None, 0, None) == -1


def test_every_export_has_typed_arguments(binding):
    """ctypes passes an untyped Python int as a 32-bit C int; as a stack argument that leaves the
    upper half of a size_t parameter (a workspace size) undefined.  Every export must therefore
    declare its argument and result types, with as many arguments as the header's prototype."""
    import re
    L = binding.lib()
    header = open(os.path.join(ROOT, "include", "a2d.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    for name in binding.EXPORTS:
        fn = getattr(L, name)
        assert fn.argtypes is not None, name + ": argtypes not declared in the binding"
        assert fn.restype is not ctypes.c_int or name.startswith("a2d_"), name
        m = re.search(r"\b%s\s*\(([^;]*?)\)\s*;" % name, header, flags=re.S)
        assert m, name + ": prototype not found in include/a2d.h"
        params = m.group(1).strip()
        n = 0 if params in ("", "void") else params.count(",") + 1
        assert len(fn.argtypes) == n, "%s: %d argument types declared, the header has %d" % (name, len(fn.argtypes), n)
        # sizes travel as size_t, row counts as int64
        for i, p_ in enumerate(x.strip() for x in params.split(",")) if n else []:
            if p_.startswith("size_t"):
                assert fn.argtypes[i] is ctypes.c_size_t, "%s: argument %d must be c_size_t" % (name, i)
            if p_.startswith("int64_t"):
                assert fn.argtypes[i] is ctypes.c_int64, "%s: argument %d must be c_int64" % (name, i)


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stderr + r.stdout)
