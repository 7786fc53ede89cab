#!/usr/bin/env python3
"""Benchmark of the Attention2D per-device hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic tiles of the chosen
workload (default: the GPT-3-like causal workload, 4096 x 4096 x H128 tiles, 96 heads):
  partial_fwd (diagonal tile) + partial_fwd (unmasked tile)  ->  fix over the sqrt(P) partials
  ->  partial_bwd of both tiles  ->  fix_bwd for dQ (grid row) and dK, dV (grid column).
All inputs are resident in HBM before the timed region.  Prints ONE JSON line.

  value            = algorithmic tile FLOPs of the step / wall time of the step (TFLOP/s)
  roofline         = the dominant kernel (the longest single launch of the step: the dK/dV kernel of the
                     unmasked backward tile) against the roofline that bounds it, its duration measured with
                     HIP events the library records on the launch stream around every kernel, inside the
                     timed region (a2d_debug_trace); traffic = HBM bytes per launch from profiles/
  per_kernel       = the same object for every kernel of the step (MFMA kernels against the bf16 MFMA peak,
                     streaming kernels and the dQ-from-dS kernel against the HBM peak)
  kernels          = per call of the step (a backward call = delta + dK/dV + dQ kernels)
  cpu_baseline     = the fp64 oracle timed on the host cores on a bounded sample
  mfma_ceiling     = what the bf16 MFMA units sustain on their own on this chip (diagnostic probe of the
                     library: register operands, no other work), with random and with constant operands,
                     and the shader clock during each; context for the roofline fraction, not its peak
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E


def tile_flops(w, nq, nkv, causal_diag):
    """Algorithmic FLOPs of one tile, all heads: fwd 4 Nq Nkv H, bwd 10 Nq Nkv H per head; a
    diagonal causal tile counts its visible fraction (T + 1) / (2 T)."""
    frac = (nq + 1) / (2.0 * nq) if causal_diag else 1.0
    base = w.heads * nq * nkv * w.hdim * frac
    return 4.0 * base, 10.0 * base


def call_kernels(call, w, recompute):
    """The library kernels one call of the step launches, in launch order."""
    if call.startswith("partial_fwd"):
        return ["fwd_mfma_kernel" if w.dtype == "bf16" else "fwd_generic_kernel"]
    if call.startswith("partial_bwd"):
        if w.dtype != "bf16":
            return ["delta_kernel", "bwd_dkdv_generic_kernel", "bwd_dq_generic_kernel"]
        return ["delta_kernel", "bwd_dkdv_kernel", "bwd_dq_kernel" if recompute else "bwd_dq_ds_kernel"]
    if call == "fix":
        return ["fix_kernel"]
    if call.startswith("fix_bwd"):
        return ["sum_kernel"]
    if call == "copy_probe":
        return ["copy_probe_kernel"]
    raise KeyError(call)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3", choices=["c2", "c3", "c4", "c5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-mfma-probe", action="store_true")
    ap.add_argument("--no-gathered", action="store_true",
                    help="skip the extra measurements appended after the timed steps (gathered key row, "
                         "normalised partials, grouped-query heads, small and rectangular tiles)")
    ap.add_argument("--no-extras", action="store_true", help="--no-gathered and --no-mfma-probe together")
    ap.add_argument("--recompute-bwd", action="store_true",
                    help="do not set A2D_DESC_KEEP_DS: the dQ kernel then recomputes S and dP instead of reading "
                         "the dS the dK/dV kernel left in the (larger) workspace")
    ap.add_argument("--grid-emulation", action="store_true",
                    help="also time Alg. 1 + Alg. 3 over all P tiles of the c2 sequence (8192 tokens, 4 x 4 grid)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="after the timed steps launch the library's plain copy kernel once on 1 GiB, so that a "
                         "rocprofv3 --pmc run of this command also holds the counter reading of a copy of "
                         "known size (the scale factor for FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--launch-log", default=None,
                    help="write, as JSON, which call every library kernel launch of this process belongs to, in "
                         "launch order (paper_2503_15758_amd.rocprof_summary matches profiler rows against it)")
    args = ap.parse_args()
    if args.no_extras:
        args.no_gathered = args.no_mfma_probe = True
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the sqrt(P) x sqrt(P) grid is emulated as "
                 "independent tiles on one device); --gpus %d is not supported" % args.gpus)

    import torch
    from paper_2503_15758_amd import binding as a2d, synth, rocprof_summary

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    a2d.lib()
    w = synth.WORKLOADS[args.workload]
    T, G, H = w.tile, w.grid, w.hdim
    scale = 1.0 / math.sqrt(H)
    dt = synth.torch_dtype(w.dtype)
    r = G - 1                                   # the query block with every partial non-empty
    # tiles of the step: (key block c, is_diagonal)
    tiles = [(r, True), (0, False)] if w.causal else [(0, False)]
    launch_log = []                             # (kernel, call, phase) of every library launch, in order

    def log_call(call, phase):
        for k in call_kernels(call, w, args.recompute_bwd):
            launch_log.append({"kernel": k, "call": call, "phase": phase})

    dev = lambda t: t.to("cuda")
    Q = dev(synth.q_block(w, r))
    dO = dev(synth.do_block(w, r)) if w.backward else None
    Kc = {c: dev(synth.k_block(w, c)) for c, _ in tiles}
    Vc = {c: dev(synth.v_block(w, c)) for c, _ in tiles}

    f32 = dict(dtype=torch.float32, device="cuda")
    # sqrt(P) partial triples of the query block; the tiles of the step are recomputed every step,
    # the others are produced once here (same kernels, other key blocks)
    parts = [(torch.empty(w.heads, T, H, **f32), torch.empty(w.heads, T, **f32),
              torch.empty(w.heads, T, **f32)) for _ in range(G)]
    timed_cols = {c for c, _ in tiles}
    for c in range(G):
        if c not in timed_cols:
            a2d.partial_fwd(Q, dev(synth.k_block(w, c)), dev(synth.v_block(w, c)), r * T, c * T, w.causal,
                            scale, out=parts[c])
            log_call("partial_fwd_full", "setup")
    O = torch.empty(w.heads, T, H, dtype=dt, device="cuda")
    lse = torch.empty(w.heads, T, **f32)
    if w.backward:
        # with the dS hand-over (A2D_DESC_KEEP_DS) the workspace holds delta + dS: 2 T^2 bytes per head more
        ws_op = a2d.OP_PARTIAL_BWD if args.recompute_bwd else a2d.OP_PARTIAL_BWD_DS
        ws = torch.empty(a2d.workspace_bytes(a2d.tile_desc(Q, Kc[tiles[0][0]], 0, 0, w.causal, scale), ws_op),
                         dtype=torch.uint8, device="cuda")
        # gradient partials: dQ over the grid row (one per key block), dK / dV over the grid column
        dq_parts = [torch.zeros(w.heads, T, H, **f32) for _ in range(G)]
        dk_parts = [torch.zeros(w.heads, T, H, **f32) for _ in range(G)]
        dv_parts = [torch.zeros(w.heads, T, H, **f32) for _ in range(G)]
        for x in range(G):   # untimed partials hold plausible values
            dq_parts[x].normal_(); dk_parts[x].normal_(); dv_parts[x].normal_()
        dQ = torch.empty(w.heads, T, H, dtype=dt, device="cuda")
        dK = torch.empty(w.heads, T, H, dtype=dt, device="cuda")
        dV = torch.empty(w.heads, T, H, dtype=dt, device="cuda")
    torch.cuda.synchronize()

    calls = []      # (name, fn)
    for i, (c, diag) in enumerate(tiles):
        tag = "diag" if diag else "full"
        calls.append(("partial_fwd_" + tag, lambda c=c: a2d.partial_fwd(
            Q, Kc[c], Vc[c], r * T, c * T, w.causal, scale, out=parts[c])))
    calls.append(("fix", lambda: a2d.fix([p[0] for p in parts], [p[1] for p in parts],
                                         [p[2] for p in parts], out=(O, lse))))
    if w.backward:
        for i, (c, diag) in enumerate(tiles):
            tag = "diag" if diag else "full"
            calls.append(("partial_bwd_" + tag, lambda c=c, i=i: a2d.partial_bwd(
                Q, Kc[c], Vc[c], O, dO, lse, r * T, c * T, w.causal, scale,
                out=(dq_parts[c], dk_parts[i], dv_parts[i]), workspace=ws, ds_handover=not args.recompute_bwd)))
        calls.append(("fix_bwd_dq", lambda: a2d.fix_bwd(dq_parts, out=dQ)))
        calls.append(("fix_bwd_dk", lambda: a2d.fix_bwd(dk_parts, out=dK)))
        calls.append(("fix_bwd_dv", lambda: a2d.fix_bwd(dv_parts, out=dV)))
    names = [n for n, _ in calls]
    kernel_seq = [(n, k) for n in names for k in call_kernels(n, w, args.recompute_bwd)]   # launches of one step
    events_per_step = len(kernel_seq) + len(calls)          # one event before every call, one after every kernel

    def step(phase=None):
        for name, fn in calls:
            fn()
            if phase:
                log_call(name, phase)

    for _ in range(args.warmup):
        step(phase="warmup")
    torch.cuda.synchronize()
    # per-kernel times: HIP events recorded by the library on the launch stream, one before every call
    # and one after every kernel (the only events inside the timed region)
    trace = a2d.KernelTrace(args.steps * events_per_step)
    torch.cuda.synchronize()
    with trace:
        t0 = time.perf_counter()
        for s in range(args.steps):
            step(phase="timed")
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    assert trace.count == args.steps * events_per_step, (trace.count, args.steps, events_per_step)
    iv = trace.intervals_ms()
    trace.close()
    kern_ms = {}                                # (call, kernel) -> average duration over the timed steps
    for s in range(args.steps):
        pos = s * events_per_step               # index of the call's "before" event
        for name in names:
            for k in call_kernels(name, w, args.recompute_bwd):
                kern_ms[(name, k)] = kern_ms.get((name, k), 0.0) + iv[pos] / args.steps
                pos += 1
            pos += 1
    if args.copy_probe:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        a2d.copy_probe(dst, src)
        log_call("copy_probe", "probe")
        torch.cuda.synchronize()
        del src, dst
    if args.launch_log:
        with open(args.launch_log, "w") as f:
            json.dump(launch_log, f)

    # a call's time: from the event before it to the event after its last kernel
    avg_ms = {n: sum(kern_ms[(n, k)] for k in call_kernels(n, w, args.recompute_bwd)) for n in names}

    # ---- algorithmic work of each call and of each kernel
    esz = 2 if w.dtype == "bf16" else 4
    rows = w.heads * T
    flops, bytes_ = {}, {}
    kflops, kbytes, knote = {}, {}, {}
    for c, diag in tiles:
        tag = "diag" if diag else "full"
        f, b = tile_flops(w, T, T, diag)
        vis = (T + 1) / (2.0 * T) if diag else 1.0
        flops["partial_fwd_" + tag] = f
        kflops[("partial_fwd_" + tag, call_kernels("partial_fwd_" + tag, w, False)[0])] = f
        if w.backward:
            n = "partial_bwd_" + tag
            flops[n] = b
            ks = call_kernels(n, w, args.recompute_bwd)
            kbytes[(n, ks[0])] = rows * (2 * H * esz + 4)
            kflops[(n, ks[1])] = 0.8 * b                      # four of the five counted contractions: S, dP, dV, dK
            if ks[2] == "bwd_dq_ds_kernel":
                # one contraction over the stored dS: dS (2 bytes per visible score) + K read, dQ written
                kbytes[(n, ks[2])] = w.heads * (2.0 * T * T * vis + T * H * esz + T * H * 4)
                knote[(n, ks[2])] = "bytes = dS read back (2 per visible score) + K + the fp32 dQ partial; " \
                                    "mfma_frac = its one contraction against the MFMA peak"
            kflops[(n, ks[2])] = 0.2 * b                      # dQ = scale dS K (recomputation of S and dP not counted)
    bytes_["fix"] = rows * (G * (H + 2) * 4 + H * esz + 4)
    kbytes[("fix", "fix_kernel")] = bytes_["fix"]
    if w.backward:
        for n in ("fix_bwd_dq", "fix_bwd_dk", "fix_bwd_dv"):
            bytes_[n] = rows * (G * H * 4 + H * esz)
            kbytes[(n, "sum_kernel")] = bytes_[n]
    total_flops = sum(flops.values())
    value = total_flops / (ms_per_step * 1e-3) / 1e12

    traffic_name = w.name + ("_recompute" if args.recompute_bwd else "")
    traffic, traffic_sha = rocprof_summary.read_traffic(traffic_name)
    src_sha = rocprof_summary.source_hash()

    def entry(ms, fl=None, by=None, note=None):
        if by is not None and (fl is None or note):           # HBM-bound
            ach = by / (ms * 1e-3) / 1e9
            e = {"avg_ms": round(ms, 4), "bound": "hbm", "achieved": round(ach, 1), "unit": "GB/s",
                 "frac": round(ach / PEAK_HBM_GBS, 4), "peak": PEAK_HBM_GBS}
            if fl is not None:
                e["mfma_frac"] = round(fl / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)
        else:
            ach = fl / (ms * 1e-3) / 1e12
            e = {"avg_ms": round(ms, 4), "bound": "mfma", "achieved": round(ach, 2), "unit": "TFLOP/s",
                 "frac": round(ach / PEAK_BF16_TFLOPS, 4), "peak": PEAK_BF16_TFLOPS}
        if note:
            e["note"] = note
        return e

    kernels = {n: entry(avg_ms[n], flops.get(n), bytes_.get(n)) for n in names}
    per_kernel = {}
    for (n, k), ms in kern_ms.items():
        e = entry(ms, kflops.get((n, k)), kbytes.get((n, k)), knote.get((n, k)))
        e["traffic"] = traffic.get("%s/%s" % (n, k))
        per_kernel["%s/%s" % (n, k)] = e
    for n in names:
        kernels[n]["traffic"] = traffic.get(n)
    # the dominant kernel: the longest single launch of the step
    dom = max(kern_ms, key=lambda nk: kern_ms[nk])
    de = per_kernel["%s/%s" % dom]
    roofline = {"kernel": dom[1], "call": dom[0], "bound": de["bound"], "achieved": de["achieved"], "peak": de["peak"],
                "unit": de["unit"], "frac": de["frac"], "avg_ms": de["avg_ms"], "traffic": de["traffic"],
                "algorithmic": ("4 of the call's 5 counted contractions (S, dP, dV, dK): 8 Nq Nkv H per head"
                                if dom[1] == "bwd_dkdv_kernel" else "the call's counted work"),
                "traffic_source": {"file": "profiles/%s_hbm_traffic.txt" % traffic_name if traffic else None,
                                   "measured_on_sources": traffic_sha, "current_sources": src_sha,
                                   "current": bool(traffic) and traffic_sha == src_sha}}
    if w.backward:
        roofline["bwd_path"] = "recompute" if args.recompute_bwd else "dS hand-over"
        # the call's inputs and outputs read / written once (Q, K, V, O, dO in the model's dtype, three fp32
        # gradient partials, lse): what the call's `traffic` is to be held against.  The dS hand-over adds 2
        # bytes per visible score written and read back (an intermediate traded for two contractions).
        roofline["call_algorithmic_bytes"] = w.heads * (5 * T * H * esz + 3 * T * H * 4 + T * 4)
        roofline["call_traffic"] = traffic.get(dom[0])

    result = {
        "metric": "fwd+bwd attention TFLOP/s per tile + % bf16 MFMA peak; AttnFix GB/s",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": "%s: %s tiles %dx%dxH%d, %d heads, sqrtP=%d, %s" % (
            w.name, "causal" if w.causal else "non-causal", T, T, H, w.heads, G,
            "fwd+bwd" if w.backward else "fwd only"),
            "tiles_per_step": [("diagonal" if d else "unmasked") for _, d in tiles], "fix_k": G},
        "frac_bf16_peak": round(value / PEAK_BF16_TFLOPS, 4),
        "attnfix_gbs": kernels["fix"]["achieved"], "attnfix_frac_hbm": kernels["fix"]["frac"],
        "roofline": roofline, "kernels": kernels, "per_kernel": per_kernel,
    }
    # ---- extra measurements after the timed steps; none of them may cost the line above
    def extra(key, fn):
        try:
            result[key] = fn()
        except Exception as e:                       # report and go on
            result[key] = {"error": "%s: %s" % (type(e).__name__, str(e)[:200])}

    def graph_step():
        # the same step replayed from a HIP graph (the calls only enqueue kernels, so a step captures as is)
        side_g = torch.cuda.Stream()
        side_g.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side_g):
            step()
        torch.cuda.current_stream().wait_stream(side_g)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side_g):
            step()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        msg = (time.perf_counter() - t0) * 1e3 / args.steps
        return {"ms_per_step": round(msg, 4), "tflops": round(total_flops / (msg * 1e-3) / 1e12, 2),
                "launches_per_step": len(calls) + (2 * len(tiles) if w.backward else 0),
                "what": "the timed step captured once into a HIP graph and replayed"}

    def plain_step():
        # the same eager step with nothing between the calls: no per-call events, no kernel trace
        # (they cost a short step more than a long one: every event is a packet of its own in the queue)
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        msp = (time.perf_counter() - t0) * 1e3 / args.steps
        return {"ms_per_step": round(msp, 4), "tflops": round(total_flops / (msp * 1e-3) / 1e12, 2),
                "what": "the timed step, eager, without the per-call events and the kernel trace of the timed region"}

    def two_stream_step():
        # the same step with the two backward tile calls on two streams (their own workspaces): the
        # HBM-bound dQ-from-dS kernel of one tile then runs beside the MFMA-bound dK/dV kernel of the other
        side = torch.cuda.Stream()
        ws2 = torch.empty_like(ws)
        fork, join = torch.cuda.Event(), torch.cuda.Event()
        (c_a, _), (c_b, _) = tiles

        def step_two_streams():
            for name, fn in calls:
                if name.startswith("partial_bwd_") and name.endswith("full"):
                    fork.record()
                    side.wait_event(fork)
                    with torch.cuda.stream(side):
                        a2d.partial_bwd(Q, Kc[c_b], Vc[c_b], O, dO, lse, r * T, c_b * T, w.causal, scale,
                                        out=(dq_parts[c_b], dk_parts[1], dv_parts[1]), workspace=ws2,
                                        ds_handover=not args.recompute_bwd)
                        join.record()
                elif name == "fix_bwd_dq":
                    torch.cuda.current_stream().wait_event(join)
                    fn()
                else:
                    fn()

        for _ in range(args.warmup):
            step_two_streams()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step_two_streams()
        torch.cuda.synchronize()
        ms2 = (time.perf_counter() - t0) * 1e3 / args.steps
        return {"ms_per_step": round(ms2, 4), "tflops": round(total_flops / (ms2 * 1e-3) / 1e12, 2),
                "what": "the timed step with its two backward tile calls on two streams"}

    def mfma_ceiling():
        tf_r, mhz_r = a2d.mfma_ceiling(20000, True)
        tf_c, mhz_c = a2d.mfma_ceiling(20000, False)
        tf_m, mhz_m = a2d.forward_mix_ceiling(6000)
        tf_b, mhz_b = a2d.backward_mix_ceiling(6000)
        without = {name: round(a2d.backward_mix_ceiling(6000, bits)[0], 1)
                   for name, bits in (("mailbox", a2d.LEAVE_MAILBOX), ("arithmetic", a2d.LEAVE_ARITHMETIC),
                                      ("mailbox_barrier", a2d.LEAVE_MAILBOX | a2d.LEAVE_BARRIER),
                                      ("mailbox_barrier_arithmetic", 7))}
        lds_n, lds_t = a2d.lds_read_ceiling(20000, False)[0], a2d.lds_read_ceiling(20000, True)[0]
        return {"random_operands": {"tflops": round(tf_r, 1), "shader_mhz": round(mhz_r)},
                "constant_operands": {"tflops": round(tf_c, 1), "shader_mhz": round(mhz_c)},
                "forward_loop_model": {"tflops": round(tf_m, 1), "shader_mhz": round(mhz_m),
                                       "what": "MFMA + one LDS fragment + softmax arithmetic per MFMA, random operands, "
                                               "nothing else of the kernel"},
                "dkdv_loop_model": {"tflops": round(tf_b, 1), "shader_mhz": round(mhz_b),
                                    "what": "paired score / gradient wavefronts, natural and transposing LDS fragments, "
                                            "fp32 mailbox, one barrier per 32-row step, random operands, nothing else "
                                            "of the kernel",
                                    "tflops_without": without},
                "lds_read_tbytes_per_s": {"b128": round(lds_n, 1), "b64_transposing": round(lds_t, 1),
                                          "what": "eight wavefronts per compute unit that only read LDS"},
                "unit": "TFLOP/s", "kind": "MFMA-only probe, register operands"}

    if not args.no_gathered:
        extra("plain_step", plain_step)
        extra("hip_graph_step", graph_step)
        if w.backward and len(tiles) == 2:
            extra("two_stream_step", two_stream_step)
        if w.name == "c3":
            if w.causal:
                extra("gathered", lambda: gathered_tile(a2d, synth, w, scale, kernels))
            extra("normalised_partials", lambda: normalised_format(a2d, synth, w, scale, kernels))
            extra("attnfix_hops", lambda: attnfix_hops(a2d, w))
            extra("grouped_query", lambda: grouped_query(a2d, synth, w, scale, kernels))
            extra("strided_inputs", lambda: strided_inputs(a2d, synth, w, scale, kernels))
            extra("rectangular_tiles", lambda: rectangular_tiles(a2d, synth, w, scale))
            extra("small_tiles", lambda: small_tiles(a2d, synth))
    if args.grid_emulation:
        extra("grid_emulation", lambda: grid_emulation(synth))
    if not args.no_mfma_probe:
        extra("mfma_ceiling", mfma_ceiling)
        ceil = result.get("mfma_ceiling", {}).get("random_operands", {}).get("tflops")
        if ceil:   # context: the same kernel against what the MFMA units sustain on random operands on this chip
            result["roofline"]["frac_of_random_operand_mfma_rate"] = round(roofline["achieved"] / ceil, 4)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, scale)
    print(json.dumps(result))


def gathered_tile(a2d, synth, w, scale, kernels):
    """The last query block against ALL sqrt(P) key/value blocks in ONE launch (a2d_partial_fwd_seg /
    a2d_partial_bwd_seg: the step-like causal mask of a gathered K_g, V_g), timed beside what the same
    work costs as one launch per key block (sqrt(P) - 1 unmasked tiles + the diagonal one, from the
    per-call times above) plus, forward, the merge of their partials."""
    import torch
    T, G, H = w.tile, w.grid, w.hdim
    r = G - 1
    dev = lambda t: t.to("cuda")
    Q = dev(synth.q_block(w, r))
    dO = dev(synth.do_block(w, r))
    K = torch.cat([dev(synth.k_block(w, c)) for c in range(G)], dim=1)
    V = torch.cat([dev(synth.v_block(w, c)) for c in range(G)], dim=1)
    segs = [(c * T, T) for c in range(G)]
    out = a2d.partial_fwd(Q, K, V, r * T, 0, True, scale, segments=segs)
    O, lse = a2d.fix([out[0]], [out[1]], [out[2]])
    o3 = a2d.partial_bwd(Q, K, V, O, dO, lse, r * T, 0, True, scale, segments=segs)
    # the workspace size that selects the dS hand-over, as in the timed steps (2 bytes per score: 24 GiB here)
    ws = torch.empty(a2d.workspace_bytes(a2d.tile_desc(Q, K, r * T, 0, True, scale), a2d.OP_PARTIAL_BWD_DS),
                     dtype=torch.uint8, device="cuda")

    def timeit(fn, n=5):
        fn(); fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(3):      # median of three loops: the first one after an idle stretch runs at lower clocks
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) / n)
        return sorted(ts)[1]

    t_f = timeit(lambda: a2d.partial_fwd(Q, K, V, r * T, 0, True, scale, out=out, segments=segs))
    t_b = timeit(lambda: a2d.partial_bwd(Q, K, V, O, dO, lse, r * T, 0, True, scale, out=o3, workspace=ws,
                                         segments=segs, ds_handover=True))
    # accumulating form on one unmasked tile: starts from the triple in `acc` and merges in place
    K0, V0 = dev(synth.k_block(w, 0)), dev(synth.v_block(w, 0))
    acc = a2d.partial_fwd(Q, dev(synth.k_block(w, 1)), dev(synth.v_block(w, 1)), r * T, T, True, scale)
    plain = a2d.partial_fwd(Q, K0, V0, r * T, 0, True, scale)
    t_plain = timeit(lambda: a2d.partial_fwd(Q, K0, V0, r * T, 0, True, scale, out=plain), n=10)
    t_acc = timeit(lambda: a2d.partial_fwd(Q, K0, V0, r * T, 0, True, scale, out=acc, accumulate=True), n=10)
    frac = (G - 1) + (T + 1) / (2.0 * T)                      # visible tiles of the row
    base = w.heads * T * T * H * frac
    sep_f = (G - 1) * kernels["partial_fwd_full"]["avg_ms"] + kernels["partial_fwd_diag"]["avg_ms"] + \
        kernels["fix"]["avg_ms"]
    sep_b = (G - 1) * kernels["partial_bwd_full"]["avg_ms"] + kernels["partial_bwd_diag"]["avg_ms"]
    return {"what": "query block %d against all %d key/value blocks in one launch" % (r, G),
            "fwd_ms": round(t_f, 4), "fwd_tflops": round(4 * base / t_f / 1e9, 1),
            "bwd_ms": round(t_b, 4), "bwd_tflops": round(10 * base / t_b / 1e9, 1),
            "fwd_ms_one_launch_per_block_plus_fix": round(sep_f, 4),
            "bwd_ms_one_launch_per_block": round(sep_b, 4),
            "fwd_acc_unmasked_tile_ms": round(t_acc, 4), "fwd_plain_unmasked_tile_ms": round(t_plain, 4),
            "fwd_acc_note": "a2d_partial_fwd_acc (merges into an existing triple) and a2d_partial_fwd on the same "
                            "unmasked tile, timed back to back"}


def normalised_format(a2d, synth, w, scale, kernels):
    """The bf16 normalised partial format (a2d_partial_fwd_norm / a2d_fix_norm): the merge of the
    sqrt(P) partials of a query block moves half the bytes of the fp32 unnormalised format."""
    import torch
    T, G, H = w.tile, w.grid, w.hdim
    r = G - 1
    dev = lambda t: t.to("cuda")
    Q = dev(synth.q_block(w, r))
    parts = []
    for c in range(G):
        parts.append(a2d.partial_fwd_norm(Q, dev(synth.k_block(w, c)), dev(synth.v_block(w, c)), r * T, c * T,
                                          True, scale))
    K0, V0 = dev(synth.k_block(w, 0)), dev(synth.v_block(w, 0))
    O = torch.empty(w.heads, T, H, dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(w.heads, T, dtype=torch.float32, device="cuda")

    def timeit(fn, n=20):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(3):      # median of three loops: the first one after an idle stretch runs at lower clocks
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) / n)
        return sorted(ts)[1]

    t_fix = timeit(lambda: a2d.fix_norm([p[0] for p in parts], [p[1] for p in parts], out=(O, lse)))
    t_fwd = timeit(lambda: a2d.partial_fwd_norm(Q, K0, V0, r * T, 0, True, scale, out=parts[0]), n=10)
    rows = w.heads * T
    nbytes = rows * (G * (H * 2 + 4) + H * 2 + 4)
    return {"fix_norm_ms": round(t_fix, 4), "fix_norm_gbs": round(nbytes / t_fix / 1e6, 1),
            "fix_norm_frac_hbm": round(nbytes / t_fix / 1e6 / PEAK_HBM_GBS, 4), "fix_norm_bytes": nbytes,
            "fix_fp32_ms": kernels["fix"]["avg_ms"], "partial_fwd_norm_unmasked_tile_ms": round(t_fwd, 4)}


def attnfix_hops(a2d, w):
    """a2d_attnfix on its own: one hop of a pairwise reduce-scatter (two partials of a query block
    merged into one, still unnormalised) and the whole k-way merge left unnormalised."""
    import torch
    T, G, H = w.tile, w.grid, w.hdim
    gen = torch.Generator(device="cuda"); gen.manual_seed(5)
    f32 = dict(dtype=torch.float32, device="cuda")
    Ns = [torch.randn(w.heads, T, H, generator=gen, **f32) for _ in range(G)]
    ms = [torch.randn(w.heads, T, generator=gen, **f32) for _ in range(G)]
    ls = [torch.rand(w.heads, T, generator=gen, **f32) + 1.0 for _ in range(G)]
    out = a2d.attnfix(Ns[:2], ms[:2], ls[:2])
    rows = w.heads * T
    t2 = _timeit(torch, lambda: a2d.attnfix(Ns[:2], ms[:2], ls[:2], out=out), n=20)
    tk = _timeit(torch, lambda: a2d.attnfix(Ns, ms, ls, out=out), n=20)
    b2, bk = rows * 3 * (H + 2) * 4, rows * (G + 1) * (H + 2) * 4
    return {"what": "two partials -> one (a hop of the reduce-scatter of Alg. 1 line 5), and all %d -> one" % G,
            "pair_ms": round(t2, 4), "pair_gbs": round(b2 / t2 / 1e6, 1), "pair_frac_hbm": round(b2 / t2 / 1e6 / PEAK_HBM_GBS, 4),
            "kway_ms": round(tk, 4), "kway_gbs": round(bk / tk / 1e6, 1), "kway_frac_hbm": round(bk / tk / 1e6 / PEAK_HBM_GBS, 4)}


def strided_inputs(a2d, synth, w, scale, kernels):
    """The unmasked tile with Q, K, V read in place from a [rows][3][heads][H] buffer (a fused QKV
    projection) and O, dO from [rows][heads][H] ones, through the descriptor's strides, timed beside
    the plain-layout tile of the timed steps."""
    import torch
    if not w.backward:
        return None
    T, H, r = w.tile, w.hdim, w.grid - 1
    dev = lambda t: t.to("cuda")
    packed = torch.stack([dev(synth.q_block(w, r)), dev(synth.k_block(w, 0)), dev(synth.v_block(w, 0))], 0)
    packed = packed.permute(2, 0, 1, 3).contiguous()                 # [rows][3][heads][H]
    Q, K0, V0 = (packed[:, i].permute(1, 0, 2) for i in range(3))    # [heads][rows][H] views
    dO = dev(synth.do_block(w, r)).permute(1, 0, 2).contiguous().permute(1, 0, 2)
    out = a2d.partial_fwd(Q, K0, V0, r * T, 0, True, scale)
    O, lse = a2d.fix([out[0]], [out[1]], [out[2]])
    O = O.permute(1, 0, 2).contiguous().permute(1, 0, 2)
    o3 = tuple(torch.empty(w.heads, T, H, dtype=torch.float32, device="cuda") for _ in range(3))
    ws = torch.empty(a2d.workspace_bytes(a2d.tile_desc(Q, K0, r * T, 0, True, scale), a2d.OP_PARTIAL_BWD_DS),
                     dtype=torch.uint8, device="cuda")

    def timeit(fn, n=10):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(3):      # median of three loops: the first one after an idle stretch runs at lower clocks
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) / n)
        return sorted(ts)[1]

    Qc, Kc, Vc, Oc, dOc = (t.contiguous() for t in (Q, K0, V0, O, dO))     # plain copies, timed the same way
    # alternating, median of three: the first loop after an idle stretch runs at lower clocks
    med = lambda v: sorted(v)[len(v) // 2]
    tf, pf, tb, pb = [], [], [], []
    for _ in range(3):
        tf.append(timeit(lambda: a2d.partial_fwd(Q, K0, V0, r * T, 0, True, scale, out=out)))
        pf.append(timeit(lambda: a2d.partial_fwd(Qc, Kc, Vc, r * T, 0, True, scale, out=out)))
    for _ in range(3):
        tb.append(timeit(lambda: a2d.partial_bwd(Q, K0, V0, O, dO, lse, r * T, 0, True, scale, out=o3, workspace=ws, ds_handover=True)))
        pb.append(timeit(lambda: a2d.partial_bwd(Qc, Kc, Vc, Oc, dOc, lse, r * T, 0, True, scale, out=o3, workspace=ws,
                                                 ds_handover=True)))
    t_f, p_f, t_b, p_b = med(tf), med(pf), med(tb), med(pb)
    return {"what": "unmasked tile, Q / K / V views of one [rows][3][heads][H] buffer, O / dO [rows][heads][H]; "
                    "plain_*: the same calls on plain copies, alternating, medians of three",
            "row_stride_bytes": int(Q.stride(1) * Q.element_size()), "fwd_ms": round(t_f, 4), "bwd_ms": round(t_b, 4),
            "plain_fwd_ms": round(p_f, 4), "plain_bwd_ms": round(p_b, 4)}


def grouped_query(a2d, synth, w, scale, kernels):
    """The unmasked tile with grouped-query heads (a2d_partial_fwd_gqa / a2d_partial_bwd_gqa): the
    workload's query heads against 8 and against heads / 8 key/value heads, timed beside the
    multi-head tile."""
    import torch
    T, H, r = w.tile, w.hdim, w.grid - 1
    dev = lambda t: t.to("cuda")
    Q, dO = dev(synth.q_block(w, r)), dev(synth.do_block(w, r))
    K0, V0 = dev(synth.k_block(w, 0)), dev(synth.v_block(w, 0))
    # the workspace size that selects the dS hand-over, as in the timed steps
    ws = torch.empty(a2d.workspace_bytes(a2d.tile_desc(Q, K0, r * T, 0, True, scale), a2d.OP_PARTIAL_BWD_DS),
                     dtype=torch.uint8, device="cuda")

    def timeit(fn, n=10):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(3):      # median of three loops: the first one after an idle stretch runs at lower clocks
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) / n)
        return sorted(ts)[1]

    f_fl, b_fl = tile_flops(w, T, T, False)
    res = {"what": "%d query heads, unmasked tile, key/value heads as listed" % w.heads,
           "multi_head_fwd_ms": kernels["partial_fwd_full"]["avg_ms"],
           "multi_head_bwd_ms": kernels["partial_bwd_full"]["avg_ms"], "cases": []}
    for kvh in sorted({8, w.heads // 8}):
        if kvh < 1 or w.heads % kvh:
            continue
        K, V = K0[:kvh].contiguous(), V0[:kvh].contiguous()
        out = a2d.partial_fwd(Q, K, V, r * T, 0, True, scale)
        O, lse = a2d.fix([out[0]], [out[1]], [out[2]], torch.bfloat16)
        grads = a2d.partial_bwd(Q, K, V, O, dO, lse, r * T, 0, True, scale, workspace=ws, ds_handover=True)
        fwd = lambda: a2d.partial_fwd(Q, K, V, r * T, 0, True, scale, out=out)
        t_f = min(timeit(fwd), timeit(fwd, 20))     # the first batch still runs at the clock the set-up left
        t_b = timeit(lambda: a2d.partial_bwd(Q, K, V, O, dO, lse, r * T, 0, True, scale, out=grads, workspace=ws,
                                             ds_handover=True))
        # A2D_TILE_SPLIT_GROUPS: key blocks may be shared out over the group's query heads (larger workspace)
        ws2 = torch.empty(a2d.workspace_bytes(a2d.tile_desc(Q, K, r * T, 0, True, scale), a2d.OP_PARTIAL_BWD_SPLIT, kvh),
                          dtype=torch.uint8, device="cuda")
        t_s = timeit(lambda: a2d.partial_bwd(Q, K, V, O, dO, lse, r * T, 0, True, scale, out=grads, workspace=ws2,
                                             split_groups=True, ds_handover=True))
        del ws2
        res["cases"].append({"kv_heads": kvh, "fwd_ms": round(t_f, 4), "fwd_tflops": round(f_fl / t_f / 1e9, 1),
                             "bwd_ms": round(t_b, 4), "bwd_tflops": round(b_fl / t_b / 1e9, 1),
                             "bwd_split_groups_ms": round(t_s, 4), "bwd_split_groups_tflops": round(b_fl / t_s / 1e9, 1)})
    return res


def _timeit(torch, fn, n=10):
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(3):      # median of three loops: the first one after an idle stretch runs at lower clocks
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) / n)
    return sorted(ts)[1]


def rectangular_tiles(a2d, synth, w, scale):
    """Tiles with Nq != Nkv (Sec. 3.2 allows rectangular device grids; 8 GPUs of a node are a 2 x 4
    grid): the workload's heads on unmasked tiles of the same area as the square one, both
    orientations, forward and backward on both backward paths, with the launch shape each kernel took."""
    import torch
    H, heads = w.hdim, w.heads
    gen = torch.Generator(device="cuda"); gen.manual_seed(11)
    mk = lambda rows: torch.randn(heads, rows, H, device="cuda", generator=gen).to(torch.bfloat16)
    out = {"what": "%d heads, unmasked tiles of equal area, Nq x Nkv; fwd_wg / dq_wg = query rows per workgroup of the "
                   "forward / dQ kernels (256: eight wavefronts; 128: four, or eight in two key lanes when at most one block "
                   "comes to a compute unit), dkdv_wgs = workgroups of 128 keys" % heads,
           "cases": []}
    for nq, nkv in ((4096, 4096), (2048, 8192), (8192, 2048), (1024, 16384), (16384, 1024)):
        Q, dO, K, V = mk(nq), mk(nq), mk(nkv), mk(nkv)
        o = a2d.partial_fwd(Q, K, V, 0, 0, False, scale)
        O, lse = a2d.fix([o[0]], [o[1]], [o[2]])
        d = a2d.tile_desc(Q, K, 0, 0, False, scale)
        ws = torch.empty(a2d.workspace_bytes(d, a2d.OP_PARTIAL_BWD_DS), dtype=torch.uint8, device="cuda")
        g3 = a2d.partial_bwd(Q, K, V, O, dO, lse, 0, 0, False, scale, workspace=ws, ds_handover=True)
        t_f = _timeit(torch, lambda: a2d.partial_fwd(Q, K, V, 0, 0, False, scale, out=o))
        t_b = _timeit(torch, lambda: a2d.partial_bwd(Q, K, V, O, dO, lse, 0, 0, False, scale, out=g3, workspace=ws,
                                                     ds_handover=True), 5)
        t_r = _timeit(torch, lambda: a2d.partial_bwd(Q, K, V, O, dO, lse, 0, 0, False, scale, out=g3, workspace=ws), 5)
        base = float(heads) * nq * nkv * H
        big = heads * ((nq + 255) // 256) >= 256
        out["cases"].append({"nq": nq, "nkv": nkv, "fwd_ms": round(t_f, 4), "fwd_tflops": round(4 * base / t_f / 1e9, 1),
                             "bwd_ds_ms": round(t_b, 4), "bwd_ds_tflops": round(10 * base / t_b / 1e9, 1),
                             "bwd_recompute_ms": round(t_r, 4), "bwd_recompute_tflops": round(10 * base / t_r / 1e9, 1),
                             "fwd_wg": 256 if big else 128, "dq_wg": 256 if big else 128,
                             "dkdv_wgs": heads * ((nkv + 127) // 128)})
        del Q, dO, K, V, o, O, lse, ws, g3
    return out


def small_tiles(a2d, synth):
    """The c2 workload (2048 x 2048 tiles, 16 heads: too few workgroups to fill 256 compute units with
    256-row blocks) as a whole eager step with nothing between the calls, beside its replay from a
    HIP graph: what launch overhead costs on tiles this small."""
    import torch
    w = synth.WORKLOADS["c2"]
    T, G, H = w.tile, w.grid, w.hdim
    scale = 1.0 / math.sqrt(H)
    dev = lambda t: t.to("cuda")
    Q, dO, K, V = dev(synth.q_block(w, 0)), dev(synth.do_block(w, 0)), dev(synth.k_block(w, 0)), dev(synth.v_block(w, 0))
    f32 = dict(dtype=torch.float32, device="cuda")
    parts = [a2d.partial_fwd(Q, K, V, 0, 0, False, scale) for _ in range(G)]
    O, lse = a2d.fix([p[0] for p in parts], [p[1] for p in parts], [p[2] for p in parts])
    ws = torch.empty(a2d.workspace_bytes(a2d.tile_desc(Q, K, 0, 0, False, scale), a2d.OP_PARTIAL_BWD_DS),
                     dtype=torch.uint8, device="cuda")
    gq, gk, gv = ([torch.randn(w.heads, T, H, **f32) for _ in range(G)] for _ in range(3))
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(Q), torch.empty_like(Q)

    def step():
        a2d.partial_fwd(Q, K, V, 0, 0, False, scale, out=parts[0])
        a2d.fix([p[0] for p in parts], [p[1] for p in parts], [p[2] for p in parts], out=(O, lse))
        a2d.partial_bwd(Q, K, V, O, dO, lse, 0, 0, False, scale, out=(gq[0], gk[0], gv[0]), workspace=ws, ds_handover=True)
        a2d.fix_bwd(gq, out=dQ); a2d.fix_bwd(gk, out=dK); a2d.fix_bwd(gv, out=dV)

    def wall(fn, n=200):
        for _ in range(20):
            fn()
        torch.cuda.synchronize()
        best = None
        for _ in range(3):
            t0 = time.perf_counter()
            for _ in range(n):
                fn()
            torch.cuda.synchronize()
            t = (time.perf_counter() - t0) * 1e3 / n
            best = t if best is None or t < best else best
        return best

    eager = wall(step)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    replay = wall(graph.replay)
    fl = 14.0 * w.heads * T * T * H
    return {"workload": "c2: non-causal tile %dx%dxH%d, %d heads, fwd + fix (k=%d) + bwd + 3 fix_bwd" % (T, T, H, w.heads, G),
            "eager_ms": round(eager, 4), "eager_tflops": round(fl / eager / 1e9, 1),
            "graph_ms": round(replay, 4), "graph_tflops": round(fl / replay / 1e9, 1),
            "eager_over_graph": round(eager / replay, 3)}


def grid_emulation(synth):
    """Alg. 1 + Alg. 3 over the whole 4 x 4 grid of the c2 sequence (causal, both layouts) on one GPU:
    all tile calls on several streams, merges, gathers and scatters included."""
    import torch
    from paper_2503_15758_amd import grid as g2d
    w = synth.WORKLOADS["c2"]
    n, G, H = w.tile * w.grid, w.grid, w.hdim
    gen = torch.Generator(device="cuda"); gen.manual_seed(7)
    mk = lambda: torch.randn(w.heads, n, H, device="cuda", generator=gen).to(torch.bfloat16)
    Q, K, V, dO = mk(), mk(), mk(), mk()
    out = {}
    flops = 14.0 * w.heads * n * n * H * (n + 1) / (2.0 * n)          # causal fwd + bwd, algorithmic
    for layout in ("cyclic", "contiguous"):
        for streams in (1, 4):
            def run():
                O, lse = g2d.forward(Q, K, V, G, True, layout, None, streams)
                return g2d.backward(Q, K, V, O, dO, lse, G, True, layout, None, streams)
            run(); run()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(5):
                run()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / 5
            out["%s_%dstream" % (layout, streams)] = {"ms": round(ms, 3), "tflops": round(flops / ms / 1e9, 1)}
    out["what"] = "causal fwd + bwd of %d tokens, %d heads, H%d over a %dx%d grid" % (n, w.heads, H, G, G)
    return out


def cpu_baseline(w, scale):
    """The fp64 oracle, as it stands, on the host cores: partial forward + AttnFix (k = 1) + partial
    backward of an unmasked tile for a bounded number of heads (about 1.2e12 algorithmic FLOPs, some
    15 s on 16 cores)."""
    import oracle
    from paper_2503_15758_amd import synth
    T, H = w.tile, w.hdim
    per_head = (14.0 if w.backward else 4.0) * T * T * H
    nh = int(max(1, min(w.heads, round(1.2e12 / per_head))))
    nq_s = T if per_head <= 1.2e12 else max(64, int(1.2e12 / ((14.0 if w.backward else 4.0) * T * H)))
    sub = synth.Workload(w.name, w.dtype, nh, H, w.seq, w.grid, w.causal, w.backward, w.sigma_qk, w.seed)
    n64 = lambda t: t.double().numpy()
    Q = n64(synth.q_block(sub, w.grid - 1, nq_s)); K = n64(synth.k_block(sub, 0)); V = n64(synth.v_block(sub, 0))
    dO = n64(synth.do_block(sub, w.grid - 1, nq_s))
    t0 = time.perf_counter()
    N, m, l = oracle.partial_fwd(Q, K, V, 0, 0, False, scale)
    O, lse = oracle.fix([N], [m], [l])
    fl = 4.0 * nh * nq_s * T * H
    if w.backward:
        oracle.partial_bwd(Q, K, V, O, dO, lse, 0, 0, False, scale)
        fl += 10.0 * nh * nq_s * T * H
    sec = time.perf_counter() - t0
    return {"value": round(fl / sec / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": round(sec, 2),
            "sample": "%d head(s), %d query rows x %d keys x H%d of an unmasked tile, fp64 partial "
                      "fwd + fix%s" % (nh, nq_s, T, H, " + partial bwd" if w.backward else "")}


if __name__ == "__main__":
    main()
