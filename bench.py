"""Benchmark of the MoE dispatch/combine shuffle on one MI355X.

A step is one pass of the whole hot path (layout, dispatch_send, dispatch_recv,
combine_send, combine_reduce) over one synthetic batch that is already resident
in HBM.  Prints ONE JSON line.  `value` is the achieved rate in GB/s: the
algorithmic bytes of the staged data flow divided by the step time.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload dsv3_decode]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
WRITES = {}          # per kernel: bytes written per step (filled by algorithmic_bytes)


def algorithmic_bytes(wl, ttot, D, P, sizes, push=False, partial=False, ready=False):
    """Bytes the method itself has to move (reads + writes), per kernel.  Staged
    (default): pack into send buffers, scatter, unpack.  Push: the send kernels
    write into the receive buffers, so the send-buffer write and the scatter's
    read and write are not part of the method."""
    Be = sizes.expert_x_row_bytes + 4 * sizes.scales_per_row
    # a dispatched row as the method defines it; the library pads e4m3 wire rows to whole
    # 128-byte lines, and that padding is not counted as useful traffic
    Bx, Bw, Bc = sizes.x_row_bytes, min(sizes.wire_row_bytes, Be), sizes.combine_row_bytes
    if ready:        # the pack kernel reads wire-format rows instead of bf16 rows
        Bx = Bw
    k = {
        "dispatch_pack_kernel": ttot * Bx + D * Bw,
        "fabric_copy_kernel(dispatch)": 2 * D * Bw,
        "dispatch_unpack_kernel": D * Bw + P * Be,
        "combine_pack_kernel": 2 * P * Bc,
        "fabric_copy_kernel(combine)": 2 * P * Bc,
        "combine_reduce_kernel": P * Bc + ttot * Bc,
    }
    if partial:      # one reply row per received row: P rows read, D written, D moved, D read
        del k["combine_pack_kernel"]
        k["combine_partial_pack_kernel"] = P * Bc + D * Bc
        k["fabric_copy_kernel(combine)"] = 2 * D * Bc
        k["combine_reduce_kernel"] = D * Bc + ttot * Bc
    if push:
        del k["fabric_copy_kernel(dispatch)"], k["fabric_copy_kernel(combine)"]
    if wl.dispatch_dtype != "bf16" and not ready:
        k["dispatch_pack_e4m3_kernel"] = k.pop("dispatch_pack_kernel")
    # bytes each kernel writes (the rest it reads): for the one-directional ceilings
    WRITES.clear()
    WRITES.update({"dispatch_pack_kernel": D * Bw, "dispatch_pack_e4m3_kernel": D * Bw,
                   "fabric_copy_kernel(dispatch)": D * Bw, "dispatch_unpack_kernel": P * Be,
                   "combine_pack_kernel": P * Bc, "combine_partial_pack_kernel": D * Bc,
                   "fabric_copy_kernel(combine)": (D if partial else P) * Bc,
                   "combine_reduce_kernel": ttot * Bc})
    dispatch = sum(v for n, v in k.items() if n.startswith(("dispatch", "fabric_copy_kernel(d")))
    combine = sum(v for n, v in k.items() if n.startswith(("combine", "fabric_copy_kernel(c")))
    return k, dispatch, combine


def step_time(workloads, harness, torch, name, steps, warmup, two_streams=False, **mode):
    """ms per step of one named workload in one mode (a context of its own, inputs resident,
    identity expert stage or a resident expert_y), with the rate against THAT workload's and
    mode's own algorithmic bytes.  Used for the side measurements beside the headline."""
    wl = workloads.WORKLOADS[name]
    inp = workloads.make_inputs(wl)
    st = workloads.describe(inp)
    dev = harness.to_device(inp, "cuda:0")
    cf = None if wl.zipf_alpha > 0 else (1.1 if wl.tokens >= 2048 else 1.5)
    sh = harness.make_shuffle(inp, capacity_factor=cf, **mode)
    _, bd, bc = algorithmic_bytes(wl, st["tokens_total"], st["dedup_rows"], st["pairs"], sh.sizes,
                                  mode.get("peer_push", False), mode.get("partial_sums", False))
    y = sh.expert_x
    if wl.dispatch_dtype != "bf16":
        y = torch.zeros((wl.n_ranks, sh.expert_capacity_rows, wl.hidden), dtype=torch.bfloat16,
                        device="cuda:0")
    if two_streams:
        streams = (torch.cuda.Stream(), torch.cuda.Stream())
        run = lambda: harness.run_step_two_streams(sh, dev, expert_y=y, streams=streams)
    else:
        run = lambda: harness.run_hot_path(sh, dev, None if y is sh.expert_x else y)
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    assert sh.status() == 0, f"device status not clean: {name} {mode}"
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    assert sh.status() == 0
    sh.close()
    del sh, dev, y
    torch.cuda.empty_cache()
    gbps = (bd + bc) / (ms * 1e-3) / 1e9
    return {"ms_per_step": round(ms, 4), "step_us": round(ms * 1e3, 1), "steps": steps,
            "algorithmic_bytes": bd + bc, "value": round(gbps, 1), "unit": "GB/s",
            "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4)}


def compare_modes(workloads, harness, torch, name, variants, steps, rounds=4):
    """Step times of several modes of one workload measured in turns (round-robin, `rounds`
    rounds of `steps` steps each, median over the rounds), all contexts alive at once: the
    machine's speed drifts by a few percent over seconds, so modes measured one after the
    other cannot be compared, modes measured in turns can.  variants: {label: kwargs of
    make_shuffle, plus two_streams=True for senders and receivers on two streams}."""
    import numpy as np
    wl = workloads.WORKLOADS[name]
    inp = workloads.make_inputs(wl)
    st = workloads.describe(inp)
    dev = harness.to_device(inp, "cuda:0")
    cf = None if wl.zipf_alpha > 0 else (1.1 if wl.tokens >= 2048 else 1.5)
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    runs = {}
    for label, kw in variants.items():
        kw = dict(kw)
        two = kw.pop("two_streams", False)
        sh = harness.make_shuffle(inp, capacity_factor=cf, **kw)
        _, bd, bc = algorithmic_bytes(wl, st["tokens_total"], st["dedup_rows"], st["pairs"], sh.sizes,
                                      kw.get("peer_push", False), kw.get("partial_sums", False))
        if two:
            fn = lambda sh=sh: harness.run_step_two_streams(sh, dev, expert_y=sh.expert_x, streams=streams)
        else:
            fn = lambda sh=sh: harness.run_hot_path(sh, dev)
        runs[label] = (sh, fn, bd + bc, [])
    for rnd in range(rounds + 1):                # round 0 warms up
        for label, (sh, fn, nbytes, times) in runs.items():
            for _ in range(5):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                fn()
            torch.cuda.synchronize()
            if rnd:
                times.append((time.perf_counter() - t0) * 1e3 / steps)
    out = {}
    for label, (sh, fn, nbytes, times) in runs.items():
        assert sh.status() == 0, f"device status not clean: {label}"
        sh.close()
        ms = float(np.median(times))
        gbps = nbytes / (ms * 1e-3) / 1e9
        out[label] = {"step_us": round(ms * 1e3, 1), "step_us_rounds": [round(t * 1e3, 1) for t in times],
                      "algorithmic_bytes": nbytes, "value": round(gbps, 1), "unit": "GB/s",
                      "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4)}
    torch.cuda.empty_cache()
    return out


def interleaved_caller_work(workloads, harness, torch, steps=100, rounds=3):
    """Section MoE Dispatch/Combine: the send and the receive half of dispatch and of combine are
    calls of their own so that the caller's other work can run between them.  The decode step in
    the default mode on one stream, with a compute-bound kernel of the caller (a bf16 matrix
    product from the BLAS library: the stand-in for shared-expert or attention work of another
    micro-batch, no part of the shuffle) enqueued on a second stream right after each send call.
    Measured in turns: the step alone, the two products alone, both together."""
    import numpy as np
    wl = workloads.WORKLOADS["dsv3_decode"]
    inp = workloads.make_inputs(wl)
    dev = harness.to_device(inp, "cuda:0")
    sh = harness.make_shuffle(inp, capacity_factor=1.5)
    a = torch.randn(4096, wl.hidden, device="cuda:0", dtype=torch.bfloat16)
    b = torch.randn(wl.hidden, 4096, device="cuda:0", dtype=torch.bfloat16)
    c = torch.empty(4096, 4096, device="cuda:0", dtype=torch.bfloat16)
    side = torch.cuda.Stream()
    main_stream = torch.cuda.current_stream()

    def step(shuffle, work):
        if work:
            main_stream.wait_stream(side)        # the previous step's products have ended
            side.wait_stream(main_stream)
        if shuffle:
            sh.layout(dev["indices"], dev["num_tokens"])
            sh.dispatch_send(dev["x"])
        if work:
            with torch.cuda.stream(side):
                torch.matmul(a, b, out=c)
        if shuffle:
            sh.dispatch_recv()
            sh.combine_send(sh.expert_x)
        if work:
            with torch.cuda.stream(side):
                torch.matmul(a, b, out=c)
        if shuffle:
            sh.combine_reduce(dev["weights"])

    cases = {"step_alone_us": (True, False), "products_alone_us": (False, True), "together_us": (True, True)}
    times = {k: [] for k in cases}
    for rnd in range(rounds + 1):                # round 0 warms up
        for k, (shuffle, work) in cases.items():
            for _ in range(5):
                step(shuffle, work)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                step(shuffle, work)
            torch.cuda.synchronize()
            if rnd:
                times[k].append((time.perf_counter() - t0) * 1e6 / steps)
    assert sh.status() == 0
    sh.close()
    out = {k: round(float(np.median(v)), 1) for k, v in times.items()}
    out["hidden_us"] = round(out["step_alone_us"] + out["products_alone_us"] - out["together_us"], 1)
    out["caller_work"] = "two bf16 matrix products [4096 x %d] x [%d x 4096] per step on a second stream, " \
                         "one enqueued after each send call" % (wl.hidden, wl.hidden)
    del a, b, c
    torch.cuda.empty_cache()
    return out


def ordering_name(args):
    if args.stream_ordered:
        return "stream order supplied by the caller (no announce, no gate kernels)"
    if args.progressive:
        return "arrival counters only, per-wave progress, polling receive kernels"
    return "arrival counters only (announce kernel after each send, gate kernel before each receive)"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="0 = 1000, or 10 for the prefill workload")
    ap.add_argument("--warmup", type=int, default=-1, help="-1 = 200, or 2 for the prefill workload")
    ap.add_argument("--workload", default="dsv3_decode")
    ap.add_argument("--capacity-factor", type=float, default=1.5,
                    help="per-rank buffer capacity as a multiple of the mean load (0 = worst case)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stream-ordered", action="store_true",
                    help="FL_FLAG_STREAM_ORDERED: the caller keeps sends before receives in stream order, "
                         "the library launches no announce and no gate kernels (the counters are then "
                         "bookkeeping, not a completion signal)")
    ap.add_argument("--progressive", action="store_true",
                    help="FL_FLAG_PROGRESSIVE_RECV: write-through senders, every wave reports, receive "
                         "kernels poll per source on capped grids")
    ap.add_argument("--overlap", action="store_true",
                    help="send calls on a second stream: the receivers wait on the arrival counters "
                         "while the fabric copy runs (reports the step time only)")
    ap.add_argument("--push", action="store_true",
                    help="FL_FLAG_PEER_PUSH: send kernels store into the peers' receive buffers, no "
                         "send buffer and no scatter; GB/s is then computed against the smaller byte "
                         "count of that method")
    ap.add_argument("--partial-sums", action="store_true",
                    help="FL_FLAG_PARTIAL_SUMS: combine sends one bf16 partial sum per (token, expert "
                         "rank); another arithmetic than the default, fewer bytes")
    ap.add_argument("--chunk-tokens", type=int, default=0,
                    help="chunked prefill: step a context sized for this many tokens per rank over the "
                         "workload's batch (reports time per whole batch and the workspace size)")
    ap.add_argument("--ready-e4m3", action="store_true",
                    help="e4m3 workloads: dispatch tokens that are already quantised (synthetic codes and "
                         "scales), the payload of the paper's microbenchmark, instead of quantising bf16")
    ap.add_argument("--private-rows", type=int, default=0,
                    help="first rows per (source, destination) sent to private slots in a scatter "
                         "of their own (ablation of section Ablation: Private Buffer Size)")
    ap.add_argument("--headline-only", action="store_true",
                    help="skip the side measurements that launch the kernels at other sizes or in "
                         "other modes (single-rank split, peer-push variant); for profiler runs")
    ap.add_argument("--profile-steps", type=int, default=200)
    ap.add_argument("--counters", action="store_true",
                    help="short run for `rocprofv3 --pmc`: a few steps plus one plain 1 GiB copy "
                         "of known size to calibrate the byte counters; no timing output")
    ap.add_argument("--interleaved", action="store_true",
                    help="only the decode step with a caller's matrix products on a second stream between "
                         "the send and receive halves (the side measurement interleaved_caller_work)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs the whole simulated expert-parallel group on ONE GPU; "
              "--gpus above 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2510_27656_amd import flmoe, harness, workloads

    if args.interleaved:
        res = interleaved_caller_work(workloads, harness, torch, steps=max(20, min(args.steps or 100, 100)))
        print(json.dumps({"metric": "interleaved_caller_work", "ms_per_step": round(res["together_us"] / 1e3, 4),
                          "config": {"workload": "dsv3_decode"}, "library_build_id": flmoe.fl_moe_build_id(),
                          "interleaved_caller_work": res}))
        return

    wl = workloads.WORKLOADS[args.workload]
    big = wl.tokens >= 2048
    if args.steps <= 0:
        args.steps = 10 if big else 1000
    if args.warmup < 0:
        args.warmup = 2 if big else 200
    if big:
        args.profile_steps = min(args.profile_steps, 5)
    inp = workloads.make_inputs(wl)
    stats = workloads.describe(inp)
    dev = harness.to_device(inp, "cuda:0")
    cf = args.capacity_factor if args.capacity_factor > 0 else None
    if wl.zipf_alpha > 0:
        cf = None                       # skewed routing: size for the worst case
    elif big:
        cf = min(cf or 1.1, 1.1)        # 16 GB buffers at 1.1x the mean; the worst case would not fit
    sh = harness.make_shuffle(inp, capacity_factor=cf,
                              stream_ordered=args.stream_ordered, progressive_recv=args.progressive,
                              max_private_rows=args.private_rows, peer_push=args.push,
                              partial_sums=args.partial_sums)
    ttot, D, P = stats["tokens_total"], stats["dedup_rows"], stats["pairs"]
    per_kernel, bytes_dispatch, bytes_combine = algorithmic_bytes(wl, ttot, D, P, sh.sizes, args.push, args.partial_sums, args.ready_e4m3)
    bytes_step = bytes_dispatch + bytes_combine

    expert_y = None
    if wl.dispatch_dtype != "bf16":     # e4m3 dispatch: combine needs a resident bf16 expert output
        expert_y = torch.zeros((wl.n_ranks, sh.expert_capacity_rows, wl.hidden),
                               dtype=torch.bfloat16, device="cuda:0")

    ready = None
    if args.ready_e4m3:
        assert wl.dispatch_dtype != "bf16", "--ready-e4m3 needs a workload with e4m3 dispatch"
        gen = torch.Generator(device="cuda:0").manual_seed(7)
        codes = torch.randint(0, 0x78, (wl.n_ranks, wl.tokens, wl.hidden), dtype=torch.uint8,
                              device="cuda:0", generator=gen)           # finite, positive codes
        scales = torch.rand((wl.n_ranks, wl.tokens, wl.hidden // 128), device="cuda:0", generator=gen) + 0.5
        ready = (codes, scales)

    def step():
        harness.run_hot_path(sh, dev, expert_y, ready)

    if args.chunk_tokens:
        C = args.chunk_tokens
        whole_bytes = int(sh.sizes.workspace_bytes)
        sh.close()
        pieces = [(t0, workloads.token_chunk(inp, t0, C)) for t0 in range(0, wl.tokens, C)]
        chunks = [(t0, harness.to_device(p, "cuda:0")) for t0, p in pieces]
        # small chunks fluctuate more around the mean load than the whole batch does
        cfc = cf if cf is None or C >= 1024 else max(cf, 1.5)
        shc = harness.make_shuffle(pieces[0][1], capacity_factor=cfc, peer_push=args.push,
                                   partial_sums=args.partial_sums)
        out_full = torch.empty((wl.n_ranks, wl.tokens, wl.hidden), dtype=torch.bfloat16, device="cuda:0")
        for _ in range(max(1, args.warmup // 2)):
            harness.run_chunked(shc, chunks, out_full, with_expert=False)
        torch.cuda.synchronize()
        assert shc.status() == 0
        t0 = time.perf_counter()
        for _ in range(args.steps):
            harness.run_chunked(shc, chunks, out_full, with_expert=False)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        assert shc.status() == 0
        print(json.dumps({"metric": f"dispatch+combine achieved HBM GB/s, workload {wl.name} in chunks of "
                                    f"{C} tokens per rank",
                          "value": round(bytes_step / (ms * 1e-3) / 1e9, 1), "unit": "GB/s", "n_gpus": 1,
                          "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
                          "higher_is_better": True,
                          "config": {"workload": wl.name, "chunk_tokens": C, "chunks": len(chunks),
                                     "workspace_bytes": int(shc.sizes.workspace_bytes),
                                     "workspace_bytes_one_shot": whole_bytes}}))
        shc.close()
        return

    if args.overlap:
        streams = (torch.cuda.Stream(), torch.cuda.Stream())
        y = sh.expert_x if expert_y is None else expert_y

        def ostep():
            harness.run_step_two_streams(sh, dev, expert_y=y, streams=streams)

        for _ in range(args.warmup):
            ostep()
        torch.cuda.synchronize()
        assert sh.status() == 0
        t0 = time.perf_counter()
        for _ in range(args.steps):
            ostep()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        assert sh.status() == 0
        print(json.dumps({"metric": "dispatch+combine achieved HBM GB/s, senders and receivers on "
                                    "two streams",
                          "value": round(bytes_step / (ms * 1e-3) / 1e9, 1), "unit": "GB/s",
                          "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                          "ms_per_step": round(ms, 4), "higher_is_better": True,
                          "library_build_id": flmoe.fl_moe_build_id(),
                          "config": {"workload": wl.name, "ordering": ordering_name(args), "streams": 2}}))
        sh.close()
        return

    if args.counters:
        for _ in range(3):
            step()
        a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
        b = torch.ones(1 << 30, dtype=torch.uint8, device="cuda:0")
        flmoe.fl_moe_debug_copy(a, b, 1 << 30)
        torch.cuda.synchronize()
        assert sh.status() == 0
        print(json.dumps({"counters_run": True, "workload": wl.name, "copy_bytes": 1 << 30, "steps": 3,
                          "library_build_id": flmoe.fl_moe_build_id(), "algorithmic_bytes": per_kernel}))
        sh.close()
        return

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    assert sh.status() == 0, "device status not clean after warm-up"
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    assert sh.status() == 0

    # host cost of enqueueing one step (the five C calls through the binding, nothing
    # waited for): the part of the paper's CPU-overhead table that exists here
    torch.cuda.synchronize()
    h0 = time.perf_counter()
    for _ in range(10):
        step()
    host_enqueue_us = (time.perf_counter() - h0) * 1e6 / 10
    torch.cuda.synchronize()

    # per-call split with events on the stream the library launches on
    calls = ["layout", "dispatch_send", "dispatch_recv", "combine_send", "combine_reduce"]
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.profile_steps)]
    for i in range(args.profile_steps):
        ev[i][0].record()
        sh.layout(dev["indices"], dev["num_tokens"]); ev[i][1].record()
        if ready is None:
            sh.dispatch_send(dev["x"], weights=harness.send_weights(sh, dev))
        else:
            sh.dispatch_send(ready[0], scales=ready[1], weights=harness.send_weights(sh, dev))
        ev[i][2].record()
        sh.dispatch_recv(); ev[i][3].record()
        sh.combine_send(sh.expert_x if expert_y is None else expert_y); ev[i][4].record()
        sh.combine_reduce(dev["weights"]); ev[i][5].record()
    torch.cuda.synchronize()
    per_call = {c: np.array([ev[i][j].elapsed_time(ev[i][j + 1]) for i in range(args.profile_steps)]) * 1e3
                for j, c in enumerate(calls)}
    call_us = {c: float(np.median(v)) for c, v in per_call.items()}
    disp = per_call["layout"] + per_call["dispatch_send"] + per_call["dispatch_recv"]
    comb = per_call["combine_send"] + per_call["combine_reduce"]

    def dist(v):      # the paper's latency figures show mean and p01..p99
        return {"mean": round(float(v.mean()), 1), "p01": round(float(np.percentile(v, 1)), 1),
                "p50": round(float(np.percentile(v, 50)), 1), "p99": round(float(np.percentile(v, 99)), 1)}
    latency_us = {"dispatch": dist(disp), "combine": dist(comb), "samples": args.profile_steps}
    dispatch_us = call_us["layout"] + call_us["dispatch_send"] + call_us["dispatch_recv"]
    combine_us = call_us["combine_send"] + call_us["combine_reduce"]

    # One real rank's share (rank_count = 1): rank 0's four payload calls timed alone, the
    # other ranks' launches issued around them outside the brackets.  The layout call
    # cannot be split this way (its planning kernel waits for every peer's counts).
    single_rank_us = None
    if wl.n_ranks > 1 and not big and not args.headline_only and ready is None:
        me, rest = (0, 1), (1, wl.n_ranks - 1)
        y = sh.expert_x if expert_y is None else expert_y
        reps = min(args.profile_steps, 50)
        sev = [[torch.cuda.Event(enable_timing=True) for _ in range(8)] for _ in range(reps)]
        for i in range(reps):
            e = sev[i]
            sh.layout(dev["indices"], dev["num_tokens"])
            sw = harness.send_weights(sh, dev)
            sh.dispatch_send(dev["x"], rest, weights=sw)
            e[0].record(); sh.dispatch_send(dev["x"], me, weights=sw); e[1].record()
            e[2].record(); sh.dispatch_recv(me); e[3].record()
            sh.dispatch_recv(rest)
            sh.combine_send(y, rest)
            e[4].record(); sh.combine_send(y, me); e[5].record()
            e[6].record(); sh.combine_reduce(dev["weights"], me); e[7].record()
            sh.combine_reduce(dev["weights"], rest)
        torch.cuda.synchronize()
        assert sh.status() == 0
        single_rank_us = {c: round(float(np.median([sev[i][2 * j].elapsed_time(sev[i][2 * j + 1])
                                                    for i in range(reps)])) * 1e3, 1)
                          for j, c in enumerate(calls[1:])}

    # per-kernel durations (HIP events inside the library, on the same stream)
    flmoe.fl_moe_profile_enable(sh.ctx, 1)
    for _ in range(args.profile_steps):
        step()
        flmoe.fl_moe_profile_collect(sh.ctx)
    flmoe.fl_moe_profile_enable(sh.ctx, 0)
    prof = flmoe.fl_moe_profile_read(sh.ctx)
    kern_us = {n: ms / cnt * 1e3 for n, (ms, cnt) in prof.items() if cnt}          # per launch
    # launches per step: 1, except for calls that move
    # several GB, which the library issues as one launch per group of ranks
    kern_launches = {n: cnt / args.profile_steps for n, (ms, cnt) in prof.items() if cnt}
    step_us_of = {n: kern_us[n] * kern_launches[n] for n in kern_us}
    dominant = max((n for n in kern_us if n in per_kernel), key=lambda n: step_us_of[n])
    launch_bytes = per_kernel[dominant] / kern_launches[dominant]
    achieved = launch_bytes / (kern_us[dominant] * 1e-6) / 1e9
    # HBM bytes of that kernel from the stored rocprofv3 --pmc passes; only figures measured
    # with the very library build that is being timed count (else null, with the reason)
    from paper_2510_27656_amd import profiling
    build_id = flmoe.fl_moe_build_id()
    mode_tag = "stream_ordered" if args.stream_ordered else ("progressive" if args.progressive else "")
    plain_mode = not (args.push or args.partial_sums or args.private_rows or args.ready_e4m3)
    traffic, traffic_note = (profiling.stored_traffic(args.workload, dominant, build_id, mode_tag)
                             if plain_mode else (None, "no counter run stored for this mode"))
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                "traffic": traffic, "algorithmic_bytes": round(launch_bytes),
                "avg_us": round(kern_us[dominant], 2),
                "launches_per_step": round(kern_launches[dominant], 2)}
    if traffic is None:
        roofline["traffic_stale"] = traffic_note

    # cold protocol (the paper clears caches between iterations): a 2 GiB copy between
    # steps evicts the 256 MB last-level cache; per-call medians with HIP events
    flush_src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda:0")
    flush_dst = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
    cold = []
    for i in range(args.profile_steps):
        flmoe.fl_moe_debug_copy(flush_dst, flush_src, 1 << 30)
        e = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        e[0].record(); step(); e[1].record()
        cold.append(e)
    torch.cuda.synchronize()
    cold_us = float(np.median([a.elapsed_time(b) for a, b in cold])) * 1e3
    # copy ceiling of this machine: plain 16-byte copy of 1 GiB (2 GiB of traffic)
    ce = []
    for i in range(12):
        e = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        e[0].record(); flmoe.fl_moe_debug_copy(flush_dst, flush_src, 1 << 30); e[1].record()
        ce.append(e)
    torch.cuda.synchronize()
    copy_gbps = 2 * (1 << 30) / (float(np.median([a.elapsed_time(b) for a, b in ce[2:]])) * 1e-3) / 1e9
    # one-directional ceilings, same launch shape: write-only (fill) and read-only, 1 GiB each
    sink = torch.zeros(4, dtype=torch.int32, device="cuda:0")

    def ceiling(fn):
        evs = []
        for i in range(12):
            e = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            e[0].record(); fn(); e[1].record()
            evs.append(e)
        torch.cuda.synchronize()
        return (1 << 30) / (float(np.median([a.elapsed_time(b) for a, b in evs[2:]])) * 1e-3) / 1e9
    write_gbps = ceiling(lambda: flmoe.fl_moe_debug_fill(flush_dst, 1 << 30))
    read_gbps = ceiling(lambda: flmoe.fl_moe_debug_read(flush_src, 1 << 30, sink))
    del flush_src, flush_dst
    # A kernel that reads r and writes w bytes cannot beat r / read ceiling + w / write ceiling
    # (for r = w this is the measured copy ceiling to within a few percent): each kernel's
    # time against that bound
    rw_bound_us = {k: ((per_kernel[k] - WRITES[k]) / read_gbps + WRITES[k] / write_gbps) / 1e3 / kern_launches[k]
                   for k in kern_us if k in per_kernel and k in WRITES}

    # The same step captured once in a HIP graph and replayed (the five calls only
    # enqueue kernels); what it saves is host launch work, which shows on small shapes.
    graph_line = None
    if not big and not args.headline_only:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        for _ in range(min(args.warmup, 20)):
            g.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        gms = (time.perf_counter() - g0) * 1e3 / args.steps
        assert sh.status() == 0
        graph_line = {"ms_per_step": round(gms, 4), "value": round(bytes_step / (gms * 1e-3) / 1e9, 1),
                      "unit": "GB/s"}
        del g

    # The same step with FL_FLAG_PEER_PUSH, beside the headline: fewer bytes by
    # construction, so its GB/s is computed against its own byte count.
    push_line = None
    if not args.push and not big and not args.progressive and not args.headline_only and not args.partial_sums \
            and not args.ready_e4m3:
        shp = harness.make_shuffle(inp, capacity_factor=cf, max_private_rows=args.private_rows,
                                   peer_push=True, stream_ordered=args.stream_ordered)
        _, pd, pc = algorithmic_bytes(wl, ttot, D, P, shp.sizes, True)
        for _ in range(args.warmup):
            harness.run_hot_path(shp, dev, expert_y)
        torch.cuda.synchronize()
        p0 = time.perf_counter()
        for _ in range(args.steps):
            harness.run_hot_path(shp, dev, expert_y)
        torch.cuda.synchronize()
        pms = (time.perf_counter() - p0) * 1e3 / args.steps
        assert shp.status() == 0
        shp.close()
        push_line = {"ms_per_step": round(pms, 4), "step_us": round(pms * 1e3, 1), "algorithmic_bytes": pd + pc,
                     "value": round((pd + pc) / (pms * 1e-3) / 1e9, 1), "unit": "GB/s",
                     "frac_of_hbm_peak": round((pd + pc) / (pms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}

    # The modes and workloads that are not the headline, measured in the same run: the
    # fabric that keeps the arrival-counter contract with no ordering assumed (one stream,
    # and with senders and receivers on two streams), and the other four named workloads.
    side = args.workload == "dsv3_decode" and not args.headline_only and not (
        args.push or args.stream_ordered or args.progressive or args.partial_sums or args.private_rows
        or args.ready_e4m3)
    modes = others = interleaved = None
    if side:
        sh.close()
        n = max(20, min(args.steps, 300))
        w = max(5, min(args.warmup, 50))
        modes = compare_modes(workloads, harness, torch, "dsv3_decode", {
            "default (counters order everything; one stream)": {},
            "default, senders and receivers on two streams": {"two_streams": True},
            "FL_FLAG_STREAM_ORDERED (no announce, no gate kernels)": {"stream_ordered": True},
            "FL_FLAG_PROGRESSIVE_RECV, one stream": {"progressive_recv": True},
            "FL_FLAG_PROGRESSIVE_RECV, two streams": {"progressive_recv": True, "two_streams": True},
            "FL_FLAG_PEER_PUSH (fewer bytes by construction)": {"peer_push": True},
        }, steps=max(20, min(args.steps, 100)))
        interleaved = interleaved_caller_work(workloads, harness, torch)
        others = {}
        for name, note in [("tiny", "launch-bound: eleven kernels on a few KB"),
                           ("qwen3_skew", "cache-assisted: the working set partly fits the 256 MB last-level cache"),
                           ("dsv3_fp8", "e4m3 dispatch quantised on the fly, bf16 combine"),
                           ("dsv3_prefill", "4096 tokens per rank, payload calls cut into launches of 2 ranks")]:
            big_w = workloads.WORKLOADS[name].tokens >= 2048
            # the short steps need a few hundred repetitions to reach their steady rate
            others[name] = step_time(workloads, harness, torch, name, 5 if big_w else max(n, 200),
                                     2 if big_w else max(w, 20))
            others[name]["note"] = note

    cpu = None
    if not args.no_cpu_baseline:
        from oracle.reference_step import oracle_step
        cpu_inp, cpu_bytes, what = inp, bytes_step, f"full {wl.name} steps"
        if big:      # bounded sample: the first 128 tokens of every rank as a step of their own
            cpu_inp = workloads.token_chunk(inp, 0, 128)
            st = workloads.describe(cpu_inp)
            _, cd, cc = algorithmic_bytes(wl, st["tokens_total"], st["dedup_rows"], st["pairs"], sh.sizes,
                                          args.push, args.partial_sums, args.ready_e4m3)
            cpu_bytes, what = cd + cc, f"steps over the first 128 tokens per rank of {wl.name}"
        reps, c0 = 0, time.perf_counter()
        while reps < 40 and (reps == 0 or time.perf_counter() - c0 < 12.0):
            oracle_step(cpu_inp)
            reps += 1
        per = (time.perf_counter() - c0) / reps
        cpu = {"value": round(cpu_bytes / per / 1e9, 3), "unit": "GB/s", "cores": 1,
               "kind": "oracle", "seconds_per_step": round(per, 3), "repetitions": reps,
               "sample": f"{reps} {what} (all {wl.n_ranks} ranks, {int(cpu_inp.num_tokens.sum())} tokens in all), "
                         "algorithmic byte count of the sample, single thread"}
        # The same untouched oracle on all the host cores this job may use: one whole
        # step per thread, side by side (its C routines run outside the interpreter lock).
        workers = max(1, min(16, len(os.sched_getaffinity(0))))
        if workers > 1:
            from concurrent.futures import ThreadPoolExecutor
            rounds = max(1, min(4, int(10.0 / max(per, 1e-3) / workers + 0.5)))
            a0 = time.perf_counter()
            with ThreadPoolExecutor(workers) as pool:
                list(pool.map(lambda _: [oracle_step(cpu_inp) for _ in range(rounds)], range(workers)))
            aper = (time.perf_counter() - a0) / (rounds * workers)
            cpu["all_cores"] = {"value": round(cpu_bytes / aper / 1e9, 3), "unit": "GB/s", "cores": workers,
                                "sample": f"{rounds * workers} of the same steps, {workers} threads with "
                                          f"{rounds} step(s) each"}

    value = bytes_step / (ms_per_step * 1e-3) / 1e9
    line = {
        "metric": "dispatch+combine achieved HBM GB/s (algorithmic bytes / step time), "
                  "T=128 H=7168 top-8, 256 experts" if args.workload == "dsv3_decode"
                  else f"dispatch+combine achieved HBM GB/s, workload {args.workload}",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if wl.dispatch_dtype == "bf16" else "e4m3+bf16",
        "data": "synthetic", "library_build_id": build_id,
        "config": {"workload": wl.name, "ranks_simulated": wl.n_ranks, "experts": wl.n_experts,
                   "tokens_per_rank": wl.tokens, "hidden": wl.hidden, "top_k": wl.top_k,
                   "dedup_rows": D, "pairs": P, "capacity_factor": cf, "private_rows": int(sh.sizes.private_rows),
                   "method": "peer push (no send buffer, no scatter)" if args.push else "staged (pack, scatter, unpack)",
                   "combine": "sender-side bf16 partial sums" if args.partial_sums else "fp32 sum in k order",
                   "dispatch_input": "ready-made e4m3 codes + scales" if args.ready_e4m3 else "bf16",
                   "ordering": ordering_name(args),
                   "expert_stage": "identity (expert_y aliases expert_x)" if expert_y is None
                   else "none in the timed path (resident bf16 expert_y)"},
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4),
        "algorithmic_bytes": {"dispatch": bytes_dispatch, "combine": bytes_combine},
        "dispatch_us": round(dispatch_us, 1), "combine_us": round(combine_us, 1),
        "cold_step_us": round(cold_us, 1),
        "cold_gbps": round(bytes_step / (cold_us * 1e-6) / 1e9, 1),
        "copy_ceiling_gbps": round(copy_gbps, 1),
        "write_ceiling_gbps": round(write_gbps, 1), "read_ceiling_gbps": round(read_gbps, 1),
        "kernel_frac_of_read_write_bound": {k: round(v / kern_us[k], 4) for k, v in rw_bound_us.items()},
        "frac_of_copy_ceiling": round(value / copy_gbps, 4),
        "latency_us": latency_us,
        "call_us": {k: round(v, 1) for k, v in call_us.items()},
        "single_rank_call_us": single_rank_us,
        "host_enqueue_us_per_step": round(host_enqueue_us, 1),
        "kernel_us": {k: round(v, 2) for k, v in kern_us.items()},
        "kernel_launches_per_step": {k: round(v, 2) for k, v in kern_launches.items()},
        "kernel_gbps": {k: round(per_kernel[k] / (step_us_of[k] * 1e-6) / 1e9, 1)
                        for k in kern_us if k in per_kernel},
        "hip_graph_replay": graph_line,
        "step_us": round(ms_per_step * 1e3, 1),
        "gbps_note": "GB/s divides each method's OWN algorithmic bytes by its step time: compare methods "
                     "by step_us, not by GB/s (peer push moves fewer bytes and is the faster method)",
        "peer_push_variant": push_line,
        "modes_measured_in_turns": modes,
        "other_workloads": others,
        "interleaved_caller_work": interleaved,
        "roofline": roofline, "cpu_baseline": cpu,
    }
    if sh.ctx is not None:
        sh.close()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
