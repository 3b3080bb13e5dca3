#!/usr/bin/env python3
"""Benchmark of the PMPD decode linear-layer path on one MI355X.

Workload: the Llama-7B-shaped decode step (32 blocks x {q,k,v,o 4096x4096, up/gate 11008x4096,
down 4096x11008}, batch 1, one token), seeded synthetic weights and activations, run at
b = 4, 3 and 2.  A "step" is one decoded token = one launch of the whole stack; K steps are timed at
each bit-width (fresh activations per step).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak


def cpu_baseline(shape, seed, bits, budget_s=15.0):
    """Time the CPU oracle (as it stands) on whole blocks of the stack: every row of the seven projections of
    block 0, then block 1, ... for as long as the budget lasts; the only scaling left is blocks done -> all blocks."""
    import oracle
    import pmpd_synth as synth

    threads = oracle.threads()
    t_per_b = {b: 0.0 for b in bits}
    done = 0
    weights_per_block = sum(o * i for _, o, i in shape.proj_shapes())
    t_start = time.perf_counter()
    for blk in range(shape.n_blocks):
        layers = []
        for pi, (nm, o, i) in enumerate(shape.proj_shapes()):
            q4, s, a = synth.draw_weights(seed, blk, pi, o, i)
            layers.append((q4, s, a, synth.draw_x(seed, 0, blk, pi, i)[0]))
        for b in bits:
            t0 = time.perf_counter()
            for (q4, s, a, x) in layers:
                oracle.linear(q4, s, a, b, x, want_budget=False)
            t_per_b[b] += time.perf_counter() - t0
        done += 1
        del layers
        if time.perf_counter() - t_start > budget_s:
            break
    scale = shape.n_blocks / done
    us = {b: t_per_b[b] * scale * 1e6 for b in bits}
    return {
        "value": sum(us.values()) / len(us),
        "unit": "us/token",
        "cores": threads,
        "kind": "oracle",
        "per_bits_us_per_token": {str(b): us[b] for b in us},
        "sample": f"every row of all 7 projections of the first {done} of {shape.n_blocks} blocks "
                  f"({done * weights_per_block} weights, one token) at each bit-width, times {scale:g} for the whole stack",
    }


def measured_traffic(b: int):
    """HBM bytes per launch from the committed rocprofv3 counter summary (separate --pmc runs), or None."""
    path = os.path.join(ROOT, "profiles", "decode_step_7b_stack_kernel.txt")
    try:
        for line in open(path):
            tok = line.split()
            if len(tok) >= 3 and tok[0] == "traffic_bytes" and tok[1] == f"b={b}":
                return float(tok[2])
    except OSError:
        pass
    return None


def _ramp(fn, seconds=0.5):
    """Run fn repeatedly for `seconds` so that the GPU clocks settle before anything is timed."""
    import torch

    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        fn()
        torch.cuda.synchronize()


def _timed(fn, n):
    """Mean milliseconds of n back-to-back calls of fn, HIP events on the current stream."""
    import torch

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    stream = torch.cuda.current_stream()
    torch.cuda.synchronize()
    e0.record(stream)
    for _ in range(n):
        fn()
    e1.record(stream)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n


# ---------------------------------------------------------------------------------------------
# The other workloads.  Each function measures one of them and returns a dict; `--workload NAME`
# prints it as a line of its own, and the default run gathers short forms of four of them under
# "secondary" (the benchmark line's own fields are not touched by that).
def _device_randn(n, seed):
    """fp16 ~N(0,1) activations drawn on the device (seeded): host RNG time stays out of the run."""
    import torch

    g = torch.Generator(device="cuda").manual_seed(seed)
    return torch.randn(n, device="cuda", generator=g, dtype=torch.float32).half()


def wl_schedule(pmpd, synth, stack, seed, reps):
    """configs[2]: 256 decode steps on the 7B-shaped stack, 64 at 4 bits, 96 at 3, 96 at 2."""
    import torch

    P, st, n_steps = synth.SCHEDULE_7B_256
    sch = pmpd.Schedule(P, st, n_steps)
    x = _device_randn(n_steps * stack.x_elems, seed + 1).view(n_steps, stack.x_elems)
    y = torch.zeros(stack.y_elems, dtype=torch.float32, device="cuda")
    run = lambda k0, n: pmpd.decode_run(stack, sch, k0, n, x[k0:], stack.x_elems, y, 0)
    _ramp(lambda: run(0, 64))
    phases = [(4, 0, 64), (3, 64, 96), (2, 160, 96)]
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(phases) + 1)]
    tot = {b: 0.0 for b, _, _ in phases}
    for _ in range(reps):
        ev[0].record()
        for j, (b, k0, n) in enumerate(phases):
            run(k0, n)
            ev[j + 1].record()
        torch.cuda.synchronize()
        for j, (b, _, _) in enumerate(phases):
            tot[b] += ev[j].elapsed_time(ev[j + 1])
    per, total_ms = {}, 0.0
    for b, k0, n in phases:
        ms = tot[b] / reps
        total_ms += ms
        gbps = stack.bytes_at(b) * n / (ms * 1e-3) / 1e9
        per[str(b)] = {"steps": n, "ms": ms, "us_per_token": ms * 1e3 / n, "GBps": gbps, "frac_of_peak": gbps / HBM_PEAK_GBS,
                       "launch_shape": stack.variant(b)}
    overall = sum(stack.bytes_at(b) * n for b, _, n in phases) / (total_ms * 1e-3) / 1e9
    res = {"workload": "Llama-7B-shaped stack, 256 decode steps, b per step from the schedule 64@4, 96@3, 96@2",
           "total_ms": total_ms, "avg_bits": sch.avg_bits(n_steps), "per_phase": per, "GBps_overall": overall,
           "frac_of_peak_overall": overall / HBM_PEAK_GBS, "repetitions": reps}
    sch.close()
    return res


def wl_single(pmpd, synth, seed, K):
    """configs[0]: one 4096 x 4096 layer, batch 1.  Latency of an isolated GEMV, and throughput when every launch
    reads weights that are not in the 256 MB cache (64 packed copies = 570 MB at b = 4)."""
    import torch

    o = i = 4096
    n_copies = 64
    q4, s_, a_ = synth.draw_weights(seed, 0, 0, o, i)
    planes, sm = pmpd.pack(q4, s_, a_)
    copies = [pmpd.upload_layer(planes, sm, o, i) for _ in range(n_copies)]
    x = torch.from_numpy(synth.draw_x(seed, 0, 0, 0, i)[0]).cuda()
    y = torch.zeros(o, dtype=torch.float32, device="cuda")
    # the same 64 copies as one list of layers: one launch keeps the memory pipe full across layer boundaries
    pipelined = pmpd.Stack(copies)
    xs = x.repeat(n_copies)
    ys = torch.zeros(pipelined.y_elems, dtype=torch.float32, device="cuda")
    res = {}
    for b in (4, 3, 2):
        warm = lambda: pmpd.gemv(copies[0], b, x, y)

        def cold():
            for c in copies:
                pmpd.gemv(c, b, x, y)

        _ramp(cold, 0.3)
        t_cold = _timed(cold, max(3, K // 5)) * 1e3 / n_copies
        _ramp(warm, 0.2)
        t_warm = _timed(warm, 10 * K) * 1e3
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(200):
            warm()
            torch.cuda.synchronize()
        t_iso = (time.perf_counter() - t0) / 200 * 1e6
        one = lambda: pmpd.decode_step(pipelined, b, xs, ys)
        _ramp(one, 0.2)
        t_pipe = _timed(one, K) * 1e3 / n_copies
        nbytes = copies[0].bytes_at(b)
        res[f"b{b}"] = {"cold_weights_us": t_cold, "cold_GBps": nbytes / (t_cold * 1e-6) / 1e9,
                        "warm_back_to_back_us": t_warm, "isolated_launch_and_sync_us": t_iso,
                        "pipelined_64_copies_one_launch_us": t_pipe,
                        "pipelined_GBps": nbytes / (t_pipe * 1e-6) / 1e9,
                        "pipelined_frac_of_peak": nbytes / (t_pipe * 1e-6) / 1e9 / HBM_PEAK_GBS,
                        "pipelined_launch_shape": pipelined.variant(b)}
    pipelined.close()
    return {"workload": "one 4096x4096 layer, batch 1; 64 packed copies rotated (cold weights) or listed in one launch (pipelined)",
            "results": res}


def wl_batches(pmpd, synth, workload, which, seed, K, batches=(1, 2, 3, 4, 8, 16), stacks=None):
    """configs[3] (which = "mobile": two distinct copies of the mobile-scale stack, alternated, so that no step finds
    its weights in the 256 MB cache) or the same skinny batches on the 7B-shaped stack (which = "batch7b")."""
    import torch

    own = stacks is None
    if own:
        if which == "batch7b":
            stacks = [workload.build_stack(synth.LLAMA_7B, seed=seed, verbose=True)[0]] * 2
        else:
            stacks = [workload.build_stack(synth.MOBILE, seed=seed + c)[0] for c in range(2)]
    res = {}
    for m in batches:
        X = _device_randn(m * stacks[0].x_elems, seed + 2)
        Y = torch.zeros(m * stacks[0].y_elems, dtype=torch.float32, device="cuda")
        for b in (4, 3, 2):
            # which matrix unit the library's batch step uses for this (m, b)
            unit = ("fp8 x fp4 scaled MFMA" if m <= 2 else "fp16 MFMA, codes as subnormals" if 9 <= m <= 16 or (5 <= m <= 16 and b == 4)
                    else "int8 MFMA" if m <= 16 else "fp16 MFMA")
            def step():
                for stc in stacks:
                    pmpd.batch_step(stc, b, X, m, Y)
            _ramp(step, 0.2)
            ms = _timed(step, K) / 2
            gbps = stacks[0].bytes_at(b) / (ms * 1e-3) / 1e9
            res[f"m{m}_b{b}"] = {"us_per_step": ms * 1e3, "GBps": gbps, "frac_of_peak": gbps / HBM_PEAK_GBS, "macs_on": unit}
    name = "mobile-scale stack (22 blocks, 2048/5632)" if which == "mobile" else "7B-shaped stack (32 blocks, 4096/11008)"
    out = {"workload": name + (", two alternating copies" if which == "mobile" else "") +
           ", batch " + "/".join(str(m) for m in batches) + " x b=4/3/2; GB/s counts the weights' bytes only",
           "launch_shape_batch1": {str(b): stacks[0].variant(b) for b in (4, 3, 2)}, "results": res}
    if own and which == "mobile":
        for stc in stacks:
            stc.close()
    return out


def wl_13b(pmpd, synth, workload, seed, K):
    """configs[4]: 13B-shaped stack, 512-token prefill at b = 4, then 128 decode steps 48 @ 3 bits + 80 @ 2 bits."""
    import torch

    shape = synth.LLAMA_13B
    stack, layers, _ = workload.build_stack(shape, seed=seed, verbose=True)
    m = 512
    X = _device_randn(m * stack.x_elems, seed + 3)
    Y = torch.zeros(m * stack.y_elems, dtype=torch.float32, device="cuda")
    pre = lambda: pmpd.prefill_step(stack, 4, X, m, Y)
    _ramp(pre, 0.5)
    ms_pre = _timed(pre, max(3, K // 10))
    flops = 2.0 * m * shape.n_weights()
    other = {}
    for b in (3, 2):  # the same prefill at the lower precisions (not part of the named workload: reported beside it)
        fn = lambda b=b: pmpd.prefill_step(stack, b, X, m, Y)
        fn()
        ms_b = _timed(fn, max(3, K // 10))
        other[f"b{b}"] = {"ms": ms_b, "TFLOPs": flops / (ms_b * 1e-3) / 1e12, "frac_of_2500_TFLOPs": flops / (ms_b * 1e-3) / 1e12 / 2500.0}
    P, st, n_steps = synth.SCHEDULE_13B_128
    sch = pmpd.Schedule(P, st, n_steps)
    xs = _device_randn(n_steps * stack.x_elems, seed + 4).view(n_steps, stack.x_elems)
    y = torch.zeros(stack.y_elems, dtype=torch.float32, device="cuda")
    dec = lambda: pmpd.decode_run(stack, sch, 0, n_steps, xs, stack.x_elems, y, 0)
    _ramp(dec, 0.5)
    ms_dec = _timed(dec, max(2, K // 20))
    dec_bytes = 48 * stack.bytes_at(3) + 80 * stack.bytes_at(2)
    res = {"workload": "13B-shaped stack (40 blocks, 5120/13824): 512-token prefill at b=4, then 128 decode steps 48@3 + 80@2",
           "prefill": {"ms": ms_pre, "TFLOPs": flops / (ms_pre * 1e-3) / 1e12,
                       "frac_of_2500_TFLOPs": flops / (ms_pre * 1e-3) / 1e12 / 2500.0, "other_precisions": other},
           "decode": {"ms": ms_dec, "avg_bits": sch.avg_bits(n_steps), "GBps": dec_bytes / (ms_dec * 1e-3) / 1e9,
                      "frac_of_peak": dec_bytes / (ms_dec * 1e-3) / 1e9 / HBM_PEAK_GBS,
                      "us_per_token": ms_dec * 1e3 / n_steps,
                      "launch_shape": {str(b): stack.variant(b) for b in (3, 2)}}}
    sch.close()
    stack.close()
    return res


def secondary_workload(args) -> int:
    """One of the other workloads as a JSON line of its own."""
    import numpy as np
    import torch

    import pmpd_synth as synth
    import paper_2410_13461_amd as pmpd
    from paper_2410_13461_amd import workload

    torch.cuda.set_device(0)
    K = args.steps
    out = {"n_gpus": 1, "data": "synthetic", "steps": K, "warmup": args.warmup}
    if args.workload == "schedule":
        stack, layers, _ = workload.build_stack(synth.LLAMA_7B, seed=args.seed, verbose=True)
        r = wl_schedule(pmpd, synth, stack, args.seed, max(1, K // 20))
        out.update({"metric": "total linear-layer time of the 256-step progressive schedule (64@4, 96@3, 96@2)",
                    "value": r["total_ms"], "unit": "ms", "higher_is_better": False, "config": {"workload": r.pop("workload")}})
        out.update(r)
    elif args.workload == "single":
        r = wl_single(pmpd, synth, args.seed, K)
        out.update({"metric": "single 4096x4096 layer, batch 1: us per GEMV (cold weights, warm back-to-back, isolated launch+sync, 64 copies in one launch)",
                    "unit": "us", "value": r["results"]["b4"]["cold_weights_us"], "higher_is_better": False,
                    "config": {"workload": r["workload"]}, "results": r["results"]})
    elif args.workload in ("mobile", "batch7b"):
        r = wl_batches(pmpd, synth, workload, args.workload, args.seed, K)
        out.update({"metric": "us per step at batch 1,2,3,4,8,16", "unit": "us/step",
                    "value": r["results"]["m1_b4"]["us_per_step"], "higher_is_better": False,
                    "config": {"workload": r["workload"]}, "launch_shape_batch1": r["launch_shape_batch1"], "results": r["results"]})
    elif args.workload == "13b":
        r = wl_13b(pmpd, synth, workload, args.seed, K)
        out.update({"metric": "13B-shaped stack: 512-token prefill at b=4 (ms) then 128 decode steps 48@3 + 80@2 (ms)",
                    "unit": "ms", "value": r["prefill"]["ms"] + r["decode"]["ms"], "higher_is_better": False,
                    "config": {"workload": r["workload"]}, "prefill": r["prefill"], "decode": r["decode"]})
    elif args.workload == "alternate":
        # The paper rejects per-token switching because of the cost of swapping weights in its system
        # (Section 3.2); with the nested plane store a switch is only a different launch argument.
        shape = synth.LLAMA_7B
        stack, layers, _ = workload.build_stack(shape, seed=args.seed, verbose=True)
        n_steps = 256
        x = torch.from_numpy(np.stack([workload.draw_step_activations(shape, args.seed, k) for k in range(8)])).cuda()
        y = torch.zeros(stack.y_elems, dtype=torch.float32, device="cuda")
        stream = torch.cuda.current_stream()

        def run(bits_of_step):
            for k in range(n_steps):
                pmpd.decode_step(stack, bits_of_step(k), x[k % 8], y, stream)

        res = {}
        for name, f in (("b4", lambda k: 4), ("b2", lambda k: 2), ("alternating_4_2", lambda k: 4 if k % 2 == 0 else 2),
                        ("cycling_4_3_2", lambda k: 4 - k % 3)):
            _ramp(lambda: run(f), 0.5)
            reps = max(1, K // 50)
            res[name] = _timed(lambda: run(f), reps) * 1e3 / n_steps  # us per token
        out.update({"metric": "us/token when the bit-width changes at every step, against the fixed-precision runs",
                    "unit": "us/token", "value": res["alternating_4_2"], "higher_is_better": False,
                    "config": {"workload": "Llama-7B-shaped stack, 256 decode steps per run, b switched every token"},
                    "results": res,
                    "switching_overhead_us": res["alternating_4_2"] - 0.5 * (res["b4"] + res["b2"])})
    elif args.workload == "ordered":
        # Dependency order of a decoder block: (q, k, v) -> o -> (up, gate) -> down, block after block:
        # one launch per stage, 4 x 32 launches per token, eager and as a replayed graph.  The glue
        # between the stages (attention, norms, activation) is not part of this path: only the order
        # of the launches is enforced, every layer keeps its own input buffer.
        shape = synth.LLAMA_7B
        stack, layers, _ = workload.build_stack(shape, seed=args.seed, verbose=True)
        stages = ((0, 1, 2), (3,), (4, 6), (5,))  # projection indices q,k,v,o,up,down,gate
        stage_stacks = []
        for blk in range(shape.n_blocks):
            for st_ in stages:
                idx = [blk * 7 + pi for pi in st_]
                stage_stacks.append(pmpd.Stack([layers[i] for i in idx], [stack.x_offsets[i] for i in idx],
                                               [stack.y_offsets[i] for i in idx]))
        # the same order inside one cooperative launch, first with every layer on its own input (the
        # same arithmetic as the launches above), then with the data really flowing from layer to
        # layer: o <- q, (up, gate) <- o, down <- up, next block <- down, x = fp16(gain * y)
        n_layers = len(layers)
        stage_of = [4 * (li // 7) + {0: 0, 1: 0, 2: 0, 3: 1, 4: 2, 6: 2, 5: 3}[li % 7] for li in range(n_layers)]
        src_of = []
        for li in range(n_layers):
            blk, pi = divmod(li, 7)
            src_of.append({0: 7 * blk - 2, 1: 7 * blk - 2, 2: 7 * blk - 2, 3: 7 * blk, 4: 7 * blk + 3, 6: 7 * blk + 3,
                           5: 7 * blk + 4}[pi] if (blk or pi > 2) else -1)
        # y has std sqrt(in) * 0.028 for unit-variance x (a = -8 s, uniform codes): the gain undoes it
        gain_of = [1.0 if k < 0 else 1.0 / (0.028 * layers[li].in_features ** 0.5) for li, k in enumerate(src_of)]
        persistent_free = pmpd.Ordered(stack, stage_of, [-1] * n_layers, [1.0] * n_layers)
        persistent_chain = pmpd.Ordered(stack, stage_of, src_of, gain_of)
        x = torch.from_numpy(workload.draw_step_activations(shape, args.seed, 0)).cuda()
        y = torch.zeros(stack.y_elems, dtype=torch.float32, device="cuda")
        y_ref = torch.zeros_like(y)
        res = {}
        for b in (4, 3, 2):
            def step():
                for ss in stage_stacks:
                    pmpd.decode_step(ss, b, x, y)
            pmpd.decode_step(stack, b, x, y_ref)
            step()
            torch.cuda.synchronize()
            same = bool(torch.equal(y, y_ref))  # same kernels' arithmetic per row: bit-identical is expected only per launch shape
            close = bool(torch.allclose(y, y_ref, rtol=1e-4, atol=1e-4))
            _ramp(step, 0.3)
            eager = _timed(step, max(3, K // 10)) * 1e3
            graph, replays = None, []
            if not args.no_graph:
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    step()
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g, stream=side):
                        step()
                torch.cuda.current_stream().wait_stream(side)
                torch.cuda.synchronize()
                for _ in range(3):  # every replay is checked against the eager result
                    y.zero_()
                    g.replay()
                    torch.cuda.synchronize()
                    replays.append(bool(torch.allclose(y, y_ref, rtol=1e-4, atol=1e-4)))
                _ramp(g.replay, 0.3)
                graph = _timed(g.replay, max(3, K // 10)) * 1e3
            _ramp(lambda: pmpd.decode_step(stack, b, x, y), 0.3)
            one = _timed(lambda: pmpd.decode_step(stack, b, x, y), K) * 1e3
            y.zero_()
            persistent_free.step(b, x, y)
            torch.cuda.synchronize()
            pers_ok = bool(torch.allclose(y, y_ref, rtol=1e-4, atol=1e-4)) and not persistent_free.timed_out()
            _ramp(lambda: persistent_free.step(b, x, y), 0.3)
            pers = _timed(lambda: persistent_free.step(b, x, y), K) * 1e3
            _ramp(lambda: persistent_chain.step(b, x, y), 0.3)
            chain = _timed(lambda: persistent_chain.step(b, x, y), K) * 1e3
            torch.cuda.synchronize()
            chain_ok = bool(torch.isfinite(y).all()) and not persistent_chain.timed_out()
            res[f"b{b}"] = {"one_launch_us": one, "ordered_eager_us": eager, "ordered_graph_us": graph,
                            "ordered_one_cooperative_launch_us": pers, "ordered_chained_inputs_us": chain,
                            "matches_one_launch": close, "bit_identical": same, "graph_replays_match": all(replays) if replays else None,
                            "cooperative_matches_one_launch": pers_ok, "chained_finite_and_no_timeout": chain_ok}
        # nothing of this branch is left for the interpreter's exit handlers to tear down
        persistent_free.close()
        persistent_chain.close()
        for ss in stage_stacks:
            ss.close()
        stack.close()
        g = None
        out.update({"metric": "us/token of the 7B-shaped step launched in dependency order (128 stage launches) vs one launch",
                    "unit": "us/token", "value": res["b4"]["ordered_chained_inputs_us"], "higher_is_better": False,
                    "config": {"workload": "Llama-7B-shaped stack, stages (q,k,v) -> o -> (up,gate) -> down per block"},
                    "results": res})
    elif args.workload == "learned":
        # learned scheduler, once per prompt: key / value cache of one block of a 7B-shaped model (32 heads x 128),
        # hidden layer of 256 units, 5 candidate switch points; random parameters (trained ones are not public)
        d, hidden, n_cls = 4096, 256, 5
        res = {}
        for T in (128, 512, 2048, 8192):
            Kh, Vh, q, W1, b1, W2, b2 = synth.draw_learned_scheduler(args.seed, T, d, d, hidden, n_cls)
            net = pmpd.LearnedScheduler(q, W1, b1, W2, b2)
            cache_bytes = 2 * T * (d + d)
            copies = max(2, min(64, (640 << 20) // cache_bytes))  # rotate over more than the 256 MiB last-level cache
            Ks = [torch.from_numpy(Kh).cuda() for _ in range(copies)]
            Vs = [torch.from_numpy(Vh).cuda() for _ in range(copies)]
            probs = torch.empty(n_cls, dtype=torch.float32, device="cuda")
            cls = torch.empty(1, dtype=torch.int32, device="cuda")
            ctx = torch.empty(d, dtype=torch.float32, device="cuda")
            state = {"i": 0}

            def call():
                i = state["i"] = (state["i"] + 1) % copies
                net.forward(Ks[i], Vs[i], probs, cls, ctx)

            _ramp(call, 0.3)
            ms = _timed(call, max(K, copies))
            warm = lambda: net.forward(Ks[0], Vs[0], probs, cls, ctx)
            ms_warm = _timed(warm, K)
            import oracle  # bench-side check of the last result against the CPU definition
            O_ref, p_ref, c_ref = oracle.learned_scheduler(q, Kh, Vh, W1, b1, W2, b2)
            torch.cuda.synchronize()
            ok = bool(np.max(np.abs(probs.cpu().numpy() - p_ref)) <= 1e-4 and int(cls.item()) == int(np.argmax(probs.cpu().numpy())))
            res[f"T{T}"] = {"us_per_call_cold_cache": ms * 1e3, "us_per_call_warm_cache": ms_warm * 1e3,
                            "cache_bytes": cache_bytes, "GBps_cold": cache_bytes / (ms * 1e-3) / 1e9,
                            "matches_oracle": ok}
            del Ks, Vs
        out.update({"metric": "learned scheduler forward pass, us per prompt (K/V cache of one 7B-shaped block, fp16)",
                    "unit": "us/prompt", "value": res["T512"]["us_per_call_cold_cache"], "higher_is_better": False,
                    "config": {"workload": f"d_k = d_v = {d}, hidden {hidden}, {n_cls} classes, T = 128/512/2048/8192; "
                                           "five kernels per call, back-to-back calls on rotating cache copies"},
                    "results": res})
    else:
        print(f"unknown workload {args.workload}", file=sys.stderr)
        return 2
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--blocks", type=int, default=None, help="debug: fewer blocks (result is then not the named workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true", help="default workload: skip the 'secondary' object (the other configurations)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-graph", action="store_true", help="ordered workload: skip the HIP-graph replay of the stage launches (the profiler's exit handler crashes after captured graphs)")
    ap.add_argument("--workload", default="7b", choices=["7b", "schedule", "alternate", "ordered", "single", "mobile", "batch7b", "13b", "learned"],
                    help="7b (default) is the benchmark line; the others print a line for the secondary workloads")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import pmpd_synth as synth
    import paper_2410_13461_amd as pmpd
    from paper_2410_13461_amd import workload

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    if args.workload != "7b":
        return secondary_workload(args)
    torch.cuda.set_device(0)
    shape = synth.LLAMA_7B
    bits = (4, 3, 2)
    K, W = args.steps, args.warmup

    t0 = time.time()
    stack, layers, _ = workload.build_stack(shape, seed=args.seed, n_blocks=args.blocks, verbose=True)
    print(f"stack ready: {len(layers)} layers in {time.time() - t0:.0f} s", file=sys.stderr, flush=True)

    # activations of every step already on the device
    xs = np.stack([workload.draw_step_activations(shape, args.seed, k, n_blocks=args.blocks) for k in range(W + K)])
    x_dev = torch.from_numpy(xs).cuda()
    y_dev = torch.zeros(stack.y_elems, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    # The GPU idles at a few hundred MHz and needs some tenths of a second of work before its
    # clocks settle: run untimed steps for that long first, then the W warm-up steps proper.
    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < 0.5:
        for b in bits:
            pmpd.decode_step(stack, b, x_dev[0], y_dev, stream)
        torch.cuda.synchronize()

    # PMPD lowers the precision progressively, so steps of one bit-width come in long runs:
    # each bit-width gets its own W warm-up steps and K timed steps, back to back.
    per_b_ms = {b: [] for b in bits}
    total_ms = 0.0
    t_wall = 0.0
    for b in bits:
        for k in range(W):
            pmpd.decode_step(stack, b, x_dev[k], y_dev, stream)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
        torch.cuda.synchronize()
        t0w = time.perf_counter()
        ev[0].record(stream)
        for k in range(K):
            pmpd.decode_step(stack, b, x_dev[W + k], y_dev, stream)
            ev[k + 1].record(stream)
        torch.cuda.synchronize()
        t_wall += time.perf_counter() - t0w
        per_b_ms[b] = [ev[k].elapsed_time(ev[k + 1]) for k in range(K)]
        total_ms += ev[0].elapsed_time(ev[K])

    per_bits = {}
    for b in bits:
        ms = float(np.mean(per_b_ms[b]))
        nbytes = stack.bytes_at(b)
        per_bits[str(b)] = {
            "us_per_token": ms * 1e3,
            "median_us": float(np.median(per_b_ms[b])) * 1e3,
            "min_us": float(np.min(per_b_ms[b])) * 1e3,
            "algorithmic_bytes": nbytes,
            "GBps": nbytes / (ms * 1e-3) / 1e9,
            "frac_of_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        }
    us_per_token = total_ms * 1e3 / (K * len(bits))

    # the rate a plain read-only stream reaches on this machine over the same number of bytes
    buf = torch.empty(stack.bytes_at(4) // 4, dtype=torch.int32, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    nread = pmpd.read_stream(buf, sink, stream)
    _ramp(lambda: pmpd.read_stream(buf, sink, stream), 0.3)
    stream_ms = _timed(lambda: pmpd.read_stream(buf, sink, stream), 50)
    stream_gbps = nread / (stream_ms * 1e-3) / 1e9
    del buf
    for b in bits:
        per_bits[str(b)]["frac_of_read_stream"] = per_bits[str(b)]["GBps"] / stream_gbps

    # the unquantised fp16 matrix-vector kernel over the same shapes (2 bytes per weight), one launch per token:
    # the denominator of the paper's speedup figures (Section 5.2, Table 3), measured here on this device
    gen = torch.Generator(device="cuda").manual_seed(args.seed)
    n_blocks = shape.n_blocks if args.blocks is None else args.blocks
    dW = [torch.empty(o, i, dtype=torch.float16, device="cuda").normal_(0.0, 0.02, generator=gen)
          for _ in range(n_blocks) for (_, o, i) in shape.proj_shapes()]
    ref = pmpd.Fp16Stack(dW)
    y_ref = torch.zeros(ref.y_elems, dtype=torch.float32, device="cuda")
    _ramp(lambda: pmpd.fp16_step(ref, x_dev[0], y_ref, stream), 0.3)
    for k in range(W):
        pmpd.fp16_step(ref, x_dev[k], y_ref, stream)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    ev[0].record(stream)
    for k in range(K):
        pmpd.fp16_step(ref, x_dev[W + k], y_ref, stream)
    ev[1].record(stream)
    torch.cuda.synchronize()
    ref_us = ev[0].elapsed_time(ev[1]) * 1e3 / K
    ref_bytes = ref.weight_bytes() + 2 * ref.x_elems + 4 * ref.y_elems
    fp16_reference = {
        "kernel": "fp16_stack_kernel (unquantised fp16 weights, same shapes, one launch per token)",
        "us_per_token": ref_us,
        "algorithmic_bytes": ref_bytes,
        "GBps": ref_bytes / (ref_us * 1e-6) / 1e9,
        "frac_of_peak": ref_bytes / (ref_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
        "speedup_over_fp16": {str(b): ref_us / per_bits[str(b)]["us_per_token"] for b in bits},
    }
    ref.close()
    del dW, ref

    dom = per_bits["4"]
    props = torch.cuda.get_device_properties(0)
    out = {
        "metric": "decode linear-layer us/token (mean over b=4,3,2; per-bit figures in per_bits), batch 1",
        "value": us_per_token,
        "unit": "us/token",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": total_ms / (K * len(bits)),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u4 bit-plane weights as fp4 pairs x f16 activations as 3 exact fp8 pieces, f32 accumulate",
        "data": "synthetic",
        "config": {
            "workload": "Llama-7B-shaped decode step: 32 blocks x 7 projections (224 linear layers, 6.476e9 weights), "
                        "batch 1, one token per launch, run at b=4,3,2" if args.blocks is None else f"DEBUG {args.blocks} blocks",
            "group_size": 128,
            "step": "one decode token (one launch); K timed steps at each of b=4,3,2, the three runs back to back",
            "wall_ms_per_step_incl_host": t_wall * 1e3 / (K * len(bits)),
        },
        "per_bits": per_bits,
        "device": {"name": props.name, "compute_units": props.multi_processor_count, "hbm_bytes": props.total_memory,
                   "gcn_arch": getattr(props, "gcnArchName", "")},
        "fp16_reference": fp16_reference,
        "roofline": {
            "bound": "hbm",
            "kernel": "pmpd_stack_kernel<B=4, SETS=1, NW=4, SPLITK=1> (one launch = one b=4 decode step)"
                      if stack.variant(4) == 0 else f"pmpd_stack_kernel<B=4>, launch shape {stack.variant(4)}",
            "launch_shape": {str(b): stack.variant(b) for b in bits},
            "achieved": dom["GBps"],
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": dom["GBps"] / HBM_PEAK_GBS,
            "traffic": measured_traffic(4) if args.blocks is None else None,
            "read_stream_GBps": stream_gbps,
            "frac_of_read_stream": dom["GBps"] / stream_gbps,
        },
    }
    if not args.no_secondary and args.blocks is None:
        # The other configurations, measured in the same run (each with its own warm-up; stacks smaller than the
        # 256 MB cache are rotated).  Parity of exactly these stacks and calls: tests/test_gpu_full_size.py.
        sec = {}
        print("secondary: 256-step schedule on the 7B stack", file=sys.stderr, flush=True)
        sec["schedule_256_steps_7b"] = wl_schedule(pmpd, synth, stack, args.seed, max(2, K // 20))
        stack.close()
        del stack, layers, x_dev
        torch.cuda.empty_cache()
        print("secondary: single 4096x4096 layer", file=sys.stderr, flush=True)
        sec["single_layer_4096"] = wl_single(pmpd, synth, args.seed, K)
        print("secondary: mobile-scale stack, batches", file=sys.stderr, flush=True)
        sec["mobile_stack_batches"] = wl_batches(pmpd, synth, workload, "mobile", args.seed, K, batches=(1, 2, 4, 8, 16))
        print("secondary: 13B-shaped stack, prefill + decode", file=sys.stderr, flush=True)
        sec["prefill_and_decode_13b"] = wl_13b(pmpd, synth, workload, args.seed, K)
        out["secondary"] = sec
    else:
        stack.close()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, args.seed, bits)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
