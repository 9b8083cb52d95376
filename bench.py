#!/usr/bin/env python3
"""Benchmark of the interruptible-decoding hot path on one MI355X.

One "step" of this benchmark is one pass of the whole hot path of the 8B-shaped workload:
BLOCK greedy decoding steps at batch 1 (token chosen on the device, read back by the host as
the paper's token monitor needs it) followed by one in-flight injection of an interrupt block
into the live K/V cache.  The default workload is the Llama-3-8B-shaped preset: bf16,
1024-token prompt, 24-token interrupts every 64 decoding steps.

Prints ONE JSON line:
  value          generated tokens per second over the timed steps, injections included
  decode_*       decode-only rate and its fraction of the HBM roofline (algorithmic bytes / time / 8 TB/s);
                 10th / 50th / 90th percentile of the single steps (an event after every step)
  inject_*       microseconds per interrupt (mean; min / median / max), its cost in decoding steps and its fraction
                 of the HBM roofline (one pass over the same weights and cache)
  prefill_*      seconds for the prompt and the fraction of the bf16 matrix-core peak that 2 flop per weight and
                 token amount to
  reprefill_*, kv_swap_*, merged_*   the stateless re-prefill of the same context (Sec. 5.5), the K/V swap of a
                 trapped session (Sec. 5.4) and the interrupt riding with the next token (Sec. 5.3)
  streaming_read_ceiling   what the longest plain stream of the step (the output head) reaches on this device
  roofline       dominant kernel (gate/up projection + SwiGLU): algorithmic bytes per launch over its mean duration
                 measured here with HIP events on the library's stream around every launch of real decoding steps (the
                 launch gap is inside that figure); roofline.trace repeats it with the kernel's mean duration in the
                 committed rocprofv3 kernel trace of this command (profiles/8b_bench_kernel_stats.md)
  other_workloads   the recorded lines of `bench.py --workload W --record` for the other presets (profiles/*_bench_line.md)
  cpu_baseline   the CPU oracle timed on this host on a bounded sample (a baseline, not a target)
Other modes: --trap-map (Sec. 5.4 swap against recomputation), --e2e-calls N (Sec. 6.3 synchronous against
asynchronous calling, measured end to end next to the latency model).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12  # bytes/s, MI355X published peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="8b", choices=["tiny", "8b", "8b-long", "8b-ragged16", "70b"])
    ap.add_argument("--layers", type=int, default=0, help="truncate the model (0 = full depth); for experiments only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--chunk", type=int, default=0, help="override the library's rows per forward pass for prefill/inject")
    ap.add_argument("--opt", action="append", default=[], help="library option name=value (repeatable), for experiments")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain device copies of 1 GiB (torch copy kernel) so that a counter run can be scaled by them")
    ap.add_argument("--trap-map", action="store_true",
                    help="instead of the benchmark: time K/V swap-out + swap-in against recomputation (re-prefill) over a range of "
                         "context lengths (Sec. 5.4 trade-off) and print them as one JSON line")
    ap.add_argument("--e2e-calls", type=int, default=0,
                    help="instead of the benchmark: N scripted function calls with timer-backed executions, run synchronously "
                         "and asynchronously through the library, against the latency model of Sec. 6.3 (one JSON line)")
    ap.add_argument("--fused", type=int, default=-1, help="1/0: force the single-kernel / per-operation decoding step (default: library's choice)")
    ap.add_argument("--kv-format", type=int, default=0, help="cache format of the library (0 default, 1 single bf16 plane, 2 pairs with row-major values as well)")
    ap.add_argument("--step-timeline", action="store_true",
                    help="instead of the benchmark: the decoding step on one stream and on two streams (option \"pipeline\") on the same "
                         "context, with the device time stamps of every kernel of one two-stream step, as one JSON line")
    ap.add_argument("--record", action="store_true",
                    help="also write the JSON line, with its command, to profiles/<workload>_bench_line.md (the default run quotes those files)")
    return ap.parse_args()


def trace_duration_us(kernel_row):
    """Mean duration (us) of a kernel in the committed rocprofv3 kernel-trace summary of the default command: the `avg us`
    column of the row of profiles/8b_bench_kernel_stats.md that starts with `kernel_row`, or None."""
    try:
        for line in open(os.path.join(ROOT, "profiles", "8b_bench_kernel_stats.md")):
            if line.startswith("| " + kernel_row):
                return float(line.split("|")[4])
    except (OSError, ValueError, IndexError):
        pass
    return None


def recorded_lines():
    """The committed lines of the other workloads (written by --record), keyed by workload."""
    out = {}
    pdir = os.path.join(ROOT, "profiles")
    for name in sorted(os.listdir(pdir)) if os.path.isdir(pdir) else []:
        if not name.endswith("_bench_line.md"):
            continue
        try:
            text = open(os.path.join(pdir, name)).read().splitlines()
            line = next(l for l in text if l.startswith('{"metric"'))
            cmd = next((l.strip() for l in text if l.strip().startswith("python bench.py")), None)
            d = json.loads(line)
            keep = ("value", "unit", "ms_per_step", "steps", "decode_tokens_per_s", "decode_ms_per_token", "decode_hbm_frac", "inject_us",
                    "inject_tokens", "inject_in_decode_steps", "inject_hbm_frac", "batch_ms_per_step", "batch_hbm_frac", "prefill_s",
                    "reprefill_us", "reprefill_over_inject")
            out[name[:-len("_bench_line.md")]] = dict({k: d[k] for k in keep if k in d}, workload=d["config"]["workload"], command=cmd)
        except (OSError, ValueError, KeyError, StopIteration):
            continue
    return out


def emit(args, out):
    line = json.dumps(out)
    if args.record:
        cmd = "python bench.py " + " ".join(a for a in sys.argv[1:] if a != "--record")
        path = os.path.join(ROOT, "profiles", "%s_bench_line.md" % args.workload.replace("-", "_"))
        with open(path, "w") as f:
            f.write("# bench.py line of the %s workload (one MI355X; written by --record)\n\nCommand:\n\n    %s\n\nLine:\n\n%s\n" % (args.workload, cmd, line))
    print(line)


def recorded_traffic(model):
    """HBM bytes per launch of the gate/up kernel from the committed hardware-counter record, or None when the
    record is for another shape or the kernel's sources have changed since the counters were taken."""
    import hashlib
    path = os.path.join(ROOT, "traffic_gate_up.json")
    try:
        rec = json.load(open(path))
        h = hashlib.sha256()
        for f in rec["source_files"]:
            h.update(open(os.path.join(ROOT, f), "rb").read())
        if h.hexdigest() != rec["sources_sha256"] or (model.d_model, model.ffn, model.dtype) != (4096, 14336, "bf16"):
            return None
        return float(rec["fetch_bytes_per_launch"] + rec["write_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        return None


def cpu_baseline(wl, model, w_dev, spec, seconds_budget=25.0):
    """Times the oracle's cached decoder (fp32 numpy) on this host: decode steps on 4- and 8-layer
    truncations of the same weights, extrapolated linearly in depth to the full model."""
    import numpy as np
    import torch
    import asynclm_inputs as ai
    from oracle import asynclm_oracle as orc
    try:
        import threadpoolctl
        threads = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=1)
    except Exception:
        threads = os.cpu_count() or 1
    conv = lambda t: t.detach().to("cpu").to(torch.float32).numpy()
    depth = min(8, model.n_layers)
    w = {k: conv(w_dev[k]) for k in ("embed", "final_norm", "lm_head")}
    for k in ("attn_norm", "wqkv", "wo", "ffn_norm", "wgate_up", "wdown"):
        w[k] = [conv(t) for t in w_dev[k][:depth]]
    P = min(256, len(spec["prompt"]))
    times = {}
    t_begin = time.perf_counter()
    depths = sorted({max(depth // 2, 1), depth})
    for nl in depths:
        sh = orc.Shape.of(ai.truncated(model, nl))
        dec = orc.CachedDecoder(sh, w, dtype=np.float32)
        dec.prefill(spec["prompt"][:P])
        dec.decode_step()                                   # warm the BLAS threads
        n, t0 = 0, time.perf_counter()
        while n < 4 or time.perf_counter() - t0 < seconds_budget / (2 * len(depths)):
            dec.decode_step()
            n += 1
        times[nl] = (time.perf_counter() - t0) / n
    ks = sorted(times)
    if len(ks) == 2:
        per_layer = max((times[ks[1]] - times[ks[0]]) / (ks[1] - ks[0]), 0.0)
        head = max(times[ks[1]] - per_layer * ks[1], 0.0)
    else:
        per_layer, head = times[ks[0]] / ks[0], 0.0
    full = per_layer * model.n_layers + head
    return {
        "value": 1.0 / full, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
        "sample": "oracle CachedDecoder (numpy fp32, BLAS matmuls) decode steps after a %d-token prompt on %s-layer "
                  "truncations of the same weights (%s s/step), extrapolated linearly to %d layers + output head; "
                  "%.1f s of CPU work" % (P, "/".join(map(str, ks)), "/".join("%.3f" % times[k] for k in ks),
                                          model.n_layers, time.perf_counter() - t_begin),
    }


def bench_ragged(args):
    """The 16-sequence preset: every step is one asynclm_step_batch call (one pass over the weights for all
    sequences; the interrupts that arrived after the previous token ride with the chosen tokens).  A bench
    "step" is one such batched step; value = generated tokens per second summed over the sequences."""
    import numpy as np
    import torch
    import asynclm_inputs as ai
    import paper_2412_07017_amd as pkg
    wl = ai.preset(args.workload)
    model = wl.model if not args.layers else ai.truncated(wl.model, args.layers)
    spec = ai.build_workload(args.workload)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    t0 = time.perf_counter()
    w_dev = ai.make_weights(model, device=dev)
    torch.cuda.synchronize()
    t_weights = time.perf_counter() - t0
    stream = torch.cuda.Stream(device=dev)
    ns = wl.n_seqs
    n_steps = min(args.warmup + args.steps, spec["n_decode"])
    grow = [n_steps + sum(len(t) for ev in spec["step_events"][:n_steps] for s, t in ev if s == q) for q in range(ns)]
    max_pos = max(len(p) + g for p, g in zip(spec["prompts"], grow)) + 8
    lm = pkg.AsyncLM(model, w_dev, max_positions=max_pos, max_seqs=ns, stream=stream, kv_format=args.kv_format)
    for kv in args.opt:
        k, v = kv.split("=")
        lm.set_option(k, int(v))
    t0 = time.perf_counter()
    for q, p in enumerate(spec["prompts"]):
        lm.prefill(q, p)
    lm.synchronize()
    t_prefill = time.perf_counter() - t0
    seqs = list(range(ns))

    def step(t):
        ev = dict(spec["step_events"][t])
        return lm.step_batch(seqs, None, [ev.get(q, []) for q in seqs])

    for t in range(args.warmup):
        step(t)
    lm.synchronize()
    len_start = sum(lm.seq_len(q) for q in seqs)
    rows = 0
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record(stream)
    for t in range(args.warmup, n_steps):
        step(t)
        rows += ns + sum(len(x) for _, x in spec["step_events"][t])
    e1.record(stream)
    lm.synchronize()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    len_end = sum(lm.seq_len(q) for q in seqs)
    timed = n_steps - args.warmup
    ms_step = e0.elapsed_time(e1) / timed
    bytes_step = model.weight_bytes_per_step() + (len_start + len_end) / 2.0 * model.kv_bytes_per_position() + ns * 4 * model.vocab
    ach = bytes_step / (ms_step * 1e-3)
    out = {
        "metric": "decode tokens/s @ batch 1 (% HBM roofline); us per k-token interrupt inject",
        "value": timed * ns / wall, "unit": "tokens/s", "n_gpus": 1, "steps": timed, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / timed, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 accumulate over %s weights and K/V" % model.dtype, "data": "synthetic",
        "config": {"workload": "%s: %d layers, d %d, %dq/%dkv heads x %d, ffn %d, vocab %d, %s; %d sequences, contexts %d..%d "
                               "tokens; step = one batched step (chosen tokens + the interrupts of 16-32 tokens that arrived, "
                               "p = 0.05 per sequence and step) in one pass over the weights"
                               % (wl.name, model.n_layers, model.d_model, model.n_q_heads, model.n_kv_heads, model.head_dim,
                                  model.ffn, model.vocab, model.dtype, ns, min(map(len, spec["prompts"])), max(map(len, spec["prompts"]))),
                   "context_tokens_total": [len_start, len_end], "rows_per_step": rows / timed, "seed": ai.MASTER_SEED},
        "batch_ms_per_step": ms_step, "batch_hbm_frac": ach / HBM_PEAK, "batch_bytes_per_step": bytes_step,
        # the same with the K/V bytes that the attention actually reads (the cache keeps every value as two bf16 planes)
        "batch_hbm_frac_as_stored": (bytes_step + (len_start + len_end) / 2.0 * model.kv_bytes_per_position())
                                    / (ms_step * 1e-3) / HBM_PEAK if model.dtype == "bf16" else ach / HBM_PEAK,
        "prefill_s": t_prefill, "weights_s": t_weights,
        "roofline": {"bound": "hbm", "kernel": "whole batched step (all kernels of one pass)", "achieved": ach / 1e9,
                     "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": ach / HBM_PEAK, "traffic": None,
                     "bytes_per_launch": bytes_step, "ms_per_launch": ms_step},
    }
    lm.close()
    emit(args, out)


def step_timeline(args):
    """The two ways to run a decoding step, on the same model and context: one stream (kernel boundaries between
    dependent kernels) and two streams (neighbouring kernels overlap and hand over through counters in device
    memory).  Per kernel of one two-stream step: when it started, when it saw the previous kernel's hand-over, when its
    first and its last workgroup were done (100 MHz device clock, microseconds from the step's first kernel).  Per
    kernel of one layer of a one-stream step: start and input vector staged of the first and the last workgroup, done
    of the earliest and the latest workgroup (microseconds from that layer's first kernel)."""
    import numpy as np
    import torch
    import asynclm_inputs as ai
    import paper_2412_07017_amd as pkg
    wl = ai.preset(args.workload)
    model = wl.model if not args.layers else ai.truncated(wl.model, args.layers)
    spec = ai.build_workload(args.workload)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w_dev = ai.make_weights(model, device=dev)
    stream = torch.cuda.Stream(device=dev)
    n = 64
    # the single-row attention kernel of the two-stream step reads the values row by row: a cache format of its own
    lm = pkg.AsyncLM(model, w_dev, max_positions=wl.prompt_len + 4 * n + 64, stream=stream, kv_format=pkg.KV_PAIR_ROWS)
    lm.prefill(0, spec["prompt"])
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def timed():
        for _ in range(8):
            lm.decode_step(0)
        lm.synchronize()
        e0, e1 = ev(), ev()
        e0.record(stream)
        for _ in range(n):
            lm.decode_step(0)
        e1.record(stream)
        lm.synchronize()
        return e0.elapsed_time(e1) / n

    one = timed()
    # the same one-stream step with time stamps
    lm.set_option("step_stamps", 1)
    for _ in range(4):
        lm.decode_step(0)
    lm.synchronize()
    tr1 = lm.profile_trace().astype(np.int64)           # [3 x kernels][first | last workgroup]
    lm.set_option("step_stamps", 0)
    nk1 = tr1.shape[0] // 3
    t1 = (tr1.reshape(nk1, 3, 2) - tr1[0, 0]) / 100.0
    names1 = ["qkv", "attention", "attention_merge", "o_proj", "gate_up", "down"]
    mid = 6 * (model.n_layers // 2)
    rows1 = [{"kernel": names1[k % 6], "layer": k // 6,
              "start_us": [round(float(v - t1[mid, 0, 0]), 2) for v in t1[k, 0]],
              "vector_staged_us": ([round(float(v - t1[mid, 0, 0]), 2) for v in t1[k, 1]] if k % 6 not in (1, 2) else None),
              "done_first_last_us": [round(float(v - t1[mid, 0, 0]), 2) for v in t1[k, 2]]} for k in range(mid, min(mid + 7, nk1))]
    one_per_layer = float(t1[6 * (model.n_layers - 1), 0, 0] - t1[6, 0, 0]) / max(model.n_layers - 2, 1) if model.n_layers > 2 else None
    lm.set_option("pipeline", 1)
    two = timed()
    tr = lm.profile_trace().astype(np.int64)            # [3 x kernels][first | last workgroup]
    nk = tr.shape[0] // 3
    t = (tr.reshape(nk, 3, 2) - tr[0, 0]) / 100.0
    names = ["qkv", "attention", "o_proj", "gate_up", "down"]
    rows = [{"kernel": (names[k % 5] if k < 5 * model.n_layers else "lm_head"), "layer": min(k // 5, model.n_layers - 1),
             "start_us": round(float(t[k, 0, 0]), 2), "handover_seen_us": round(float(t[k, 1].max()), 2),
             "first_done_us": round(float(t[k, 2, 0]), 2), "last_done_us": round(float(t[k, 2, 1]), 2)} for k in range(nk)]
    per_layer = (t[5 * (model.n_layers - 1), 1].max() - t[5, 1].max()) / max(model.n_layers - 2, 1) if model.n_layers > 2 else None
    lm.close()
    print(json.dumps({"step_timeline": args.workload, "layers": model.n_layers, "context": wl.prompt_len + 2 * n,
                      "one_stream_ms_per_token": one, "two_streams_ms_per_token": two, "two_streams_us_per_layer": per_layer,
                      "one_stream_us_per_layer": one_per_layer, "kernels_of_one_layer_of_a_one_stream_step": rows1,
                      "kernels_of_one_two_stream_step": rows[:15] + rows[-6:]}))


def trap_map(args):
    """Sec. 5.4: cost of the two ways to free a paused sequence's cache and get it back, per context length."""
    import numpy as np
    import torch
    import asynclm_inputs as ai
    import paper_2412_07017_amd as pkg
    wl = ai.preset(args.workload)
    model = wl.model if not args.layers else ai.truncated(wl.model, args.layers)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w_dev = ai.make_weights(model, device=dev)
    stream = torch.cuda.Stream(device=dev)
    lens = [256, 512, 1024, 2048, 4096, 8192, 16384]
    lm = pkg.AsyncLM(model, w_dev, max_positions=lens[-1] + 8, stream=stream)
    toks = ai.uniform_tokens(ai.MASTER_SEED, 103, lens[-1], model.vocab)
    rows = []
    for L in lens:
        lm.reset(0)
        lm.prefill(0, toks[:L])
        lm.synchronize()
        nbytes = lm.kv_bytes(0)
        pinned = torch.empty(nbytes, dtype=torch.uint8).pin_memory()
        best = {"context": L, "image_MB": nbytes / 1e6}
        for rep in range(4):                    # the first round touches the pinned pages; the fastest of the rest is kept
            t0 = time.perf_counter(); lm.kv_swap_out(0, pinned.data_ptr(), nbytes); t1 = time.perf_counter()
            lm.reset(0)
            t2 = time.perf_counter(); lm.kv_swap_in(0, pinned.data_ptr(), nbytes); t3 = time.perf_counter()
            lm.reset(0)
            t4 = time.perf_counter(); lm.prefill(0, toks[:L]); lm.synchronize(); t5 = time.perf_counter()
            if rep:
                for key, ms in (("swap_out_ms", (t1 - t0) * 1e3), ("swap_in_ms", (t3 - t2) * 1e3), ("recompute_ms", (t5 - t4) * 1e3)):
                    best[key] = min(best.get(key, ms), ms)
        rows.append(best)
        del pinned
    lm.close()
    print(json.dumps({"trap_map": rows, "workload": wl.name, "layers": model.n_layers}))


def e2e_calls(args):
    """Sec. 6.3 on the device: N independent calls, each a 20-token call block that the model has to generate and
    an execution of a seeded random duration (30-500 ms, a timer thread stands in for the executor).  Synchronous
    calling generates a block, waits for its result, appends it and goes on; asynchronous calling keeps generating
    while calls execute, appends every returned result as an interrupt block with the next token (never inside a
    call block), and waits (trap) only when nothing is left to generate.  Token values are scripted (forced): the
    timing does not depend on them."""
    import threading
    import numpy as np
    import torch
    import asynclm_inputs as ai
    import paper_2412_07017_amd as pkg
    from paper_2412_07017_amd.latency_model import Call, latency_sync, simulate_async
    wl = ai.preset(args.workload)
    model = wl.model if not args.layers else ai.truncated(wl.model, args.layers)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w_dev = ai.make_weights(model, device=dev)
    stream = torch.cuda.Stream(device=dev)
    n, block, result_len = args.e2e_calls, 20, 20
    rng = np.random.default_rng([ai.MASTER_SEED, 77, n])
    exe = rng.uniform(0.030, 0.500, n)
    prompt = ai.uniform_tokens(ai.MASTER_SEED, 105, wl.prompt_len, model.vocab)
    tok = lambda purpose, k: [int(t) for t in ai.uniform_tokens(ai.MASTER_SEED, 106, k, model.vocab, sub=purpose)]
    lm = pkg.AsyncLM(model, w_dev, max_positions=wl.prompt_len + n * (block + result_len + 8) + 64, stream=stream)

    def run(asynchronous, order, naive=False):
        # naive = the stateless variant of Sec. 5.5: every batch of returned results costs a re-prefill of the whole stream
        history = [int(t) for t in prompt]
        lm.reset(0)
        lm.prefill(0, prompt)
        lm.synchronize()
        lock, returned, timers = threading.Lock(), [], []

        def launch(i):
            def done():
                with lock:
                    returned.append(i)
            t = threading.Timer(float(exe[i]), done)
            timers.append(t)
            t.start()

        def take():
            with lock:
                out = list(returned)
                returned.clear()
            return out

        injected = events = 0                                   # results appended; passes that appended them
        t0 = time.perf_counter()
        for i in order:
            body = tok(i, block)
            for j, t in enumerate(body):
                last = j == block - 1
                if asynchronous and last:
                    launch(i)                                   # the block is complete with this token: the call starts
                ready = take() if (asynchronous and last) else []
                history.append(t)
                if ready and naive:
                    history.extend(sum((tok(1000 + r, result_len) for r in ready), []))
                    lm.reset(0)
                    lm.prefill(0, history)
                    injected += len(ready)
                    events += 1
                elif ready:                                     # outside the block again: results ride with the token
                    res = sum((tok(1000 + r, result_len) for r in ready), [])
                    history.extend(res)
                    lm.step_batch([0], [t], [res], want_tokens=False)
                    injected += len(ready)
                    events += 1
                else:
                    lm.decode_step(0, forced_token=t)
            if not asynchronous:
                lm.synchronize()
                launch(i)
                timers[-1].join()                               # the model waits for the result
                take()
                lm.inject_interrupt(0, tok(1000 + i, result_len))
                injected += 1
        while injected < n:                                     # trap: nothing left to generate, wait for results
            ready = take()
            if ready and naive:
                history.extend(sum((tok(1000 + r, result_len) for r in ready), []))
                lm.reset(0)
                lm.prefill(0, history)
                injected += len(ready)
                events += 1
            elif ready:
                lm.inject_interrupt(0, sum((tok(1000 + r, result_len) for r in ready), []))
                injected += len(ready)
                events += 1
            else:
                time.sleep(0.0005)
        lm.synchronize()
        wall = time.perf_counter() - t0
        for t in timers:
            t.join()
        return wall, events

    fifo = list(range(n))
    lpt = [int(i) for i in np.argsort(-exe)]
    run(True, fifo)                                             # warm-up (graphs, kernels)
    t_sync = run(False, fifo)[0]
    t_async_fifo = run(True, fifo)[0]
    t_async_lpt = run(True, lpt)[0]
    run(True, lpt, naive=True)
    t_naive_lpt, naive_events = run(True, lpt, naive=True)
    r0 = time.perf_counter()
    lm.reset(0)
    lm.prefill(0, ai.uniform_tokens(ai.MASTER_SEED, 105, wl.prompt_len + n * (block + result_len) // 2, model.vocab))
    lm.synchronize()
    reprefill_s = time.perf_counter() - r0                      # a re-prefill at the middle length of the run
    # the model's prediction from this device's step costs
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for t in tok(5000, 32):
        lm.decode_step(0, forced_token=t)
    e1.record(stream)
    lm.synchronize()
    step_s = e0.elapsed_time(e1) / 32 * 1e-3
    calls = [Call("f%d" % i, block * step_s, float(exe[i])) for i in range(n)]
    inject_s = 1.25 * step_s
    out = {"e2e_calls": n, "workload": wl.name, "layers": model.n_layers, "call_block_tokens": block, "result_tokens": result_len,
           "execution_s": [round(float(x), 4) for x in exe], "decode_step_ms": step_s * 1e3,
           "measured_s": {"sync": t_sync, "async_fifo": t_async_fifo, "async_lpt": t_async_lpt, "async_naive_lpt": t_naive_lpt},
           "model_s": {"sync": latency_sync(calls) + n * inject_s,
                       "async_fifo": simulate_async(calls, order=[c.name for c in calls], interrupt_cost=0.3 * step_s)[0],
                       "async_lpt": simulate_async(calls, policy="lpt", interrupt_cost=0.3 * step_s)[0],
                       "async_naive_lpt": simulate_async(calls, policy="lpt", interrupt_cost=reprefill_s)[0]},
           "reprefill_ms": reprefill_s * 1e3, "naive_reprefills": naive_events,   # results that return together share one
           "speedup_async_lpt_over_sync": t_sync / t_async_lpt}
    lm.close()
    print(json.dumps(out))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)
    if args.step_timeline:
        return step_timeline(args)
    if args.trap_map:
        return trap_map(args)
    if args.e2e_calls:
        return e2e_calls(args)
    if args.workload == "8b-ragged16":
        return bench_ragged(args)
    import numpy as np
    import torch
    import asynclm_inputs as ai
    import paper_2412_07017_amd as pkg

    wl = ai.preset(args.workload)
    model = wl.model if not args.layers else ai.truncated(wl.model, args.layers)
    spec = ai.build_workload(args.workload)
    block = wl.intr_every if wl.intr_every else 16
    k_intr = wl.intr_len
    n_blocks = args.warmup + args.steps
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    t0 = time.perf_counter()
    w_dev = ai.make_weights(model, device=dev)
    torch.cuda.synchronize()
    t_weights = time.perf_counter() - t0

    stream = torch.cuda.Stream(device=dev)
    max_pos = wl.prompt_len + n_blocks * (block + k_intr) + 3 * (k_intr + 1) + 64
    lm = pkg.AsyncLM(model, w_dev, max_positions=max_pos, max_seqs=2, stream=stream, kv_format=args.kv_format)
    if args.chunk:
        lm.set_option("chunk", args.chunk)
    if args.fused >= 0:
        lm.set_option("fused", args.fused)
    for kv in args.opt:
        k, v = kv.split("=")
        lm.set_option(k, int(v))
    t0 = time.perf_counter()
    lm.prefill(0, spec["prompt"])
    lm.synchronize()
    t_prefill = time.perf_counter() - t0

    intr = [ai.uniform_tokens(ai.MASTER_SEED, 102, k_intr, model.vocab, sub=j) for j in range(n_blocks)]
    ev = lambda: torch.cuda.Event(enable_timing=True)

    history = [int(t) for t in spec["prompt"]]          # the whole context, as the stateless variant would resend it

    step_marks = []                                     # one event after every decoding step of the timed blocks

    def run_block(j, rec):
        e0, e1, e2 = ev(), ev(), ev()
        e0.record(stream)
        marks = [e0]
        for _ in range(block):
            history.append(lm.decode_step(0))       # greedy on the device, token returned to the host
            marks.append(ev())
            marks[-1].record(stream)
        e1 = marks[-1]
        step_marks.append(marks)
        lm.inject_interrupt(0, intr[j])
        history.extend(int(t) for t in intr[j])
        e2.record(stream)
        rec.append((e0, e1, e2))

    rec = []
    for j in range(args.warmup):
        run_block(j, rec)
    lm.synchronize()
    torch.cuda.synchronize()
    rec = []
    step_marks.clear()
    len_start = lm.seq_len(0)
    t0 = time.perf_counter()
    for j in range(args.warmup, n_blocks):
        run_block(j, rec)
    lm.synchronize()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    len_end = lm.seq_len(0)

    # Sec. 5.5 stateless alternative: the session is discarded and the whole context (ending with the interrupt)
    # is prefilled again; same resulting context as the in-flight inject, timed on a second sequence slot.
    r0, r1 = ev(), ev()
    lm.prefill(1, history)
    lm.reset(1)
    lm.synchronize()
    r0.record(stream)
    lm.prefill(1, history)
    r1.record(stream)
    lm.synchronize()
    reprefill_ms = r0.elapsed_time(r1)
    lm.reset(1)

    # Sec. 5.4 trap handling: swap the paused sequence's K/V to pinned host memory and back (second run timed)
    nbytes = lm.kv_bytes(0)
    pinned = torch.empty(nbytes, dtype=torch.uint8).pin_memory()
    swap_out_ms = swap_in_ms = 0.0
    for _ in range(2):
        t_a = time.perf_counter()
        lm.kv_swap_out(0, pinned.data_ptr(), nbytes)
        t_b = time.perf_counter()
        lm.kv_swap_in(1, pinned.data_ptr(), nbytes)
        t_c = time.perf_counter()
        lm.reset(1)
        swap_out_ms, swap_in_ms = (t_b - t_a) * 1e3, (t_c - t_b) * 1e3

    # Sec. 5.3 merged form: the interrupt rides with the next chosen token in ONE forward pass
    # (asynclm_step_batch on one sequence); its cost beyond a plain decoding step is the price of the interrupt.
    merged_ms = []
    for j in range(3):
        m0, m1 = ev(), ev()
        m0.record(stream)
        lm.step_batch([0], None, [intr[j % len(intr)]])
        m1.record(stream)
        lm.synchronize()
        if j:
            merged_ms.append(m0.elapsed_time(m1))
    torch.cuda.synchronize()

    dec_ms = [a.elapsed_time(b) for a, b, c in rec]
    inj_ms = [b.elapsed_time(c) for a, b, c in rec]
    per_step_ms = np.array([m[i].elapsed_time(m[i + 1]) for m in step_marks for i in range(len(m) - 1)])
    ms_dec_step = float(np.mean(dec_ms)) / block
    ms_inject = float(np.mean(inj_ms))
    tokens = args.steps * block
    L_mid = (len_start + len_end) / 2.0
    bytes_step = model.weight_bytes_per_step() + L_mid * model.kv_bytes_per_position() \
        + model.kv_bytes_per_position() + 4 * model.vocab
    decode_tok_s = 1000.0 / ms_dec_step
    decode_frac = bytes_step / (ms_dec_step * 1e-3) / HBM_PEAK

    # dominant kernel: gate/up projection + SwiGLU (half of all weight bytes), timed per launch
    prof_ms, prof_n = 0.0, 0
    classes = {}
    for _ in range(5):
        p = lm.profile_step(0, 1)
        for name, d in p.items():
            c = classes.setdefault(name, {"ms": 0.0, "launches": 0})
            c["ms"] += d["ms"]; c["launches"] += d["launches"]
    eb = model.elem_bytes
    if "fused_step_kernel" in classes:
        # the whole step is one kernel: its algorithmic bytes are those of the step
        fk = classes["fused_step_kernel"]
        k_ms, k_bytes, k_name = fk["ms"] / fk["launches"], bytes_step, "k_decode_fused (whole decoding step)"
    else:
        gu = classes["gate_up_swiglu"]
        k_ms = gu["ms"] / gu["launches"]
        k_bytes = 2 * model.ffn * model.d_model * eb + 4 * model.d_model * 2 + 4 * model.ffn
        k_name = "gate_up_swiglu (k_gemv)"
    roofline = {"bound": "hbm", "kernel": k_name, "achieved": k_bytes / (k_ms * 1e-3) / 1e9,
                "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                "traffic": recorded_traffic(model) if "fused_step_kernel" not in classes else None,
                "bytes_per_launch": k_bytes, "ms_per_launch": k_ms,
                "timing": "HIP events on the library's stream around every launch of 5 real decoding steps (graphs off for those "
                          "steps); the gap between two launches is inside this figure"}
    roofline["frac"] = roofline["achieved"] / roofline["peak"]
    tr_us = trace_duration_us("k_gemv<bf16, 2, 4, 0>") if (args.workload == "8b" and not args.layers and "fused_step_kernel" not in classes) else None
    if tr_us:       # the same kernel's mean duration in the committed rocprofv3 kernel trace of this command
        roofline["trace"] = {"ms_per_launch": tr_us * 1e-3, "achieved": k_bytes / (tr_us * 1e-6) / 1e9, "frac": k_bytes / (tr_us * 1e-6) / HBM_PEAK,
                             "source": "profiles/8b_bench_kernel_stats.md (rocprofv3 --kernel-trace --stats)"}
    per_class = {k: {"ms_per_step": v["ms"] / 5, "launches_per_step": v["launches"] // 5} for k, v in classes.items()}
    lm.synchronize()
    # what a long plain stream reaches on this device: the output head reads its vocab x d matrix exactly once
    ceiling = None
    if "lm_head" in classes:
        head_bytes = model.vocab * model.d_model * eb + 4 * model.vocab
        ceiling = {"kernel": "output head (k_gemv), one pass over %.2f GB" % (head_bytes / 1e9),
                   "GBps": head_bytes / (classes["lm_head"]["ms"] / classes["lm_head"]["launches"] * 1e-3) / 1e9}

    out = {
        "metric": "decode tokens/s @ batch 1 (% HBM roofline); us per k-token interrupt inject",
        "value": tokens / wall, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 accumulate over %s weights and K/V" % model.dtype, "data": "synthetic",
        "config": {"workload": "%s: %d layers, d %d, %dq/%dkv heads x %d, ffn %d, vocab %d, %s; batch 1, prompt %d; "
                               "step = %d greedy decode steps + one %d-token interrupt inject"
                               % (wl.name, model.n_layers, model.d_model, model.n_q_heads, model.n_kv_heads,
                                  model.head_dim, model.ffn, model.vocab, model.dtype, wl.prompt_len, block, k_intr),
                   "context_len": [len_start, len_end], "seed": ai.MASTER_SEED},
        "decode_tokens_per_s": decode_tok_s, "decode_ms_per_token": ms_dec_step,
        "decode_hbm_frac": decode_frac, "decode_bytes_per_token": bytes_step,
        "decode_ms_per_token_p10_p50_p90": [float(np.percentile(per_step_ms, q)) for q in (10, 50, 90)],
        "decode_ms_per_token_max": float(per_step_ms.max()),
        "inject_us_min_median_max": [float(np.min(inj_ms)) * 1e3, float(np.median(inj_ms)) * 1e3, float(np.max(inj_ms)) * 1e3],
        "inject_us": ms_inject * 1e3, "inject_tokens": k_intr, "inject_in_decode_steps": ms_inject / ms_dec_step,
        # one pass over the same weights and cache: the inject's fraction of the HBM roofline
        "inject_hbm_frac": (bytes_step + (k_intr - 1) * model.kv_bytes_per_position()) / (ms_inject * 1e-3) / HBM_PEAK,
        "reprefill_us": reprefill_ms * 1e3, "reprefill_tokens": len(history), "reprefill_over_inject": reprefill_ms / ms_inject,
        "kv_swap_bytes": int(nbytes), "kv_swap_out_us": swap_out_ms * 1e3, "kv_swap_in_us": swap_in_ms * 1e3,
        "merged_step_us": float(np.mean(merged_ms)) * 1e3,
        "merged_inject_extra_in_decode_steps": float(np.mean(merged_ms)) / ms_dec_step - 1.0,
        "prefill_s": t_prefill, "weights_s": t_weights,
        # prompt through the matrix cores: 2 flop per layer weight and prompt token (the second activation plane and
        # the attention are not counted), over the bf16 matrix-core peak
        "prefill_mfma_frac": 2.0 * model.n_layers * model.layer_weight_elems() * wl.prompt_len / t_prefill / 2.5e15,
        "roofline": roofline, "streaming_read_ceiling": ceiling,
        # per kernel class, HIP events around every launch (the launch gaps are inside: the sum exceeds the step)
        "kernel_classes_incl_launch_gap": per_class,
    }
    if args.workload == "8b" and not args.layers:
        out["other_workloads"] = recorded_lines()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, model, w_dev, spec)
    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration_bytes"] = int(src.numel() * 4)
    lm.close()
    emit(args, out)


if __name__ == "__main__":
    main()
