"""Rollout throughput on one MI355X.

A "step" is one whole job of the workload with inputs and weights already resident in HBM:
for the rollout workloads, prefill of every prompt and then decode steps until every sample
has finished; for the teacher-forced workload, one log-prob pass over the packed batch.
Prints one JSON line: tokens/s, the roofline of the kernel that took the most time (HIP-event
timings gathered by the library on its own stream during the timed steps), and the CPU
oracle timed on a bounded slice of the same workload.

The default workload (`value`) is configs[1], the Qwen2.5-1.5B shape with 32 prompts x 8
samples: the largest configuration of which a couple of dozen warm-up and timed jobs fit a
benchmark run of a few minutes - one job of the 7B-shape rollout alone takes about a minute.
So that the larger configurations are measured in the same run all the same, the default run
then adds, under "other_configs" of the same JSON line, one job of configs[2] (7B-shape
rollout, 64 x 8 samples) and one teacher-forced pass over 24 of configs[4]'s packed sequences,
each with its tokens/s and the roofline of its dominant kernel (--no-other-configs skips them).
--workload runs any one of them as the main measurement; --layers and --prompts cut a
workload down for quick runs and the JSON line says so.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16


def run_job(eng, load, trace=None) -> int:
    """One generation job; returns the number of response tokens emitted.  `trace`, a list,
    receives (live samples, seconds) of every decode call (each call returns after its step has
    finished on the GPU)."""
    t0 = time.perf_counter()
    ids, toks, lps, fin = eng.rollout_prefill(load.prompt_tokens, load.prompt_offsets, load.n_samples,
                                              load.max_new_tokens, eos_id=-1, temperature=load.temperature,
                                              top_p=load.top_p)
    if trace is not None:
        trace.append((0, time.perf_counter() - t0))   # entry 0: the prefill call
    emitted = len(ids)
    steps, t_note = 0, time.perf_counter()
    while True:
        t0 = time.perf_counter()
        ids, toks, lps, fin = eng.rollout_decode_step()
        if not len(ids):
            return emitted
        if trace is not None:
            trace.append((len(ids), time.perf_counter() - t0))
        emitted += len(ids)
        steps += 1
        if t0 - t_note > 30.0:        # a long job says where it is twice a minute
            t_note = t0
            print(f"# decode step {steps}: {len(ids)} live samples, {emitted} tokens so far", file=sys.stderr, flush=True)


def write_step_trace(path, trace, load, kv_bytes_per_token, weight_bytes, command):
    """The long-tail regime change of one job as a short table: decode steps binned by the number
    of live samples B, with the cached positions they attend to (sum of c_i, every sample's
    own context, shared prompts counted per sample) and the mean step time."""
    plen = np.repeat(np.diff(load.prompt_offsets), load.n_samples).astype(np.int64)
    new = load.max_new_tokens.astype(np.int64)
    rows = []
    for t, (b, sec) in enumerate(trace[1:], start=1):      # decode call t emits response token t
        live = new > t
        assert int(live.sum()) == b, (t, b, int(live.sum()))
        rows.append((b, int((plen[live] + t).sum()), sec))
    edges = [1, 2, 3, 5, 9, 17, 33, 65, 129, 257, 513, 1 << 30]
    with open(path, "w") as f:
        f.write("Per-step trace of one job, binned by live samples B (host clock around each decode call)\n")
        f.write(f"command: {command}\n")
        f.write(f"prefill call: {1e3 * trace[0][1]:.1f} ms; decode steps: {len(rows)}; "
                f"weights read per step {weight_bytes / 1e9:.3f} GB (experts not counted); KV bytes per cached position {kv_bytes_per_token}\n")
        f.write("B range    steps  mean B  mean sum c_i  mean step us  tokens/s  weight GB/s  KV GB/s (per-sample positions)  share of decode time\n")
        total = sum(r[2] for r in rows)
        for lo, hi in zip(edges[:-1], edges[1:]):
            sel = [r for r in rows if lo <= r[0] < hi]
            if not sel:
                continue
            n = len(sel)
            mb, mc, ms = sum(r[0] for r in sel) / n, sum(r[1] for r in sel) / n, sum(r[2] for r in sel) / n
            f.write(f"{lo:4d}-{min(hi - 1, 99999):<5d} {n:6d} {mb:7.1f} {mc:13.0f} {1e6 * ms:13.1f} {mb / ms:9.0f} "
                    f"{weight_bytes / ms / 1e9:12.0f} {mc * kv_bytes_per_token / ms / 1e9:8.0f} "
                    f"{100 * n * ms / total:28.1f} %\n")


def run_queue_job(eng, load, step_ms=None) -> int:
    """The same kind of job fed through the library's prompt queue: every prompt is pushed up
    front, the scheduler admits them as slots and pages free up.  Returns the tokens emitted;
    step_ms (a list) receives the host-clock duration of every queue step."""
    eng.rollout_queue_push(load.prompt_tokens, load.prompt_offsets, load.n_samples, load.max_new_tokens,
                           eos_id=-1, temperature=load.temperature, top_p=load.top_p)
    emitted = 0
    while True:
        t0 = time.perf_counter()
        ids = eng.rollout_queue_step()[0]
        if step_ms is not None:
            step_ms.append(1e3 * (time.perf_counter() - t0))
        if not len(ids) and not eng.rollout_queue_busy():   # (a step that only caches prompt rows emits nothing)
            return emitted
        emitted += len(ids)


def run_turns_job(eng, load, turns, turn_tokens, obs_tokens, vocab, clock) -> int:
    """A multi-turn job: every sample answers `turns` times with `turn_tokens` tokens; between
    turns `obs_tokens` seeded tokens (an environment's observation) are appended to its context.
    clock accumulates the seconds spent in rollout_extend and the tokens appended there."""
    import torch
    rng = np.random.Generator(np.random.Philox(key=[7, 0x6f6273]))
    n_live = load.n_prompts * load.n_samples
    budget = np.full(n_live, turns * turn_tokens, np.int32)
    ids, toks, lps, fin = eng.rollout_prefill(load.prompt_tokens, load.prompt_offsets, load.n_samples, budget,
                                              eos_id=-1, temperature=load.temperature, top_p=load.top_p)
    emitted = len(ids)
    per_call = max(1, eng.max_batch_tokens // (obs_tokens + 1))
    for turn in range(turns):
        for _ in range(turn_tokens - 1):
            emitted += len(eng.rollout_decode_step()[0])
        if turn + 1 == turns:
            break
        live = eng.rollout_live_samples()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for a in range(0, len(live), per_call):
            part = live[a:a + per_call]
            obs = rng.integers(0, vocab, len(part) * obs_tokens).astype(np.int32)
            eng.rollout_extend(part, obs, np.arange(len(part) + 1, dtype=np.int32) * obs_tokens)
            emitted += len(part)
            clock[1] += len(part) * obs_tokens
        clock[0] += time.perf_counter() - t0
    assert not len(eng.rollout_live_samples())
    return emitted


def cpu_baseline(shape, weights, load) -> dict:
    """The oracle, as it stands, on a bounded slice: one 256-token prompt, 4 samples, 64 new
    tokens each (weights widened to fp64 beforehand, not timed)."""
    from threadpoolctl import threadpool_info
    from oracle import rollout as orollout
    from oracle import transformer as T
    model = T.Model(shape, weights)
    for name in weights:
        model.w(name)
    prompt = load.prompt_tokens[:256]
    t0 = time.perf_counter()
    emitted = orollout.decode_slice_batched(model, prompt, 4, 64, load.temperature, load.top_p, load.sampler_seed)
    dt = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    return {"value": emitted / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{shape.name}: 1 prompt x 256 tokens prefill, 4 samples x 64 new tokens, fp64, {dt:.1f} s"}


def cpu_baseline_logprobs(shape, weights, tokens) -> dict:
    """The oracle's teacher-forced pass on one 192-token sequence of the same batch."""
    from threadpoolctl import threadpool_info
    from oracle import transformer as T
    model = T.Model(shape, weights)
    for name in weights:
        model.w(name)
    toks = tokens[:192]
    t0 = time.perf_counter()
    T.packed_log_probs(model, toks, np.array([0, len(toks)]))
    dt = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    return {"value": len(toks) / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{shape.name}: one 192-token sequence, fp64, {dt:.1f} s"}


def kernel_table(eng, before):
    """Per-kernel deltas of the library's event timings since `before`; the cost of an empty
    event bracket (recorded by the library in every timed decode step) is taken off each launch."""
    kernels = []
    for k in eng.rollout_kernel_stats():
        b = before.get(k["name"], dict(launches=0, ms=0.0, bytes=0.0, flops=0.0))
        n = k["launches"] - b["launches"]
        if n:
            kernels.append(dict(name=k["name"], launches=n, ms=k["ms"] - b["ms"], bytes=k["bytes"] - b["bytes"],
                                flops=k["flops"] - b["flops"]))
    empty = [k for k in kernels if k["name"] == "(empty bracket)"]
    kernels = [k for k in kernels if k["name"] != "(empty bracket)"]
    bracket_ms = empty[0]["ms"] / empty[0]["launches"] if empty else 0.0
    for k in kernels:
        k["raw_ms"] = k["ms"]
        k["ms"] = max(k["ms"] - k["launches"] * bracket_ms, 1e-9)
    kernels.sort(key=lambda k: -k["ms"])
    return kernels, bracket_ms


def measured_traffic(kernel: str, summary: str):
    """HBM bytes per launch of `kernel` from the committed counter summary (rocprofv3 --pmc
    FETCH_SIZE / WRITE_SIZE, in KiB, each scaled by the factor a plain copy kernel of known size
    gave in the same run), or None when there is no summary for this workload or the kernel
    sources have changed since the counters were taken."""
    from paper_2506_06122_amd import build
    path = os.path.join(ROOT, "profiles", summary)
    if not os.path.exists(path):
        return None
    digest, factor, mean = None, {}, {}
    want = kernel.replace(" ", "")
    with open(path) as f:
        for line in f:
            if line.startswith("kernel-sources-sha256:"):
                digest = line.split(":", 1)[1].strip()
            elif line.startswith("factor "):
                _, counter, value = line.split()
                factor[counter] = float(value)
            elif "\tlaunches=" in line:
                name, counter, _, m = line.rstrip("\n").split("\t")[:4]
                if name.replace("void ", "").replace(" ", "") == want:
                    mean[counter] = float(m.split("=")[1])
    if digest != build.sources_digest() or set(mean) != {"FETCH_SIZE", "WRITE_SIZE"} or set(factor) != set(mean):
        return None
    return 1024.0 * sum(factor[c] * mean[c] for c in mean)


def profiled_launch_us(kernel: str, summary: str):
    """Average duration of `kernel` in the committed rocprofv3 kernel-trace summary, or None when
    there is none or the kernel sources have changed since."""
    from paper_2506_06122_amd import build
    path = os.path.join(ROOT, "profiles", summary)
    if not os.path.exists(path):
        return None
    digest, want, found = None, kernel.replace(" ", ""), None
    with open(path) as f:
        for line in f:
            if line.startswith("kernel-sources-sha256:"):
                digest = line.split(":", 1)[1].strip()
            parts = line.split(None, 4)
            if len(parts) == 5 and parts[0].isdigit() and parts[4].strip().replace("void ", "").replace(" ", "") == want:
                found = float(parts[2])
    return found if digest == build.sources_digest() else None


def roofline_of(kernels, bracket_ms, traffic_summary=None, copy_ceiling_gbs=None, kv_bytes_per_attn_flop=None):
    """Roofline object of the kernel with the most time.  Beside the contract's keys: the
    fraction of a measured plain-copy rate, and for the decode attention the rate counted
    without prefix reuse (every sample's own context, as the kernel reads it)."""
    if not kernels:
        return None
    top = kernels[0]
    ridge = MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    if top["flops"] / max(top["bytes"], 1.0) >= ridge:
        ach = top["flops"] / (top["ms"] * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None}
    else:
        ach = top["bytes"] / (top["ms"] * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": ach / HBM_PEAK_GBS, "traffic": None}
    roofline["kernel"] = top["name"]
    if roofline["bound"] == "hbm" and copy_ceiling_gbs:
        roofline["copy_ceiling"] = copy_ceiling_gbs
        roofline["frac_of_copy_ceiling"] = roofline["achieved"] / copy_ceiling_gbs
    if top["name"].startswith("attn_decode") and kv_bytes_per_attn_flop:
        roofline["achieved_without_prefix_reuse"] = top["flops"] * kv_bytes_per_attn_flop / (top["ms"] * 1e-3) / 1e9
    roofline["algorithmic_bytes_per_launch"] = top["bytes"] / top["launches"]
    if traffic_summary:
        roofline["traffic"] = measured_traffic(top["name"], traffic_summary)
        if roofline["traffic"] is not None:  # not measured in this run: read from the committed counter summary
            roofline["traffic_source"] = "profiles/" + traffic_summary
    roofline["avg_launch_us"] = 1e3 * top["ms"] / top["launches"]
    if traffic_summary:
        # the profiler's own average for the same kernel over a whole run (its timestamps, about
        # 2 us per launch above the event times with the empty bracket taken off), when the
        # committed kernel trace of this workload was taken on these kernel sources
        us = profiled_launch_us(top["name"], traffic_summary.replace("hbm_traffic", "kernel_trace"))
        if us:
            roofline["rocprofv3_avg_launch_us"] = us
            roofline["frac_at_rocprofv3_time"] = top["bytes"] / top["launches"] / (us * 1e-6) / 1e9 / HBM_PEAK_GBS \
                if roofline["bound"] == "hbm" else top["flops"] / top["launches"] / (us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS
    roofline["timed_launches"] = top["launches"]
    roofline["event_bracket_us"] = 1e3 * bracket_ms
    roofline["per_kernel"] = [
        {"name": k["name"], "launches": k["launches"], "avg_us": 1e3 * k["ms"] / k["launches"],
         "GB/s": k["bytes"] / (k["ms"] * 1e-3) / 1e9, "TFLOP/s": k["flops"] / (k["ms"] * 1e-3) / 1e12}
        for k in kernels]
    return roofline


def measure_other_configs(args, flags, copy_ceiling_gbs) -> dict:
    """One job of the 7B-shape rollout (configs[2]) and one teacher-forced pass over 24 of
    configs[4]'s sequences on the same weights: tokens/s and the dominant kernel's roofline."""
    import torch
    import paper_2506_06122_amd as R
    import workloads
    shape = workloads.C3_7B
    out = {}
    t0 = time.perf_counter()
    weights = workloads.make_weights(shape, seed=1, gains="ones")
    print(f"# other configs: 7B-shape weights generated in {time.perf_counter() - t0:.1f} s", file=sys.stderr, flush=True)
    kv_bytes_per_token = shape.n_layers * shape.n_kv_heads * shape.head_dim * 2 * 2
    kv_per_flop = shape.n_kv_heads * shape.head_dim * 4 / (4.0 * shape.n_q_heads * shape.head_dim)

    def brief(roof):
        keep = ("bound", "achieved", "peak", "unit", "frac", "traffic", "traffic_source", "kernel", "avg_launch_us",
                "rocprofv3_avg_launch_us", "frac_at_rocprofv3_time", "timed_launches", "algorithmic_bytes_per_launch", "achieved_without_prefix_reuse", "frac_of_copy_ceiling")
        r = {k: roof[k] for k in keep if k in roof}
        r["top_kernels"] = roof["per_kernel"][:6]
        return r

    # ---- configs[2]: one rollout job
    load = workloads.load_c3()
    max_prompt = int(np.diff(load.prompt_offsets).max())
    need = int(np.diff(load.prompt_offsets).sum()) + int(load.max_new_tokens.sum()) + 64 * load.n_prompts * load.n_samples
    eng = R.Rollout(shape, weights, kv_pool_bytes=need * kv_bytes_per_token, page_tokens=32,
                    max_live_samples=load.n_prompts * load.n_samples,
                    max_context=max_prompt + int(load.max_new_tokens.max()), max_batch_tokens=16384,
                    seed=load.sampler_seed, flags=flags, timing_stride=max(args.timing_stride, 1))
    ids = eng.rollout_prefill(load.prompt_tokens[:64], np.array([0, 64], np.int32), 4, np.full(4, 8, np.int32))[0]
    for _ in range(4):                                    # a short warm-up: first launches, first page faults
        eng.rollout_decode_step()
    eng.rollout_abort(ids)
    torch.cuda.synchronize()
    before = {k["name"]: k for k in eng.rollout_kernel_stats()}
    calls0 = int(eng.rollout_get_stats()["decode_steps"])
    t0 = time.perf_counter()
    emitted = run_job(eng, load)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kernels, bracket_ms = kernel_table(eng, before)
    out["configs[2]"] = {
        "workload": "Qwen2.5-7B-shaped dense decoder, bf16, %d prompts x %d samples, prompt 128-1024, response "
                    "log-normal(median 1024, sigma 1) capped 8192, T=0.99 top-p=1.0; one job, no warm-up job"
                    % (load.n_prompts, load.n_samples),
        "value": emitted / dt, "unit": "tokens/s", "ms_per_step": 1e3 * dt, "output_tokens": emitted,
        "decode_calls": int(eng.rollout_get_stats()["decode_steps"]) - calls0,
        "roofline": brief(roofline_of(kernels, bracket_ms, None, copy_ceiling_gbs, kv_per_flop))}
    eng.close()
    del eng
    torch.cuda.empty_cache()
    print(f"# other configs: configs[2] job done in {dt:.1f} s", file=sys.stderr, flush=True)

    # ---- configs[4]: teacher-forced pass, every call timed
    tokens, cu = workloads.packed_sequences(24, 512, 8192, shape.vocab, seed=2)
    chunk = 16384
    eng = R.Rollout(shape, weights, kv_pool_bytes=(chunk + 8192 + 64 * 32) * kv_bytes_per_token, page_tokens=32,
                    max_live_samples=8, max_context=8192, max_batch_tokens=chunk, seed=3, flags=flags, timing_stride=1)
    eng.rollout_logprobs(tokens[:cu[1]], cu[:2], temperature=1.0)      # warm-up: the first sequence
    torch.cuda.synchronize()
    before = {k["name"]: k for k in eng.rollout_kernel_stats()}
    t0 = time.perf_counter()
    eng.rollout_logprobs(tokens, cu, temperature=1.0)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kernels, bracket_ms = kernel_table(eng, before)
    out["configs[4]"] = {
        "workload": "teacher-forced log-prob pass, Qwen2.5-7B-shaped dense decoder, bf16, 24 packed sequences (of the "
                    "config's 512), length U{512..8192}, %d tokens; one pass after a one-sequence warm-up" % len(tokens),
        "value": len(tokens) / dt, "unit": "tokens/s", "ms_per_step": 1e3 * dt, "tokens": int(len(tokens)),
        # the counters of profiles/logprobs_c5_hbm_traffic.txt were taken on this same pass
        "roofline": brief(roofline_of(kernels, bracket_ms, "logprobs_c5_hbm_traffic.txt", copy_ceiling_gbs, kv_per_flop))}
    eng.close()
    del eng, weights
    torch.cuda.empty_cache()
    return out


def attention_launch_probe(args) -> int:
    """Decode steps of config 2's shape (4 layers unless --layers says otherwise) with --prompts
    rows that all hold --context cached positions: what one launch of the decode attention costs
    as a function of rows and bytes, without a job's mix of both.  Every launch is bracketed by
    HIP events (the empty bracket is reported beside it); under rocprofv3 --kernel-trace --stats
    the kernel's own average is the one to read."""
    import torch
    import paper_2506_06122_amd as R
    import workloads
    from paper_2506_06122_amd import binding as B
    shape = dataclasses.replace(workloads.C2_1P5B, n_layers=args.layers or 4)
    weights = workloads.make_weights(shape, seed=1, gains="ones")
    rows, ctx, steps = args.prompts or 187, args.context, max(args.steps, 12)
    rng = np.random.default_rng(1)
    toks = rng.integers(0, shape.vocab, rows * ctx).astype(np.int32)
    offs = (np.arange(rows + 1) * ctx).astype(np.int32)
    kv_per_token = 2 * shape.n_layers * shape.n_kv_heads * shape.head_dim * 2
    eng = R.Rollout(shape, weights, kv_pool_bytes=rows * (ctx + 128) * kv_per_token + (64 << 20), page_tokens=32,
                    max_live_samples=rows, max_context=ctx + 64, max_batch_tokens=16384, seed=1,
                    flags=B.RT_KERNEL_TIMING, timing_stride=1)
    per_call = max(1, min(64, 16384 // ctx))
    for i in range(0, rows, per_call):
        j = min(rows, i + per_call)
        eng.rollout_prefill(toks[offs[i]:offs[j]], offs[i:j + 1] - offs[i], 1, np.full(j - i, steps + 2, np.int32))
    before = {k["name"]: k for k in eng.rollout_kernel_stats()}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        eng.rollout_decode_step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    kernels, bracket_ms = kernel_table(eng, before)
    eng.close()
    kernels = [dict(name=k["name"], launches=k["launches"], avg_us=1e3 * k["ms"] / k["launches"],
                    **{"MB": k["bytes"] / k["launches"] / 1e6, "GB/s": k["bytes"] / (k["ms"] * 1e-3) / 1e9}) for k in kernels]
    attn = [k for k in kernels if k["name"].startswith("attn_decode")]
    out = {"metric": "decode attention launch on 1 MI355X", "value": attn[0]["avg_us"] if attn else None, "unit": "us",
           "n_gpus": 1, "steps": steps, "warmup": 0, "ms_per_step": 1e3 * dt, "higher_is_better": False,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "configs[1]'s shape with %d layers, %d rows x %d cached positions each, %d decode steps, "
                                  "every launch bracketed by HIP events" % (shape.n_layers, rows, ctx, steps)},
           "roofline": {"bound": "hbm", "achieved": attn[0]["GB/s"] if attn else None, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": attn[0]["GB/s"] / HBM_PEAK_GBS if attn else None, "traffic": None,
                        "kernel": attn[0]["name"] if attn else None, "event_bracket_us": 1e3 * bracket_ms,
                        "per_kernel": kernels[:8]},
           "cpu_baseline": None}
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--timing-stride", type=int, default=61,
                    help="bracket kernels with HIP events on every n-th library call (0 = never); a prime, so that "
                         "calls that recur with a job's period (its prefill) are sampled like any other")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="default workload only: skip the one-job measurements of configs[2] and configs[4]")
    ap.add_argument("--workload", choices=["c2", "c3", "c4", "c5", "c2-queue", "c2-turns", "c2-refresh", "loss", "c2-attn"],
                    default="c2",
                    help="c2 = headline (1.5B shape); c3 = 7B-shape rollout; c4 = 30B-A3B-shape MoE rollout; "
                         "c5 = teacher-forced log-prob pass on the 7B shape; c2-queue = config 2's model and "
                         "length laws with 4x the prompts fed through the prompt queue into the same 256 live slots; "
                         "c2-turns = config 2's model and prompts, 4 turns of 128 response tokens with 256 appended "
                         "tokens between turns (rollout_extend); c2-refresh = all of config 2's weights replaced in "
                         "place from device buffers, one bucket per layer (rollout_update_weights); loss = the "
                         "policy-gradient objective over config 5's 512 packed sequences (rollout_policy_loss)")
    ap.add_argument("--prompts", type=int, default=0, help="prompts (c5: sequences); 0 = the workload's own count")
    ap.add_argument("--layers", type=int, default=0, help="cut the model to this many layers (0 = all)")
    ap.add_argument("--context", type=int, default=400,
                    help="c2-attn: cached positions of every row (--prompts = the number of rows, default 187)")
    ap.add_argument("--chunk-rows", type=int, default=0,
                    help="c2-queue: chunked prefill, at most this many prompt rows ride along with each decode step "
                         "(0 = whole prompts before the step)")
    ap.add_argument("--prompt-groups", action="store_true",
                    help="decode attention reads shared prompt pages once per group of samples (library flag)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="accepted for the byte-counter commands that name it: the plain 256 MiB read+write kernels "
                         "(a known-size reference for byte counters, and the measured copy ceiling) now always run")
    ap.add_argument("--step-trace", default="",
                    help="c2/c3/c4: write a table of the last timed job's decode steps, binned by live samples, here")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import torch
    import paper_2506_06122_amd as R
    from paper_2506_06122_amd import binding as B
    import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    # A plain elementwise kernel that reads 256 MiB and writes 256 MiB: its rate is the measured
    # ceiling beside the nominal HBM peak, and under a byte-counter run (--copy-calibration) its
    # launches are the known-size reference.
    src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        torch.mul(src, 2.0, out=dst)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        torch.mul(src, 2.0, out=dst)
    e1.record()
    torch.cuda.synchronize()
    copy_ceiling_gbs = 5 * 2 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst

    wl = args.workload
    if wl == "loss":
        _, cu = workloads.packed_sequences(args.prompts or 512, 512, 8192, 1024, seed=2)
        total = int(cu[-1])
        g = torch.Generator(device="cuda").manual_seed(3)
        old = -torch.rand(total, device="cuda", generator=g) * 4
        new = old + 0.3 * torch.randn(total, device="cuda", generator=g)
        ref = old + 0.2 * torch.randn(total, device="cuda", generator=g)
        mask = (torch.rand(total, device="cuda", generator=g) > 0.3).to(torch.uint8)
        rewards = np.random.default_rng(4).standard_normal(len(cu) - 1).astype(np.float32) * 15
        run = lambda: R.rollout_policy_loss(cu, new, old, ref, mask, rewards, gamma=0.99, kl_coef=0.02)
        for _ in range(args.warmup):
            run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            run()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / max(args.steps, 1)
        nbytes = total * (3 * 4 + 1 + 2 * 4 + 2 * 4)  # three log-probs and the mask in; advantages out; gradient out, scaled in place
        print(json.dumps({"metric": "policy-loss tokens/sec on 1 MI355X", "value": total / dt, "unit": "tokens/s",
                          "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * dt,
                          "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
                          "data": "synthetic",
                          "config": {"workload": "%d packed sequences, length U{512..8192}, %d tokens; the call "
                                     "includes its own allocations, two small uploads and the loss coming back"
                                     % (len(cu) - 1, total)},
                          "roofline": {"bound": "hbm", "achieved": nbytes / dt / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                       "frac": nbytes / dt / 1e9 / HBM_PEAK_GBS, "traffic": None,
                                       "kernel": "policy_advantage_kernel + policy_scale_kernel (whole call)"},
                          "cpu_baseline": None}))
        return 0
    if wl == "c2-attn":
        return attention_launch_probe(args)
    shape = {"c2": workloads.C2_1P5B, "c3": workloads.C3_7B, "c4": workloads.C4_30B_A3B, "c5": workloads.C3_7B,
             "c2-queue": workloads.C2_1P5B, "c2-turns": workloads.C2_1P5B, "c2-refresh": workloads.C2_1P5B}[wl]
    cut = ""
    if args.layers and args.layers < shape.n_layers:
        cut = f", cut to {args.layers} of {shape.n_layers} layers"
        shape = dataclasses.replace(shape, n_layers=args.layers)
    t0 = time.perf_counter()
    weights = workloads.make_weights(shape, seed=1, gains="ones")
    print(f"# weights generated in {time.perf_counter() - t0:.1f} s", file=sys.stderr, flush=True)
    flags = (B.RT_KERNEL_TIMING if args.timing_stride > 0 else 0) | (B.RT_PROMPT_GROUPS if args.prompt_groups else 0)
    kv_bytes_per_token = shape.n_layers * shape.n_kv_heads * shape.head_dim * 2 * 2

    if wl == "c2-refresh":
        from paper_2506_06122_amd.binding import _to_device
        eng = R.Rollout(shape, weights, kv_pool_bytes=1 << 30, page_tokens=32, max_live_samples=8, max_context=512,
                        max_batch_tokens=512, seed=1)
        dev = {k: _to_device(v, True) for k, v in weights.items()}
        buckets = [{k: dev[k] for k in ("embed", "final_norm", "lm_head")}] + \
            [{k: v for k, v in dev.items() if k.startswith(f"layers.{i}.")} for i in range(shape.n_layers)]
        nbytes = sum(v.numel() * v.element_size() for v in dev.values())

        def refresh():
            for b in buckets:
                eng.rollout_update_weights(b)
        for _ in range(args.warmup):
            refresh()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            refresh()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / max(args.steps, 1)
        print(json.dumps({"metric": "weight refresh GB/s on 1 MI355X (bytes of the new weights per second)",
                          "value": nbytes / dt / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
                          "warmup": args.warmup, "ms_per_step": 1e3 * dt, "higher_is_better": True,
                          "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                          "config": {"workload": "all tensors of configs[1]'s model (%.2f GB) re-ordered into the "
                                     "library's layout from device buffers, %d buckets" % (nbytes / 1e9, len(buckets))},
                          "roofline": {"bound": "hbm", "achieved": 2 * nbytes / dt / 1e9, "peak": HBM_PEAK_GBS,
                                       "unit": "GB/s", "frac": 2 * nbytes / dt / 1e9 / HBM_PEAK_GBS, "traffic": None,
                                       "kernel": "pack_weight_kernel"},
                          "cpu_baseline": None}))
        eng.close()
        return 0
    if wl == "c5":
        n_seqs = args.prompts or 24
        tokens, cu = workloads.packed_sequences(n_seqs, 512, 8192, shape.vocab, seed=2)
        chunk = 16384
        eng = R.Rollout(shape, weights, kv_pool_bytes=(chunk + 8192 + 64 * 32) * kv_bytes_per_token, page_tokens=32,
                        max_live_samples=8, max_context=8192, max_batch_tokens=chunk, seed=3, flags=flags,
                        timing_stride=1)
        work = lambda: (eng.rollout_logprobs(tokens, cu, temperature=1.0), len(tokens))[1]
        desc = ("configs[4]: teacher-forced log-prob pass, Qwen2.5-7B-shaped dense decoder, bf16, %d packed sequences "
                "(of the config's 512), length U{512..8192}, %d tokens%s" % (n_seqs, len(tokens), cut))
        load = None
    elif wl == "c2-turns":
        turns, turn_tokens, obs_tokens = 4, 128, 256
        load = workloads.load_c2(n_prompts=args.prompts or 32)
        max_prompt = int(np.diff(load.prompt_offsets).max())
        max_ctx = max_prompt + turns * turn_tokens + (turns - 1) * obs_tokens
        live = load.n_prompts * load.n_samples
        eng = R.Rollout(shape, weights, kv_pool_bytes=live * (max_ctx + 64) * kv_bytes_per_token, page_tokens=32,
                        max_live_samples=live, max_context=max_ctx, max_batch_tokens=16384,
                        seed=load.sampler_seed, flags=flags, timing_stride=max(args.timing_stride, 1))
        eng.max_batch_tokens = 16384
        extend_clock = [0.0, 0]
        work = lambda: run_turns_job(eng, load, turns, turn_tokens, obs_tokens, shape.vocab, extend_clock)
        desc = ("configs[1]'s model and prompts, %d prompts x %d samples, %d turns of %d response tokens, %d tokens "
                "appended to every context between turns" % (load.n_prompts, load.n_samples, turns, turn_tokens,
                                                             obs_tokens)) + cut
    elif wl == "c2-queue":
        live = 256
        load = workloads.load_c2(n_prompts=args.prompts or 128)
        max_prompt = int(np.diff(load.prompt_offsets).max())
        max_ctx = max_prompt + int(load.max_new_tokens.max())
        # worst case: every live sample at the longest context (pages are taken at admission)
        eng = R.Rollout(shape, weights, kv_pool_bytes=live * (max_ctx + 64) * kv_bytes_per_token, page_tokens=32,
                        max_live_samples=live, max_context=max_ctx, max_batch_tokens=max(16384, max_prompt),
                        seed=load.sampler_seed, flags=flags, timing_stride=max(args.timing_stride, 1))
        if args.chunk_rows:
            eng.rollout_queue_chunking(args.chunk_rows)
        queue_step_ms = []
        work = lambda: run_queue_job(eng, load, queue_step_ms)
        desc = ("configs[1]'s model and length laws, %d prompts x %d samples pushed to the prompt queue, admitted "
                "into %d live slots as samples finish%s" % (
                    load.n_prompts, load.n_samples, live,
                    ", at most %d prompt rows per step (chunked prefill)" % args.chunk_rows if args.chunk_rows else "")) + cut
    else:
        loader = {"c2": workloads.load_c2, "c3": workloads.load_c3, "c4": workloads.load_c4}[wl]
        load = loader(n_prompts=args.prompts) if args.prompts else loader()
        max_prompt = int(np.diff(load.prompt_offsets).max())
        # every sample's pages are taken at admission: prompt pages once per prompt, the rest per sample
        need = int(np.diff(load.prompt_offsets).sum()) + int(load.max_new_tokens.sum()) + \
            64 * load.n_prompts * load.n_samples
        eng = R.Rollout(shape, weights, kv_pool_bytes=max(need * kv_bytes_per_token, 1 << 30), page_tokens=32,
                        max_live_samples=load.n_prompts * load.n_samples,
                        max_context=max_prompt + int(load.max_new_tokens.max()),
                        max_batch_tokens=max(16384, max_prompt), seed=load.sampler_seed, flags=flags,
                        timing_stride=max(args.timing_stride, 1))
        trace = [] if args.step_trace else None

        def work():
            if trace is not None:
                del trace[:]
            return run_job(eng, load, trace)
        names = {"c2": "configs[1]: Qwen2.5-1.5B-shaped dense decoder, bf16, %d prompts x %d samples, prompt 64-512, "
                       "response geometric(mean 512) capped 2048, T=1.0 top-p=1.0",
                 "c3": "configs[2]: Qwen2.5-7B-shaped dense decoder, bf16, %d prompts x %d samples, prompt 128-1024, "
                       "response log-normal(median 1024, sigma 1) capped 8192, T=0.99 top-p=1.0",
                 "c4": "configs[3]: Qwen3-30B-A3B-shaped mixture of experts (128 experts, top-8), bf16, %d prompts x %d "
                       "samples, prompt 128-1024, response log-normal(median 2048, sigma 1) capped 16384, T=1.0 top-p=1.0"}
        desc = names[wl] % (load.n_prompts, load.n_samples) + cut
    assert eng.rollout_get_stats()["matrix_core_path"] == 1
    print("# engine ready", file=sys.stderr, flush=True)

    if load is not None and args.timing_stride > 1:
        # The library times the calls whose index is a multiple of the stride, call 0 among them:
        # a one-token prompt admitted and aborted takes that index, so that a run without warm-up
        # jobs does not start its sample on the job's prefill.
        ids = eng.rollout_prefill(np.zeros(1, np.int32), np.array([0, 1], np.int32), 1, np.array([2], np.int32))[0]
        eng.rollout_abort(ids)
    for _ in range(args.warmup):
        work()
    if wl == "c2-queue":
        del queue_step_ms[:]
    torch.cuda.synchronize()
    before = {k["name"]: k for k in eng.rollout_kernel_stats()}
    calls0 = int(eng.rollout_get_stats()["decode_steps"])
    t0 = time.perf_counter()
    emitted = 0
    for _ in range(args.steps):
        emitted += work()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    stats = eng.rollout_get_stats()
    kernels, bracket_ms = kernel_table(eng, before)

    # counters exist for the full workloads only, taken over one whole job
    summary = None if (args.prompts or cut) else {"c2": "rollout_c2_hbm_traffic.txt",
                                                  "c5": "logprobs_c5_hbm_traffic.txt"}.get(wl)
    out = {
        "metric": "rollout output tokens/sec on 1 MI355X" if wl != "c5" else "teacher-forced tokens/sec on 1 MI355X",
        "value": emitted / dt, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * dt / max(args.steps, 1),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": desc,
                   "output_tokens_per_step": emitted // max(args.steps, 1),
                   "decode_calls_per_step": (int(stats["decode_steps"]) - calls0) // max(args.steps, 1)},
        # decode attention: 4 flops per cached position, query column and head dimension; K and V
        # of that position are n_kv_heads * head_dim * 2 * 2 bytes
        "roofline": roofline_of(kernels, bracket_ms, summary, copy_ceiling_gbs,
                                shape.n_kv_heads * shape.head_dim * 4 / (4.0 * shape.n_q_heads * shape.head_dim)),
    }
    if args.step_trace and wl in ("c2", "c3", "c4"):
        non_expert = shape.param_count() - shape.vocab * shape.hidden - \
            shape.n_layers * shape.n_experts * 3 * shape.expert_ffn_dim * shape.hidden
        write_step_trace(args.step_trace, trace, load, kv_bytes_per_token, 2 * non_expert,
                         "python bench.py " + " ".join(sys.argv[1:]))
    if wl == "c2-queue" and queue_step_ms:  # how long the live samples wait between two of their tokens
        q = np.sort(np.array(queue_step_ms))
        out["config"]["queue_steps"] = {"steps": len(q), "mean_ms": float(q.mean()), "p99_ms": float(q[int(0.99 * (len(q) - 1))]),
                                        "max_ms": float(q[-1]), "chunk_rows": args.chunk_rows}
    if wl == "c2-turns" and extend_clock[0] > 0:  # warm-up jobs included: a rate, not a total
        out["config"]["appended_tokens_per_s"] = extend_clock[1] / extend_clock[0]
    eng.close()
    del eng
    torch.cuda.empty_cache()
    if wl == "c2" and not (args.prompts or cut or args.no_other_configs):
        out["other_configs"] = measure_other_configs(args, flags, copy_ceiling_gbs)
    if args.no_cpu_baseline:
        out["cpu_baseline"] = None
    elif wl == "c5":
        out["cpu_baseline"] = cpu_baseline_logprobs(shape, weights, tokens)
    else:
        out["cpu_baseline"] = cpu_baseline(shape, weights, load)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
