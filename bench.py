"""Benchmark of the partition decode hot path on one MI355X.

One step = one later visit of one sample (Sec. III-D) to a partition (all its
layers: norm, fused QKV + RoPE + KV append, paged attention, output projection,
MLP).  The N samples in flight are visited round-robin, so consecutive steps
read different KV caches (the rotating-cache access pattern).  By default the
messages of all N samples are handed over per call (the node's input queue,
Sec. III-A, drained in one call) and, where the partition supports it, share
ONE pass over the weights (mdi_decode_batch); the roofline then counts the
matrices once per launch.  `--passes per-message` keeps one pass per message
(mdi_decode_steps), `--queue 1` hands the messages over one at a time
(mdi_decode_step, the paper's own rule); the default run reports both of those
rates too.  Inputs, weights and caches are resident in HBM before the timed
region; prompts are prefilled (first visit) before it and timed separately.

Any --steps / --warmup is accepted: exactly --steps steps are timed (the last
call of a window carries fewer messages when the count does not divide), and a
workload whose caches cannot hold them in one go (C1, C2) times them in several
windows, each after fresh first visits, with only the decode calls inside the
timed regions.  Workloads with several partitions (C2, C5) put all of them on
the one GPU and report every partition alone and all of them driven round-robin.

Prints ONE JSON line (see the keys below).
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, vendor figure
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
FP32_VECTOR_PEAK_TFLOPS = 157.3

# HBM bytes per launch of the decode kernel from rocprofv3 FETCH_SIZE + WRITE_SIZE runs of this script, keyed by
# (workload, messages per launch, batched arithmetic).  A figure is only reported while the kernel sources still
# hash to what they were when it was measured; otherwise `roofline.traffic` is null.
KERNEL_SOURCES = ("step_impl.h", "step_batch.h", "head_batch.h", "step_w4.hip", "step_w8.hip", "device_utils.h", "mdi_internal.h")
MEASURED_TRAFFIC = {
    (4, 8, True): {"bytes": 4.9261e9, "kernel_rev": "5a05780777ce",
                   "source": "profiles/k_step_batch_c4_decode_hbm_counters.md (FETCH_SIZE x 2.0 KiB + WRITE_SIZE x 1.0 KiB, context about 1030)"},
}


def kernel_rev():
    h = hashlib.sha1()
    for name in KERNEL_SOURCES:
        path = os.path.join(ROOT, "paper_2505_18164_amd", "csrc", name)
        if os.path.exists(path):
            h.update(open(path, "rb").read())
    return h.hexdigest()[:12]


def measured_traffic(workload, in_launch, batched):
    rec = MEASURED_TRAFFIC.get((workload, in_launch, bool(batched)))
    if rec and rec["kernel_rev"] == kernel_rev():
        return rec["bytes"], rec["source"]
    return None, None


def parse(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--paper-run", choices=["nanollama", "tinyllama"], default=None,
                    help="instead of the partition benchmark: the paper's generation experiment on this model shape "
                         "(3 samples x 800 tokens from one-token prompts, its cuts and an unbalanced one)")
    ap.add_argument("--paper-tokens", type=int, default=800, help="tokens per sample of --paper-run")
    ap.add_argument("--steps", type=int, default=1600)
    ap.add_argument("--warmup", type=int, default=80)
    ap.add_argument("--workload", type=int, default=4, help="index into the five benchmark configs (1-5)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-output-layers", action="store_true", help="skip timing the output layers of the same model")
    ap.add_argument("--no-side-runs", action="store_true", help="only the main timed region (no one-at-a-time run, no other partitions)")
    ap.add_argument("--ctx-sweep", action="store_true", help="also time decode at the middle and end context")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MiB (reference for HBM byte counters)")
    ap.add_argument("--decode-path", type=int, default=0, help="0 = automatic (persistent single-launch step), 1 = one kernel per operation")
    ap.add_argument("--passes", choices=["auto", "shared", "per-message"], default="auto",
                    help="how the messages of one call take the weights: 'shared' = one pass over the weights for all "
                         "of them (mdi_decode_batch), 'per-message' = a pass each (mdi_decode_steps, the paper's rule "
                         "inside one launch), 'auto' = shared where the partition supports it")
    ap.add_argument("--queue", type=int, default=0,
                    help="messages of different samples handed to the partition per call: 0 = all samples in flight "
                         "(mdi_decode_steps drains the queue), 1 = one at a time (mdi_decode_step)")
    return ap.parse_args(argv)


def plan_windows(n_seqs, prompt, max_ctx, steps, warmup, queue):
    """How `steps` timed decode steps (after `warmup` untimed ones) fit a workload whose caches hold max_ctx
    positions: a list of windows (warmup_steps, timed_steps); every window starts from fresh first visits of
    `prompt` tokens.  Never refuses: the queue is clamped to [1, n_seqs], a warm-up that alone would fill the
    caches is cut (the count actually run is in the result), and the timed steps are spread over as many windows
    as the context needs.  Returns (queue, windows)."""
    queue = n_seqs if queue <= 0 else max(1, min(queue, n_seqs))
    steps = max(1, int(steps))
    warmup = max(0, int(warmup))
    cap = n_seqs * (max_ctx - prompt)               # decode steps the caches hold after the first visits
    if cap < 2:
        raise ValueError("workload leaves no room for decode steps")
    warm0 = min(warmup, cap // 4)
    rewarm = min(warm0, n_seqs)                     # later windows only re-warm after their first visits
    windows, left = [], steps
    while left > 0:
        w = warm0 if not windows else rewarm
        t = min(left, cap - w)
        windows.append((w, t))
        left -= t
    return queue, windows


def calls_of(first, count, queue, n_seqs):
    """Round-robin message ids of `count` steps starting at step index `first`, cut into calls of <= queue."""
    out, k = [], first
    end = first + count
    while k < end:
        m = min(queue, end - k)
        out.append([(k + i) % n_seqs for i in range(m)])
        k += m
    return out


def cpu_baseline(cfg, w, lo, hi, seed, S, prompt, embed):
    """The oracle as it stands, timed on this host: one sample's first visit of the workload's prompt length, then
    decode steps at that context for about 12 s."""
    from oracle import mdi_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    op = O.Partition(cfg, w, lo, hi, has_embed=embed)
    T, budget_s, max_dec = prompt, 12.0, 600
    a = S.make_prompts(cfg, seed, 1, T)[0] if embed else S.make_activations(cfg, seed, 0, T)
    t0 = time.perf_counter()
    op.prefill(0, a)
    t1 = time.perf_counter()
    n_dec = 0
    toks = S.make_prompts(cfg, seed + 3, 1, max_dec)[0] if embed else None
    while n_dec < max_dec and time.perf_counter() - t1 < budget_s and T + n_dec < cfg["max_ctx"]:
        op.decode_step(0, toks[n_dec] if embed else S.make_activations(cfg, seed, 0, 1, step=n_dec + 1)[0])
        n_dec += 1
    t2 = time.perf_counter()
    return {"value": n_dec / (t2 - t1), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"float64 numpy oracle, same partition and weights, 1 sample: first visit of {T} tokens "
                      f"({t1 - t0:.1f} s, {T / (t1 - t0):.1f} tokens/s, not counted) then {n_dec} decode steps at context {T}+ ({t2 - t1:.1f} s)",
            "host_cores_available": len(os.sched_getaffinity(0))}


def paper_run(args, torch, mdi, S):
    """The paper's rate experiment (Sec. IV-B: 3 samples, 800 tokens each, from a one-token prompt) on the shapes and
    cuts it names (Sec. IV-A: the 304M model whole, 5/7 and 2/5/5; TinyLlama 10/12 and 6/8/8), random-init weights,
    plus a deliberately unbalanced cut.  Every node of the ring is a partition on this one GPU, so the nodes take
    turns instead of working side by side: the generation rate does not grow with the number of nodes here.  What
    the cut decides on real nodes - how long each waits for the slowest (Sec. III-C) - is reported from each
    stage's measured time per message."""
    from paper_2505_18164_amd.pipeline import RecurrentPipeline
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    n_seqs, n_new = 3, args.paper_tokens
    if args.paper_run == "nanollama":
        shapes = {"fp32 (the paper's precision)": S.nanollama(S.DT_F32, 2048), "bf16": S.nanollama(S.DT_BF16, 2048)}
        cuts = {"1 node": (12,), "2 nodes 5/7": (5, 7), "3 nodes 2/5/5": (2, 5, 5), "3 nodes 1/1/10 (unbalanced)": (1, 1, 10)}
    else:
        shapes = {"bf16": S.tinyllama(S.DT_BF16, 2048)}
        cuts = {"1 node": (22,), "2 nodes 10/12": (10, 12), "3 nodes 6/8/8": (6, 8, 8), "3 nodes 2/2/18 (unbalanced)": (2, 2, 18)}
    seed = 20250518 + (11 if args.paper_run == "nanollama" else 12)
    out = {"metric": f"generated tokens/s, {n_seqs} samples x {n_new} tokens from one-token prompts ({args.paper_run} shape)",
           "unit": "tokens/s", "n_gpus": 1, "data": "synthetic", "higher_is_better": True, "runs": []}
    for sname, cfg in shapes.items():
        w = S.make_weights(cfg, seed)
        prompts = [torch.from_numpy(p[:1]).to(dev) for p in S.make_prompts(cfg, seed, n_seqs, 4)]
        for cname, cut in cuts.items():
            bounds = [0]
            for c in cut:
                bounds.append(bounds[-1] + c)
            parts = [mdi.Partition(cfg, w, bounds[i], bounds[i + 1], has_embed=i == 0, has_head=i == 0, max_seqs=n_seqs,
                                   kv_page_tokens=64, max_prefill=8, stream=torch.cuda.Stream()) for i in range(len(cut))]
            pipe = RecurrentPipeline(parts, head=parts[0])
            rec = {"storage": sname, "cut": cname}
            modes = [("one message per call (the paper's rule)", False), ("queue drained per call", True)]
            if all(p.info(4) for p in parts) and parts[0].info(6):
                modes.append(("queue drained, one pass over the weights", "shared"))
            for mname, drain in modes:
                best = None
                for rep in range(2):                       # the first run also loads the kernels
                    pipe.reset(n_seqs)
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    toks, _, _ = pipe.generate(prompts, n_new, drain=drain)
                    torch.cuda.synchronize()
                    dt = time.perf_counter() - t0
                    best = dt if best is None else min(best, dt)
                for p in parts:
                    p.sync()
                rec[mname] = {"tokens_per_s": n_seqs * n_new / best, "seconds": best}
            # time per message of every stage, alone, at a context of about half the run: what each node of a real
            # ring would be busy for per token; the others wait for the slowest (Sec. III-C)
            stage_ms = []
            for i, p in enumerate(parts):
                x = (torch.zeros((1,), dtype=torch.int32, device=dev) if i == 0
                     else torch.randn((cfg["d_model"],), device=dev).to(p.tdtype))
                y = torch.empty((cfg["d_model"],), dtype=p.tdtype, device=dev)
                tok = torch.empty((1,), dtype=torch.int32, device=dev)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                with torch.cuda.stream(p.stream):
                    for rep in range(2):
                        e0.record()
                        for _ in range(100):
                            p.decode_step(0, x, y)
                            if i == 0:
                                p.sample_greedy(0, y, tok)
                        e1.record()
                        p.sync()
                stage_ms.append(e0.elapsed_time(e1) / 100)
            slowest = max(stage_ms)
            rec["stage_ms_per_message"] = stage_ms
            rec["stage_busy_fraction_on_its_own_gpu"] = [t / slowest for t in stage_ms]
            rec["tokens_per_s_bound_with_a_gpu_per_stage"] = 1000.0 / slowest * min(1.0, n_seqs / len(cut))
            out["runs"].append(rec)
            print(f"bench.py: {sname}, {cname} done", file=sys.stderr, flush=True)
            del pipe, parts
        del w
    best = max(r[m]["tokens_per_s"] for r in out["runs"] for m in r if isinstance(r[m], dict) and "tokens_per_s" in r[m])
    out["value"] = best
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (one partition per GPU is the multi-GPU design; "
              "no collectives or second device are used). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2505_18164_amd import mdi, synth as S

    if args.paper_run:
        print(json.dumps(paper_run(args, torch, mdi, S)))
        return
    wl = S.WORKLOADS[args.workload]
    cfg, seed = wl["cfg"](), S.workload_seed(args.workload)
    n_seqs, prompt = wl["n_seqs"], wl["prompt"]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    d = cfg["d_model"]
    queue, windows = plan_windows(n_seqs, prompt, cfg["max_ctx"], args.steps, args.warmup, args.queue)
    steps_run = sum(t for _, t in windows)
    warmup_run = windows[0][0]

    # ---- partitions: the first one is the benchmarked one; the others of a several-partition workload are built
    #      for the side runs (same shapes; their weight VALUES repeat the first partition's, each in its own arena)
    t0 = time.perf_counter()
    lo, hi = wl["parts"][0]
    embed = lo == 0
    w = S.make_weights(cfg, seed, lo, hi, embed=embed, head=False)
    max_prefill = max(prompt, cfg["max_ctx"] - 8 if args.ctx_sweep else prompt)

    def build_part(plo, phi, weights, has_embed):
        return mdi.Partition(cfg, weights, plo, phi, has_embed=has_embed, max_seqs=n_seqs, kv_page_tokens=64,
                             decode_path=args.decode_path, max_prefill=max_prefill)

    part = build_part(lo, hi, w, embed)
    setup_s = time.perf_counter() - t0
    tdt = part.tdtype

    def first_inputs(p_embed, T):
        if p_embed:
            return [torch.from_numpy(p).to(dev) for p in S.make_prompts(cfg, seed, n_seqs, T)]
        g = torch.Generator(device=dev).manual_seed(seed + 2)
        return [torch.randn((T, d), generator=g, device=dev, dtype=torch.float32).to(tdt) for _ in range(n_seqs)]

    def step_inputs(p_embed):
        if p_embed:
            g = torch.Generator(device=dev).manual_seed(seed + 3)
            return [torch.randint(0, cfg["vocab"], (1,), generator=g, device=dev, dtype=torch.int32) for _ in range(n_seqs)]
        g = torch.Generator(device=dev).manual_seed(seed + 3)
        return [torch.randn((d,), generator=g, device=dev, dtype=torch.float32).to(tdt) for _ in range(n_seqs)]

    def run(p, p_embed, T, wins, q, shared=False):
        """Per window: first visits of all samples at T tokens (timed separately), warm-up steps, then the timed
        steps, q messages per call (shared: one pass over the weights per call).  Returns rates over all windows."""
        ins = first_inputs(p_embed, T)
        outs = [torch.empty((T, d), dtype=tdt, device=dev) for _ in range(n_seqs)]
        xs = step_inputs(p_embed)
        douts = [torch.empty((d,), dtype=tdt, device=dev) for _ in range(q)]
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for s in range(n_seqs):
            p.seq_reset(s)
        p.prefill(0, ins[0], outs[0])          # untimed: loads the first-visit kernels
        p.seq_reset(0)
        torch.cuda.synchronize()

        def visit(ids):
            if len(ids) == 1:
                p.decode_step(ids[0], xs[ids[0]], douts[0])
            elif shared:
                p.decode_batch(ids, [xs[i] for i in ids], douts[:len(ids)])
            else:
                p.decode_steps(ids, [xs[i] for i in ids], douts[:len(ids)])

        total_ms, total_steps, launches, prefill_ms, ctx_sum = 0.0, 0, 0, None, 0.0
        for wi, (wu, timed) in enumerate(wins):
            for s in range(n_seqs):
                p.seq_reset(s)
            torch.cuda.synchronize()
            e0.record()
            for s in range(n_seqs):
                p.prefill(s, ins[s], outs[s])
            e1.record()
            torch.cuda.synchronize()
            if prefill_ms is None:
                prefill_ms = e0.elapsed_time(e1) / n_seqs
            for ids in calls_of(0, wu, q, n_seqs):
                visit(ids)
            torch.cuda.synchronize()
            ctx_first = p.seq_len(wu % n_seqs) + 1
            calls = calls_of(wu, timed, q, n_seqs)
            e0.record()
            for ids in calls:
                visit(ids)
            e1.record()
            p.sync()
            total_ms += e0.elapsed_time(e1)
            total_steps += timed
            launches += len(calls)
            ctx_last = max(p.seq_len(s) for s in range(n_seqs))
            ctx_sum += 0.5 * (ctx_first + ctx_last) * timed
        ms = total_ms / total_steps
        ctx_mean = int(round(ctx_sum / total_steps))
        # algorithmic bytes: every message reads its sample's cache and writes its row; the layer matrices are read
        # once per message, or once per call when the call's messages share a pass
        total_bytes = total_steps * p.step_bytes(ctx_mean)
        if shared:
            total_bytes -= (total_steps - launches) * p.info(5)
        nbytes = total_bytes / total_steps
        return dict(ctx=ctx_mean, ms_per_step=ms, tokens_per_s=1000.0 / ms, bytes_per_step=nbytes,
                    gbs=nbytes / ms / 1e6, prefill_ms=prefill_ms, launches=launches, steps=total_steps,
                    avg_launch_us=total_ms * 1e3 / launches)

    if args.calib_copy_mib:
        src = torch.empty(args.calib_copy_mib << 20, dtype=torch.uint8, device=dev).zero_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    shared = queue > 1 and part.info(4) > 0 and args.passes != "per-message"
    if args.passes == "shared" and not shared:
        print("bench.py: this partition cannot share a pass over the weights among messages; timing a pass per message",
              file=sys.stderr)
    main_run = run(part, embed, prompt, windows, queue, shared)
    n_local = hi - lo
    params = sum(a * b for a, b in S.layer_tensor_shapes(cfg).values())
    prefill_flops = n_local * (2.0 * prompt * params + 2.0 * prompt * prompt * cfg["n_head"] * cfg["head_dim"])
    prefill_tflops = prefill_flops / (main_run["prefill_ms"] * 1e-3) / 1e12
    bf16 = cfg["dtype"] == S.DT_BF16

    path_kind = part.info(0)          # 2 = persistent launch, 1 = one kernel per operation
    persistent = path_kind == 2
    side = not args.no_side_runs
    # next to it: the same calls with a pass over the weights per message, and the paper's own rule, one message
    # at a time
    one_run, per_msg_run = None, None
    if side and queue > 1:
        _, one_w = plan_windows(n_seqs, prompt, cfg["max_ctx"], min(400, steps_run), min(40, warmup_run), 1)
        one_run = run(part, embed, prompt, one_w, 1)
        if shared:
            _, pm_w = plan_windows(n_seqs, prompt, cfg["max_ctx"], min(800, steps_run), min(40, warmup_run), queue)
            per_msg_run = run(part, embed, prompt, pm_w, queue, False)
    kernels = {}
    if persistent:
        # the whole step is one kernel launch; its mean duration over the timed region (HIP events on the
        # partition's stream, launches back to back) against the bytes the launch must move
        in_launch = main_run["steps"] / main_run["launches"]          # messages a launch carried on average
        traffic, traffic_src = measured_traffic(args.workload, queue, shared)
        kname = (f"k_step_batch (persistent decode launch, all layers, {queue} messages share one pass over the weights)" if shared
                 else f"k_step (persistent decode launch, all layers, {queue} message(s) per launch, a pass over the weights each)")
        roofline = {"bound": "hbm", "kernel": kname,
                    "achieved": main_run["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": main_run["gbs"] / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_src,
                    "avg_launch_us": main_run["avg_launch_us"],
                    "bytes_per_launch": main_run["bytes_per_step"] * in_launch, "messages_per_launch": in_launch,
                    "launches_timed": main_run["launches"],
                    "workgroups": part.info(1) * (2 if queue > 1 and not shared else 1),
                    "kernel_rev": kernel_rev()}
    else:
        # dominant kernel: the MLP up(+gate) projection GEMV, timed with HIP events inside the library
        us, kbytes = part.time_kernel(2, 50)
        roofline = {"bound": "hbm", "kernel": "k_gemv MLP up+gate projection", "achieved": kbytes / us / 1e3,
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": kbytes / us / 1e3 / HBM_PEAK_GBS, "traffic": None,
                    "avg_launch_us": us, "bytes_per_launch": kbytes}
        for which, name in ((1, "attn_out_proj"), (2, "mlp_up"), (3, "mlp_down")):
            u_, b_ = part.time_kernel(which, 50)
            kernels[name] = {"avg_us": u_, "GB/s": b_ / u_ / 1e3}

    sweep = None
    if args.ctx_sweep:
        sweep = []
        for T in (prompt + wl["n_new"] // 2, prompt + wl["n_new"] - 8 - -(-440 // n_seqs)):   # 440 = timed + warm-up steps
            r = run(part, embed, T, [(40, 400)], queue, shared)
            sweep.append({k: r[k] for k in ("ctx", "ms_per_step", "tokens_per_s", "gbs")})

    result = {
        "metric": f"decode tokens/s per partition ({n_seqs} seqs in flight)",
        "value": main_run["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": steps_run, "warmup": warmup_run,
        "ms_per_step": main_run["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": wl["name"], "layers": [lo, hi], "seqs_in_flight": n_seqs, "prompt": prompt,
                   "context_during_timing": main_run["ctx"], "kv_page_tokens": 64, "messages_per_call": queue,
                   "weight_passes": "one per call (mdi_decode_batch)" if shared else "one per message",
                   "timed_windows": len(windows), "requested": {"steps": args.steps, "warmup": args.warmup},
                   "decode_path": {2: "persistent", 1: "per_op"}[path_kind]},
        "step_bytes": main_run["bytes_per_step"], "step_GBps": main_run["gbs"],
        "step_frac_of_hbm_peak": main_run["gbs"] / HBM_PEAK_GBS,
        "roofline": roofline, "kernels": kernels,
        "prefill": {"tokens": prompt, "ms_per_sample": main_run["prefill_ms"], "TFLOP/s": prefill_tflops,
                    "frac_of_bf16_mfma_peak": prefill_tflops / MFMA_BF16_PEAK_TFLOPS if bf16 else None,
                    "frac_of_fp32_vector_peak": None if bf16 else prefill_tflops / FP32_VECTOR_PEAK_TFLOPS},
        "setup_s": setup_s,
    }
    if side and prompt >= 512:
        # the same first visit handed over in pieces of 256 positions (mdi_prefill_chunk): later pieces attend to the
        # positions already in the cache, so other samples' messages fit in between the pieces of a long prompt
        piece = 256
        ins = first_inputs(embed, prompt)[0]
        outs = torch.empty((prompt, d), dtype=tdt, device=dev)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(prompt // piece + 2)]
        for rep in range(2):                       # the second pass is the timed one
            part.seq_reset(0)
            torch.cuda.synchronize()
            ev[0].record()
            for i, at in enumerate(range(0, prompt, piece)):
                part.prefill_chunk(0, ins[at:at + piece], outs[at:at + piece])
                ev[i + 1].record()
            torch.cuda.synchronize()
        n_p = len(range(0, prompt, piece))
        result["prefill"]["in_pieces"] = {"piece": piece, "ms_per_piece": [ev[i].elapsed_time(ev[i + 1]) for i in range(n_p)],
                                          "ms_per_sample": ev[0].elapsed_time(ev[n_p])}
    if one_run:
        result["one_message_per_launch"] = {"ms_per_step": one_run["ms_per_step"], "tokens_per_s": one_run["tokens_per_s"],
                                            "step_GBps": one_run["gbs"], "frac_of_hbm_peak": one_run["gbs"] / HBM_PEAK_GBS,
                                            "steps": one_run["steps"]}
    if per_msg_run:
        result["one_pass_per_message"] = {"ms_per_step": per_msg_run["ms_per_step"], "tokens_per_s": per_msg_run["tokens_per_s"],
                                          "step_GBps": per_msg_run["gbs"], "frac_of_hbm_peak": per_msg_run["gbs"] / HBM_PEAK_GBS,
                                          "steps": per_msg_run["steps"]}
    if sweep:
        result["ctx_sweep"] = sweep

    # ---- workloads of several partitions: each partition alone, then all of them driven round-robin -----------
    if side and len(wl["parts"]) > 1:
        others = []
        for (plo, phi) in wl["parts"][1:]:
            # same shapes as the first partition; blocks only (a secondary node), fed activations
            w2 = {"layers": {plo + i: w["layers"][lo + i] for i in range(phi - plo)}}
            others.append(build_part(plo, phi, w2, False))
        all_parts = [(part, embed)] + [(p, False) for p in others]
        sw = plan_windows(n_seqs, prompt, cfg["max_ctx"], min(400, steps_run), min(40, warmup_run), queue)[1]
        alone = [{"layers": list(wl["parts"][0]), "tokens_per_s": main_run["tokens_per_s"], "step_GBps": main_run["gbs"]}]
        for (p, pe), (plo, phi) in zip(all_parts[1:], wl["parts"][1:]):
            r = run(p, pe, prompt, sw, queue, shared)
            alone.append({"layers": [plo, phi], "tokens_per_s": r["tokens_per_s"], "step_GBps": r["gbs"]})
        # all partitions, each on a stream of its own in the library's eyes (here: one stream; persistent launches
        # of different partitions are ordered one after the other anyway), visited in ring order per round
        wu, timed = sw[0]
        ins = {id(p): (first_inputs(pe, prompt), step_inputs(pe)) for p, pe in all_parts}
        buf = torch.empty((prompt, d), dtype=tdt, device=dev)
        douts = [torch.empty((d,), dtype=tdt, device=dev) for _ in range(queue)]
        for p, pe in all_parts:
            for s in range(n_seqs):
                p.seq_reset(s)
                p.prefill(s, ins[id(p)][0][s], buf)

        def ring_visit(ids):
            for p, pe in all_parts:
                xs = ins[id(p)][1]
                if len(ids) == 1:
                    p.decode_step(ids[0], xs[ids[0]], douts[0])
                elif shared:
                    p.decode_batch(ids, [xs[i] for i in ids], douts[:len(ids)])
                else:
                    p.decode_steps(ids, [xs[i] for i in ids], douts[:len(ids)])

        n_calls = len(calls_of(wu, timed, queue, n_seqs))
        for ids in calls_of(0, wu, queue, n_seqs):
            ring_visit(ids)
        torch.cuda.synchronize()
        ctx0 = part.seq_len(wu % n_seqs) + 1
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for ids in calls_of(wu, timed, queue, n_seqs):
            ring_visit(ids)
        e1.record()
        for p, _ in all_parts:
            p.sync()
        ms = e0.elapsed_time(e1)
        ctx_mean = (ctx0 + max(part.seq_len(s) for s in range(n_seqs))) // 2
        agg_bytes = sum(p.step_bytes(ctx_mean) * timed - ((timed - n_calls) * p.info(5) if shared else 0) for p, _ in all_parts)
        result["all_partitions"] = {
            "partitions": len(all_parts), "alone": alone,
            "round_robin": {"partition_steps_per_s": len(all_parts) * timed / ms * 1e3,
                            "model_tokens_per_s": timed / ms * 1e3, "GBps": agg_bytes / ms / 1e6,
                            "frac_of_hbm_peak": agg_bytes / ms / 1e6 / HBM_PEAK_GBS, "steps_per_partition": timed,
                            "context": ctx_mean},
            "note": "partitions 2.. reuse the first partition's weight values in arenas of their own"}
        del others, all_parts, ins

    if not args.no_output_layers:
        # the starter's output layers (final norm, vocabulary projection, argmax) of the same model, on a partition
        # of their own as in the paper's layout; one call per generated token
        L = cfg["n_layer"]
        hw = S.make_weights(cfg, seed, L, L, embed=False, head=True)
        hp = mdi.Partition(cfg, hw, L, L, has_head=True, max_seqs=max(1, n_seqs))
        g = torch.Generator(device=dev).manual_seed(seed + 4)
        x = torch.randn((d,), generator=g, device=dev, dtype=torch.float32).to(tdt)
        tok = torch.empty((1,), dtype=torch.int32, device=dev)
        for _ in range(10):
            hp.sample_greedy(0, x, tok)
        torch.cuda.synchronize()
        h0, h1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        h0.record()
        for _ in range(100):
            hp.sample_greedy(0, x, tok)
        h1.record()
        hp.sync()
        us = h0.elapsed_time(h1) * 10.0
        hb = hp.step_bytes(0, head=True)
        result["output_layers"] = {"vocab": cfg["vocab"], "us_per_call": us, "bytes": hb, "GB/s": hb / us / 1e3,
                                   "frac_of_hbm_peak": hb / us / 1e3 / HBM_PEAK_GBS}
        if hp.info(6) and n_seqs > 1:
            # the same layers for every sample in flight with one pass over the vocabulary matrix (mdi_sample_batch)
            m = min(n_seqs, int(hp.info(6)))
            xs = [torch.randn((d,), generator=g, device=dev, dtype=torch.float32).to(tdt) for _ in range(m)]
            toks = torch.empty((m,), dtype=torch.int32, device=dev)
            ids = list(range(m))
            for _ in range(10):
                hp.sample_batch(ids, xs, tokens_out=toks)
            torch.cuda.synchronize()
            h0.record()
            for _ in range(100):
                hp.sample_batch(ids, xs, tokens_out=toks)
            h1.record()
            hp.sync()
            usb = h0.elapsed_time(h1) * 10.0
            bb = hb + (m - 1) * (d * xs[0].element_size() + 4)
            result["output_layers"]["shared_pass"] = {
                "samples_per_call": m, "us_per_call": usb, "us_per_sample": usb / m, "bytes": bb, "GB/s": bb / usb / 1e3,
                "frac_of_hbm_peak": bb / usb / 1e3 / HBM_PEAK_GBS}
        del hp, hw
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, w, lo, hi, seed, S, prompt, embed)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
