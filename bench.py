"""Benchmark of the partition decode hot path on one MI355X.

One step = one later visit of one sample (Sec. III-D) to the partition (all
layers: norm, fused QKV + RoPE + KV append, paged attention, output projection,
MLP), every message forwarded on its own with its own pass over the weights.
The N samples in flight are visited round-robin, so consecutive steps read
different KV caches (the rotating-cache access pattern).  By default the
messages of all N samples are handed over per call (mdi_decode_steps: the
node's input queue, Sec. III-A, drained in one launch); `--queue 1` hands them
over one at a time (mdi_decode_step), and the default run reports that rate
too.  Inputs, weights and caches are resident in HBM before the timed region;
prompts are prefilled (first visit) before it and timed separately.

Prints ONE JSON line (see the keys below).
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, vendor figure
# HBM bytes per k_step launch from rocprofv3 FETCH_SIZE + WRITE_SIZE runs of this script
# ((workload, messages per launch) -> bytes);
# the numbers and the commands are in profiles/k_step_c4_decode_hbm_counters.md
MEASURED_TRAFFIC = {(4, 8): 2.3804e10, (4, 1): 3.4074e9}
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1600)
    ap.add_argument("--warmup", type=int, default=80)
    ap.add_argument("--workload", type=int, default=4, help="index into the five benchmark configs (1-5)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-output-layers", action="store_true", help="skip timing the output layers of the same model")
    ap.add_argument("--ctx-sweep", action="store_true", help="also time decode at the middle and end context")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MiB (reference for HBM byte counters)")
    ap.add_argument("--decode-path", type=int, default=0, help="0 = automatic (persistent single-launch step), 1 = one kernel per operation, 3 = persistent launch with streaming/exchange wavefronts on tiled matrices")
    ap.add_argument("--queue", type=int, default=0,
                    help="messages of different samples handed to the partition per call: 0 = all samples in flight "
                         "(mdi_decode_steps drains the queue), 1 = one at a time (mdi_decode_step); must divide the "
                         "number of samples in flight")
    return ap.parse_args()


def cpu_baseline(cfg, w, lo, hi, seed, S):
    """The oracle as it stands, timed on this host: a short first visit plus a few decode steps."""
    import numpy as np
    from oracle import mdi_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    op = O.Partition(cfg, w, lo, hi)
    T, budget_s, max_dec = 128, 12.0, 600
    a = S.make_activations(cfg, seed, 0, T)
    t0 = time.perf_counter()
    op.prefill(0, a)
    t1 = time.perf_counter()
    n_dec = 0
    while n_dec < max_dec and time.perf_counter() - t1 < budget_s:      # about 12 s of decode steps
        op.decode_step(0, S.make_activations(cfg, seed, 0, 1, step=n_dec + 1)[0])
        n_dec += 1
    t2 = time.perf_counter()
    return {"value": n_dec / (t2 - t1), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"float64 numpy oracle, same partition and weights, 1 sample: first visit of {T} tokens "
                      f"({t1 - t0:.1f} s, not counted) then {n_dec} decode steps at context {T}+ ({t2 - t1:.1f} s)",
            "host_cores_available": len(os.sched_getaffinity(0))}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (one partition per GPU is the multi-GPU design; "
              "no collectives or second device are used). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2505_18164_amd import mdi, synth as S

    wl = S.WORKLOADS[args.workload]
    cfg, seed = wl["cfg"](), S.workload_seed(args.workload)
    lo, hi = wl["parts"][0]
    n_seqs, prompt = wl["n_seqs"], wl["prompt"]
    embed = lo == 0
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    t0 = time.perf_counter()
    w = S.make_weights(cfg, seed, lo, hi, embed=embed, head=False)
    part = mdi.Partition(cfg, w, lo, hi, has_embed=embed, max_seqs=n_seqs, kv_page_tokens=64, decode_path=args.decode_path,
                         max_prefill=max(prompt, cfg["max_ctx"] - 8 if args.ctx_sweep else prompt))
    setup_s = time.perf_counter() - t0
    d = cfg["d_model"]
    tdt = part.tdtype

    def first_inputs(T):
        if embed:
            return [torch.from_numpy(p).to(dev) for p in S.make_prompts(cfg, seed, n_seqs, T)]
        g = torch.Generator(device=dev).manual_seed(seed + 2)
        return [torch.randn((T, d), generator=g, device=dev, dtype=torch.float32).to(tdt) for _ in range(n_seqs)]

    def step_inputs():
        if embed:
            return [torch.randint(0, cfg["vocab"], (1,), device=dev, dtype=torch.int32) for _ in range(n_seqs)]
        g = torch.Generator(device=dev).manual_seed(seed + 3)
        return [torch.randn((d,), generator=g, device=dev, dtype=torch.float32).to(tdt) for _ in range(n_seqs)]

    def run(T, steps, warmup, q):
        """Prefill all samples at T tokens, then warm up and time `steps` decode steps, q messages per call."""
        for s in range(n_seqs):
            part.seq_reset(s)
        ins = first_inputs(T)
        outs = [torch.empty((T, d), dtype=tdt, device=dev) for _ in range(n_seqs)]
        part.prefill(0, ins[0], outs[0])          # untimed: loads the first-visit kernels
        part.seq_reset(0)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for s in range(n_seqs):
            part.prefill(s, ins[s], outs[s])
        e1.record()
        torch.cuda.synchronize()
        prefill_ms = e0.elapsed_time(e1) / n_seqs
        xs = step_inputs()
        douts = [torch.empty((d,), dtype=tdt, device=dev) for _ in range(q)]

        def visit(k):                      # messages k .. k + q - 1 of the round-robin order
            if q == 1:
                part.decode_step(k % n_seqs, xs[k % n_seqs], douts[0])
            else:
                ids = [(k + i) % n_seqs for i in range(q)]
                part.decode_steps(ids, [xs[i] for i in ids], douts)

        for k in range(0, warmup, q):
            visit(k)
        torch.cuda.synchronize()
        ctx_first = part.seq_len(0) + 1
        e0.record()
        for k in range(0, steps, q):
            visit(warmup + k)
        e1.record()
        part.sync()
        ms = e0.elapsed_time(e1) / steps
        ctx_last = max(part.seq_len(s) for s in range(n_seqs))
        ctx_mean = (ctx_first + ctx_last) // 2
        nbytes = part.step_bytes(ctx_mean)
        return dict(ctx=ctx_mean, ms_per_step=ms, tokens_per_s=1000.0 / ms, bytes_per_step=nbytes,
                    gbs=nbytes / ms / 1e6, prefill_ms=prefill_ms)

    if args.calib_copy_mib:
        src = torch.empty(args.calib_copy_mib << 20, dtype=torch.uint8, device=dev).zero_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    queue = args.queue if args.queue else n_seqs
    if queue < 1 or n_seqs % queue or args.steps % queue or args.warmup % queue:
        print("bench.py: --queue must divide the samples in flight, --steps and --warmup", file=sys.stderr)
        sys.exit(2)
    per_seq = -(-(args.warmup + args.steps) // n_seqs)
    if prompt + per_seq > cfg["max_ctx"]:
        print(f"bench.py: {args.warmup} + {args.steps} steps over {n_seqs} samples need a context of {prompt + per_seq}, "
              f"this workload's caches hold {cfg['max_ctx']}; use fewer steps", file=sys.stderr)
        sys.exit(2)
    main_run = run(prompt, args.steps, args.warmup, queue)
    n_local = hi - lo
    params = sum(a * b for a, b in S.layer_tensor_shapes(cfg).values())
    prefill_flops = n_local * (2.0 * prompt * params + 2.0 * prompt * prompt * cfg["n_head"] * cfg["head_dim"])
    prefill_tflops = prefill_flops / (main_run["prefill_ms"] * 1e-3) / 1e12

    persistent_kind = part.info(0) in (2, 3)
    # the paper's own rule, one message at a time, next to the queue-draining figure
    one_steps = min(400, (cfg["max_ctx"] - prompt - 1) * n_seqs * 10 // 11 // n_seqs * n_seqs)
    one_run = run(prompt, one_steps, one_steps // 10, 1) if (queue > 1 and persistent_kind and one_steps > 0) else None
    path_kind = part.info(0)          # 2 = persistent launch, 3 = persistent launch with streaming + exchange wavefronts on tiled matrices, 1 = per operation
    persistent = path_kind in (2, 3)
    kernels = {}
    if persistent:
        # the whole step is one kernel launch; its mean duration over the timed region (HIP events on the
        # partition's stream, launches back to back) against the bytes a step must move
        in_launch = queue if path_kind == 2 else 1          # messages one launch carries
        roofline = {"bound": "hbm", "kernel": ("k_step2" if path_kind == 3 else "k_step") +
                    f" (persistent decode launch, all layers, {in_launch} message(s) per launch)",
                    "achieved": main_run["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": main_run["gbs"] / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC.get((args.workload, in_launch)),
                    "avg_launch_us": main_run["ms_per_step"] * 1e3 * in_launch,
                    "bytes_per_launch": main_run["bytes_per_step"] * in_launch, "messages_per_launch": in_launch,
                    "workgroups": part.info(1) * (2 if in_launch > 1 else 1), "lds_bytes": part.info(2)}
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
            r = run(T, 400, 40, queue)
            sweep.append({k: r[k] for k in ("ctx", "ms_per_step", "tokens_per_s", "gbs")})

    result = {
        "metric": f"decode tokens/s per partition ({n_seqs} seqs in flight)",
        "value": main_run["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_run["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg["dtype"] == S.DT_BF16 else "f32", "data": "synthetic",
        "config": {"workload": wl["name"], "layers": [lo, hi], "seqs_in_flight": n_seqs, "prompt": prompt,
                   "context_during_timing": main_run["ctx"], "kv_page_tokens": 64, "messages_per_call": queue,
                   "decode_path": {3: "persistent_tiles", 2: "persistent", 1: "per_op"}[path_kind]},
        "step_bytes": main_run["bytes_per_step"], "step_GBps": main_run["gbs"],
        "step_frac_of_hbm_peak": main_run["gbs"] / HBM_PEAK_GBS,
        "roofline": roofline, "kernels": kernels,
        "prefill": {"tokens": prompt, "ms_per_sample": main_run["prefill_ms"], "TFLOP/s": prefill_tflops,
                    "frac_of_bf16_mfma_peak": prefill_tflops / MFMA_BF16_PEAK_TFLOPS},
        "setup_s": setup_s,
    }
    if not args.no_output_layers:
        # the starter's output layers (final norm, vocabulary projection, argmax) of the same model, on a partition
        # of their own as in the paper's layout; one call per generated token
        L = cfg["n_layer"]
        hw = S.make_weights(cfg, seed, L, L, embed=False, head=True)
        hp = mdi.Partition(cfg, hw, L, L, has_head=True, max_seqs=1)
        x = torch.randn((d,), device=dev, dtype=torch.float32).to(tdt)
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
        del hp, hw
    if one_run:
        result["one_message_per_launch"] = {"ms_per_step": one_run["ms_per_step"], "tokens_per_s": one_run["tokens_per_s"],
                                            "step_GBps": one_run["gbs"], "frac_of_hbm_peak": one_run["gbs"] / HBM_PEAK_GBS}
    if sweep:
        result["ctx_sweep"] = sweep
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, w, lo, hi, seed, S)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
