#!/usr/bin/env python3
"""Benchmark of the PaSS decode path on one MI355X.

A "step" is one iteration of Algorithm 1: a drafting call on (last token, k look-ahead rows), its
sampling epilogue, a validation call on the drafted block and the accept / reject epilogue, for
every sequence of the batch.  Inputs (weights, prompts' K/V) are resident in HBM before the timed
region starts.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--k K] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix rate


def algorithmic_bytes_per_call(shape, k, ctx_lens):
    """Bytes one (1+k)-row model call must move: every streamed parameter once, the cached K/V of
    every sequence once, the K/V rows written, the fp32 logits."""
    esz = 2 if shape.dtype == 1 else 4
    M = (1 + k) * len(ctx_lens)
    kv_tok = 2 * shape.n_layers * shape.n_heads * shape.head_dim * esz
    return shape.n_params_streamed * esz + kv_tok * sum(ctx_lens) + kv_tok * M + 4 * M * shape.vocab


def gate_up_kernel_bytes(shape, M):
    """Algorithmic bytes of one launch of the dominant kernel (gate/up GEMM + SiLU*mul): both
    weight matrices once, the M input rows and the M activation rows written (each a pair of bf16
    halves, 4 bytes per element)."""
    esz = 2 if shape.dtype == 1 else 4
    return 2 * shape.d_ffn * shape.d_model * esz + M * shape.d_model * 4 + M * shape.d_ffn * 4


def prefill_report(shape, prompts, rows, seconds):
    """Prompt pass: rows/s and the matrix multiplies' rate.  `flops` counts the projections only
    (2 * rows * parameters of the layers); the matrix cores issue twice that, every activation
    being a (hi, lo) pair of bf16 values, and `mfma_frac` prices the issued rate at the bf16 peak."""
    d, D, F, L = shape.d_model, shape.n_heads * shape.head_dim, shape.d_ffn, shape.n_layers
    flops = 2.0 * rows * L * (3 * D * d + d * D + 3 * F * d)
    issued = 2.0 * flops if shape.dtype == 1 else flops
    return {"prompt_rows": rows, "ms": seconds * 1e3, "rows_per_s": rows / seconds,
            "matmul_TFLOPs": flops / seconds / 1e12, "mfma_issued_TFLOPs": issued / seconds / 1e12,
            "mfma_frac": issued / seconds / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "pass": ("tiled, one call for the batch (pass_prefill_batch)" if shape.dtype == 1 and sum(len(p) - 1 for p in prompts) > 128
                     else "decode kernels in chunks")}


def measured_traffic(workload_name):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary
    (FETCH_SIZE and WRITE_SIZE runs, scaled by a copy kernel of known size); None if there is no
    summary for this workload."""
    path = os.path.join(ROOT, "profiles", "7b_k4_gate_up_gemm_hbm_traffic.txt")  # counters cannot be read from inside the run
    if workload_name != "7b_k4_greedy" or not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch:"):
            return int(line.split(":")[1])
    return None


def host_copy(W):
    """The device-generated model as host numpy arrays (bf16 as uint16 bit patterns): the bytes the
    oracle reads are the bytes the library was given."""
    import torch

    def cv(t):
        t = t.contiguous()
        return (t.view(torch.uint16) if t.dtype == torch.bfloat16 else t).cpu().numpy()
    return {name: [cv(t) for t in v] if isinstance(v, list) else cv(v) for name, v in W.items()}


def cpu_baseline(w, k, W_host, prompt, n_iters=8, prompt_rows=32):
    """The CPU oracle as it stands, timed on this machine's host cores on a bounded sample of the
    same workload: the full model (all layers, the same weight bytes), the first tokens of the
    workload's prompt, then n_iters PaSS iterations, drafting and validation calls timed apart.
    The context is short because the oracle's prompt pass costs about 0.4 s per row at 7B size;
    the cost of an oracle decode call is the weights' (attention over 512 keys would add 2 %)."""
    sys.path.insert(0, os.path.join(ROOT, "oracle"))
    import pass_oracle as O

    cores = len(os.sched_getaffinity(0))
    threads = int(os.environ.get("OMP_NUM_THREADS", cores))
    model = O.Model(w.shape, W_host, k)
    seq = model.sequence(prompt_rows + 1 + (n_iters + 2) * (k + 2) + k)
    t0 = time.perf_counter()
    seq.prefill(prompt[:prompt_rows + 1])
    prefill_s = time.perf_counter() - t0
    seed = 1
    seq.draft(w.temperature, seed)
    seq.verify(w.temperature, seed)  # one untimed iteration
    n0 = seq.n_generated
    t_d = t_v = 0.0
    for _ in range(n_iters):
        t0 = time.perf_counter()
        seq.draft(w.temperature, seed)
        t1 = time.perf_counter()
        seq.verify(w.temperature, seed)
        t_d += t1 - t0
        t_v += time.perf_counter() - t1
    toks = seq.n_generated - n0
    cpu = ""
    try:
        cpu = [l.split(":", 1)[1].strip() for l in open("/proc/cpuinfo") if l.startswith("model name")][0]
    except Exception:
        pass
    return {"value": toks / (t_d + t_v), "unit": "tokens/s", "cores": min(cores, threads), "kind": "oracle",
            "cpu": cpu, "draft_call_ms": t_d / n_iters * 1e3, "verify_call_ms": t_v / n_iters * 1e3,
            "prefill_s": prefill_s, "prefill_rows": prompt_rows, "iterations_timed": n_iters, "tokens": int(toks),
            "sample": f"oracle on the full {w.shape.n_layers}-layer model (the device-generated weights copied to the "
                      f"host), batch 1, k={k}: prompt pass over the first {prompt_rows} prompt rows, one untimed iteration, "
                      f"then {n_iters} PaSS iterations timed (context {prompt_rows + 2}..{seq.kv_len}); decode tokens/s "
                      "excludes the prompt pass"}


def train_report(binding, devgen, synth, torch, np, n_steps, path):
    """Look-ahead embedding training (the paper's Training details: frozen model, batches of 8 sequences
    cut at random positions, AdamW) on the 7B-shaped model: seconds per optimiser step, the prompt pass
    of the batch's prefixes timed apart."""
    w = synth.WORKLOADS["7b_b8_ragged_t1"]  # eight ragged prefixes, k = 4
    prompts = synth.make_prompts(w)
    g = binding.Pass(binding.make_config(w.shape, w.k, w.batch, max(len(p) for p in prompts) + 64, 64), {"path": path})
    g.load_weights(devgen.device_weights(w.shape, w.k, w.lm_head_scale, w.seed))
    torch.cuda.empty_cache()
    g.train_begin(0)
    rng = np.random.default_rng(7)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    g.prefill_batch(list(range(len(prompts))), prompts)
    torch.cuda.synchronize()
    prefill_s = time.perf_counter() - t0
    slots = list(range(w.batch))
    losses = []
    for _ in range(2):
        g.train_step(slots, rng.integers(0, w.shape.vocab, (w.batch, w.k)), 0.01)
    targets = rng.integers(0, w.shape.vocab, (w.batch, w.k))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n_steps):
        losses.append(g.train_step(slots, targets, 0.01))
    torch.cuda.synchronize()
    step_s = (time.perf_counter() - t0) / n_steps
    g.close()
    sh = w.shape
    kv_bytes = sum(len(p) - 1 + w.k + 1 for p in prompts) * sh.n_layers * 2 * sh.n_heads * sh.head_dim * 2
    weight_bytes = 2 * (sh.n_layers * (4 * sh.d_model * sh.n_heads * sh.head_dim + 3 * sh.d_model * sh.d_ffn) + sh.vocab * sh.d_model)
    return {"workload": w.name, "k": w.k, "batch": w.batch, "prefix_len": [len(p) for p in prompts], "steps": n_steps,
            "ms_per_step": step_s * 1e3, "loss_first": losses[0], "loss_last": losses[-1],
            # algorithmic bytes of a step: the frozen weights once forward and once backward (the packed
            # transposes), the batch's cached K/V once by the forward and once by the backward attention
            "algorithmic_bytes_per_step": 2 * weight_bytes + 2 * kv_bytes,
            "achieved_GBps": (2 * weight_bytes + 2 * kv_bytes) / step_s / 1e9,
            "frac_of_peak": (2 * weight_bytes + 2 * kv_bytes) / step_s / 1e9 / HBM_PEAK_GBS,
            "prefix_prompt_pass_ms": prefill_s * 1e3,
            "path": "generic" if path else "auto"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=64,
                    help="untimed iterations first; for about 0.3 s after the weights are generated and the prompt has been "
                         "prefilled (compute-heavy work) the chip runs the memory-bound decode calls about 3 %% slower")
    ap.add_argument("--settle", type=float, default=1.0,
                    help="seconds of idling between the prompt pass and the first untimed iteration")
    ap.add_argument("--workload", default="7b_k4_greedy")
    ap.add_argument("--k", type=int, default=None)
    ap.add_argument("--layers", type=int, default=None, help="debug: fewer layers (not a valid bench line)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-k0", action="store_true", help="skip the k = 0 comparison run")
    ap.add_argument("--top-k", type=int, default=0, help="top-k sampling filter (the paper samples with 10 and 25)")
    ap.add_argument("--temperature", type=float, default=None, help="override the workload's temperature")
    ap.add_argument("--path", type=int, default=0, help="1 = force the generic kernels")
    ap.add_argument("--graph", type=int, default=1)
    ap.add_argument("--gemm-cfg", type=int, action="append", default=[],
                    help="tuning: launch shape override(s), kind*10000 + wavefronts*100 + unroll")
    ap.add_argument("--option", action="append", default=[], metavar="NAME=VALUE",
                    help="tuning: a library option (pass_set_option) to set before the run")
    ap.add_argument("--train-steps", type=int, default=4,
                    help="also time that many look-ahead embedding training steps (on a context of their own; 0 = skip)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (a kernel of known traffic, for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the decode path shards by sequence; no multi-GPU "
              "figure exists); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2311_13581_amd import binding, devgen, synth

    w = synth.WORKLOADS[args.workload]
    if args.layers:
        w = synth.scaled(w, n_layers=args.layers)
    k = w.k if args.k is None else args.k
    shape = w.shape
    temp = w.temperature if args.temperature is None else args.temperature
    top_k = args.top_k
    prompts = synth.make_prompts(w)
    total_iters = args.steps + args.warmup + 8
    max_len = max(len(p) for p in prompts) + max((k + 2) * total_iters, w.max_new + 16 + 3 * (k + 2)) + k + 2
    g = binding.Pass(binding.make_config(shape, k, w.batch, max_len, 64), {"path": args.path, "graph": args.graph})
    for cfg in args.gemm_cfg:
        g.set_option("tune.gemm_cfg", cfg)
    for opt in args.option:
        name, val = opt.split("=")
        g.set_option(name, int(val))
    W = devgen.device_weights(shape, k, w.lm_head_scale, w.seed)
    g.load_weights(W)
    W_host = None if args.no_cpu_baseline else host_copy(W)
    g0 = None
    if k > 0 and not args.no_k0:
        g0 = binding.Pass(binding.make_config(shape, 0, w.batch, max_len, 64), {"path": args.path, "graph": args.graph})
        g0.load_weights(W)
    del W
    torch.cuda.empty_cache()
    g.prefill_batch(list(range(len(prompts))), prompts)
    if g0 is not None:
        g0.prefill_batch(list(range(len(prompts))), prompts)
    slots = list(range(w.batch))
    seed = synth.sampling_seed(w)

    # for a few tenths of a second after compute-heavy work (weight generation, the prompt pass) the
    # chip runs memory-bound kernels up to 3 % slower; idling does as well as running to get past it
    time.sleep(args.settle)
    g.run_iterations(slots, args.warmup, temp, seed, top_k)
    ctx0 = [g.seq_len(s)[0] for s in slots]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    st = g.run_iterations(slots, args.steps, temp, seed, top_k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ctx1 = [g.seq_len(s)[0] for s in slots]

    M = (1 + k) * w.batch
    ctx_mid = [(a + b) / 2 for a, b in zip(ctx0, ctx1)]
    call_bytes = algorithmic_bytes_per_call(shape, k, ctx_mid)
    n_calls = args.steps  # per kind
    draft_ms = st["draft_ms"] / n_calls
    verify_ms = st["verify_ms"] / n_calls
    step_gbs = call_bytes / ((draft_ms + verify_ms) / 2 * 1e-3) / 1e9

    # dominant kernel, timed live with HIP events on the library's stream
    g.set_option("kernel_timing", 1)
    g.run_iterations(slots, 4, temp, seed, top_k)
    kms, kn = g.kernel_time()
    g.set_option("kernel_timing", 0)
    k_avg_s = kms / max(kn, 1) * 1e-3
    k_bytes = gate_up_kernel_bytes(shape, M)
    achieved = k_bytes / k_avg_s / 1e9
    # yardstick: a kernel that only reads as many bytes of the model, launched back to back like the
    # kernel above (what streaming that many bytes once can at best take on this device)
    plain_bytes = k_bytes // 16 * 16
    g.plain_read(plain_bytes, 8)
    plain_us = g.plain_read(plain_bytes, 4 * shape.n_layers)

    # the same model call with no look-ahead rows (k = 0): the paper's premise is that the (1+k)-row
    # step costs about what the one-row step costs (Section 2.2)
    k0 = None
    if g0 is not None:
        g0.run_iterations(slots, max(2, args.warmup // 2), temp, seed, top_k)
        n0 = max(8, args.steps // 2)
        st0 = g0.run_iterations(slots, n0, temp, seed, top_k)
        k0_ms = (st0["draft_ms"] + st0["verify_ms"]) / (2 * n0)
        k0 = {"k0_call_ms": k0_ms, "ratio": (draft_ms + verify_ms) / 2 / k0_ms, "calls_timed": 2 * n0}
        g0.close()

    # Algorithm 1's loop through pass_generate, the entry point a caller uses: the workload end to end
    # (its prompts, max_new tokens per sequence), the prompt pass outside the timed region
    g.prefill_batch(list(range(len(prompts))), prompts)
    time.sleep(args.settle)
    g.generate(slots, 16, temp, seed, top_k)  # graphs of these lengths captured, caches warm
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    _toks, gst = g.generate(slots, w.max_new, temp, seed, top_k)
    torch.cuda.synchronize()
    gen_s = time.perf_counter() - t0
    gen = {"max_new": w.max_new, "ms": gen_s * 1e3, "tokens_per_s": w.max_new * w.batch / gen_s,
           "iterations": gst["iterations"], "ms_per_iteration": gen_s * 1e3 / max(1, gst["iterations"] // w.batch),
           "vs_run_iterations": (w.max_new * w.batch / gen_s) / (st["tokens_out"] / dt)}

    # prompt pass ("initial prompt sequence" of Algorithm 1), timed last: the same prompts into the
    # same slots again (the prefill call returns when the cache is filled).  Last, because a long
    # prompt pass keeps the matrix cores busy for hundreds of milliseconds and the chip then runs
    # the memory-bound decode calls 5-7 % slower for about a second.
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    g.prefill_batch(list(range(len(prompts))), prompts)
    torch.cuda.synchronize()
    prefill_s = time.perf_counter() - t0
    prompt_rows = sum(len(p) - 1 for p in prompts)

    out = {
        "metric": "generated tokens/s + (1+k)-token step HBM GB/s vs peak, 7B-shaped bf16, k=4",
        "value": st["tokens_out"] / dt,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if shape.dtype == 1 else "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "k": k, "batch": w.batch, "prompt_len": [len(p) for p in prompts],
                   "n_layers": shape.n_layers, "d_model": shape.d_model, "vocab": shape.vocab,
                   "temperature": temp, "top_k": top_k, "context_during_timing": [min(ctx0), max(ctx1)],
                   "graph": args.graph, "path": "generic" if args.path else "auto", "settle_s": args.settle},
        "draft_call_ms": draft_ms,
        "verify_call_ms": verify_ms,
        "acceptance_rate": st["drafts_accepted"] / max(1, st["drafts_proposed"]),
        "tokens_per_iteration": st["tokens_out"] / max(1, st["iterations"]),
        "step_hbm": {"algorithmic_bytes_per_call": call_bytes, "achieved_GBps": step_gbs,
                     "frac_of_peak": step_gbs / HBM_PEAK_GBS},
        "k_vs_k0": k0,
        "generate": gen,
        "prefill": prefill_report(shape, prompts, prompt_rows, prefill_s),
        "roofline": {"bound": "hbm", "kernel": "gate_up_gemm_silu", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(w.name) if not args.layers and k == w.k else None,
                     "bytes_per_launch": k_bytes, "avg_launch_us": k_avg_s * 1e6, "launches_timed": kn,
                     "plain_read_of_same_bytes_us": plain_us, "plain_read_GBps": plain_bytes / plain_us / 1e3},
    }
    g.close()
    if args.calibrate_copy:
        src = torch.ones(128 * 2 ** 20, dtype=torch.bfloat16, device="cuda")  # 256 MiB read, 256 MiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src * 1)  # elementwise kernel: reads 256 MiB, writes 256 MiB (then a copy of the same size)
        torch.cuda.synchronize()
    if args.train_steps > 0:
        try:  # a side figure: its failure must not take the line's main figures with it
            out["train"] = train_report(binding, devgen, synth, torch, np, args.train_steps, args.path)
        except Exception as e:  # noqa: BLE001
            out["train"] = {"error": repr(e)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, k, W_host, prompts[0])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
