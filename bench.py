#!/usr/bin/env python3
"""Benchmark of the blockwise-parallel-decoding step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Workload: Transformer-big, k = 10, bf16 (benchmark configs[2], batch 1: the paper decodes
single sentences) with an imposed acceptance schedule of mean 5 (the paper's trained k = 10
model reaches 4.95, Table 1); the batch-32 ragged workload (configs[3], mean 3) is measured in
the same run and reported under "batch32".  A "step" is one bpd_step: decoder forward over the
k proposed positions, k heads, vocabulary projection + argmax of the k x k outputs, verify /
accept / KV commit.  Inputs are seeded and synthetic (workloads.py) and already resident in
HBM when the timed region starts; encoder runs and the first invocation of each sentence are
outside the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published


def step_bytes(cfg) -> dict:
    """Algorithmic HBM bytes of one step at batch 1: every weight read once (bf16)."""
    d, F, V, k, nl = cfg.d_model, cfg.d_ff, cfg.vocab, cfg.k, cfg.n_dec
    return {
        "layers": nl * (6 * d * d + 2 * d * F) * 2,
        "head_hidden": k * d * F * 2,
        "head_out": k * F * d * 2,
        "vocab": V * d * 2,
    }


def step_flops(cfg, B: int, L_mean: float, S_mean: float) -> dict:
    d, F, V, k, nl = cfg.d_model, cfg.d_ff, cfg.vocab, cfg.k, cfg.n_dec
    M = B * k
    return {
        "layers": 2 * M * nl * (6 * d * d + 2 * d * F) + nl * B * 4 * k * d * (L_mean + k + S_mean),
        "head_hidden": 2 * M * d * k * F,
        "head_out": 2 * M * k * F * d,
        "vocab": 2 * M * k * V * d,
    }


def steps_needed(sched_col: np.ndarray, max_len: int) -> int:
    c = np.cumsum(sched_col)
    return int(np.argmax(c >= max_len)) + 1 if (c >= max_len).any() else len(sched_col)


def run_sessions(ctx, cfg, src, n, max_len, sched, k, total_steps, torch):
    """Time `total_steps` bpd_step calls spread over as many decode sessions as needed.
    Returns (seconds, accepted tokens, steps)."""
    B = src.shape[0]
    per_session = max(steps_needed(sched[:, b], int(max_len[b])) for b in range(B))
    sched_dev = torch.from_numpy(np.ascontiguousarray(sched[:per_session])).cuda()
    elapsed, accepted, done = 0.0, 0, 0
    while done < total_steps:
        ctx.bpd_encode(src, n, max_len)               # untimed: encoder + first invocation
        todo = min(per_session, total_steps - done)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(todo):
            ctx.bpd_step(k, sched_dev[s])
        torch.cuda.synchronize()
        elapsed += time.perf_counter() - t0
        accepted += int(ctx.bpd_get_stats().accepted_total)
        done += todo
    return elapsed, accepted, done


def profile_phase(ctx, phase, cfg, src, n, max_len, sched, k, steps, torch):
    ctx.bpd_profile_enable(phase)
    run_sessions(ctx, cfg, src, n, max_len, sched, k, steps, torch)
    ms, launches = ctx.bpd_profile_read()
    ctx.bpd_profile_enable(0)
    return ms / max(1, launches)


# mean accepted block size of the paper's best translation models (Table 1, column "Both") by k
PAPER_MEAN_BLOCK = {1: 1.0, 2: 1.88, 4: 3.27, 6: 4.18, 8: 4.69, 10: 4.95}


def k_sweep(ctx, cfg, src, n, max_len, torch, steps=100):
    """Step latency and accepted tokens/s by block size k on the headline workload, each k under an
    imposed schedule with the paper's mean accepted block size for that k (Section 7.4 plots
    wall-clock speedup against exactly this quantity); speedup is relative to k = 1 (greedy)."""
    res, base = {}, None
    for k in (1, 2, 4, 6, 8, 10):
        if k > cfg.k:
            continue
        mean = PAPER_MEAN_BLOCK[k]
        sched = wl.make_schedule(cfg, mean, cfg.max_out, k=k) if k > 1 else np.ones((cfg.max_out, src.shape[0]), np.int32)
        run_sessions(ctx, cfg, src, n, max_len, sched, k, 10, torch)
        sec, acc, st = run_sessions(ctx, cfg, src, n, max_len, sched, k, steps, torch)
        tps = acc / sec
        base = tps if base is None else base
        res[str(k)] = {"ms_per_step": 1e3 * sec / st, "mean_accepted": acc / st, "tokens_per_s": tps,
                       "speedup_vs_k1": tps / base}
    k1 = res["1"]["ms_per_step"]
    for v in res.values():
        v["step_cost_vs_k1"] = v["ms_per_step"] / k1
    return res


def other_configs(torch, binding, names=("C0", "C1", "C4", "C4L")):
    """bpd_step latency of the remaining workloads (parity-test configurations, reported for context):
    C0 and C1 over a decode session, C4 at three cache lengths (accepting one token per step so
    that the cache length stays put while timing), and C4L (C4 with 1D local self-attention in the decoder,
    Section 7.2) at the same lengths.  C4 is bound by the K/V cache it reads: each entry carries the step's algorithmic
    HBM bytes (weights once, the self-attention K/V rows of every sequence and layer up to the cache length, the
    cross-attention K/V) against the time of the whole step."""
    res = {}
    for name in names:
        cfg = wl.CONFIGS[name]
        ctx = binding.Context(binding.config_from_workload(cfg))
        ctx.bpd_load_weights(wl.make_weights(cfg))
        if cfg.local_q:
            ctx.bpd_set_local_attention(cfg.local_q, cfg.local_m)
        src, n = wl.make_sources(cfg)
        ml = wl.make_max_len(cfg, n)
        if name not in ("C4", "C4L"):
            mean = {"C0": 2, "C1": 4}[name]
            sched = wl.make_schedule(cfg, mean, cfg.max_out)
            run_sessions(ctx, cfg, src, n, ml, sched, cfg.k, 10, torch)
            sec, acc, st = run_sessions(ctx, cfg, src, n, ml, sched, cfg.k, 60, torch)
            res[name] = {"ms_per_step": 1e3 * sec / st, "tokens_per_s": acc / sec, "imposed_mean": mean, "batch": cfg.batch, "k": cfg.k}
        else:
            one = torch.ones((cfg.batch,), dtype=torch.int32, device="cuda")
            full = torch.full((cfg.batch,), cfg.k, dtype=torch.int32, device="cuda")
            ctx.bpd_encode(src, n, ml)
            L = 1
            for target in (256, 1536, 3000):
                while L < target - 10:
                    ctx.bpd_step(cfg.k, full)
                    L += cfg.k
                for _ in range(3):
                    ctx.bpd_step(cfg.k, one)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(20):
                    ctx.bpd_step(cfg.k, one)
                torch.cuda.synchronize()
                L += 23
                dt = time.perf_counter() - t0
                ms = 1e3 * dt / 20
                entry = {"ms_per_step": ms, "batch": cfg.batch, "k": cfg.k, "scored_positions_per_s": cfg.batch * cfg.k * 20 / dt}
                if name == "C4":
                    wbytes = sum(step_bytes(cfg).values())
                    kv = cfg.n_dec * 2 * cfg.batch * target * cfg.d_model * 2          # K and V rows 0..L of every layer and sequence
                    cross = cfg.n_dec * 2 * cfg.batch * int(n.mean()) * cfg.d_model * 2
                    total = wbytes + kv + cross
                    entry["roofline"] = {"bound": "hbm", "kernel": "whole step (self-attention over the cache dominates the bytes)",
                                         "bytes": {"weights": wbytes, "self_kv": kv, "cross_kv": cross},
                                         "achieved": total / (ms * 1e6), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                         "frac": total / (ms * 1e6) / HBM_PEAK_GBS}
                res[f"{name}@L{target}"] = entry
        ctx.close()
    return res


def cpu_baseline(cfg, weights, src, n, sched_col, tokens_target=128):
    """The oracle as it stands, on the host cores: blockwise decoding of the first
    `tokens_target` tokens of the batch-1 sentence under the same imposed schedule."""
    from oracle import CombinedModel, blockwise_decode, scorers
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    model = CombinedModel(weights, cfg.n_enc, cfg.n_dec, cfg.n_heads, cfg.k, cfg.ln_eps, cfg.local_q, cfg.local_m)
    score, block = scorers(model, src[0, :n[0]])
    t0 = time.perf_counter()
    dec = blockwise_decode(score, cfg.k, tokens_target, -1, schedule=list(sched_col), block_score=block)
    dt = time.perf_counter() - t0
    return {"value": len(dec.tokens) / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"oracle/ blockwise_decode (fp64 numpy, full recomputation per step) of the first "
                      f"{len(dec.tokens)} tokens of the batch-1 sentence, {len(dec.steps)} steps, same schedule",
            "ms_per_step": 1e3 * dt / max(1, len(dec.steps))}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-batch32", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true")
    ap.add_argument("--no-k-sweep", action="store_true")
    ap.add_argument("--no-peaks", action="store_true")
    ap.add_argument("--only", default=None,
                    help="comma-separated names among C0, C1, C4, C4L: time just these workloads and print their entries "
                         "(for profiler runs of one workload)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch a plain 256 MiB copy kernel a few times (reference for rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE scaling)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every box here has one); "
              "use --gpus 1.  The path shards by sequence (every GPU holds all weights and its slice of the batch).", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1811_03115_amd import binding

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)

    if args.copy_calibration:
        a = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")      # 256 MiB
        b = torch.empty_like(a)
        for _ in range(5):
            torch.mul(a, 1.0, out=b)          # one elementwise kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del a, b

    if args.only:
        print(json.dumps({"other_configs": other_configs(torch, binding, tuple(args.only.split(",")))}))
        return

    cfg1, cfg32 = wl.C2, wl.C3
    weights = wl.make_weights(cfg1)
    ctx = binding.Context(binding.config_from_workload(cfg32))
    ctx.bpd_load_weights(weights)
    k = cfg1.k

    # ---------------------------------------------------------------- batch 1 (headline)
    src, n = wl.make_sources(cfg1)
    max_len = wl.make_max_len(cfg1, n)
    sched = wl.make_schedule(cfg1, 5, cfg1.max_out)
    run_sessions(ctx, cfg1, src, n, max_len, sched, k, args.warmup, torch)
    sec, accepted, steps = run_sessions(ctx, cfg1, src, n, max_len, sched, k, args.steps, torch)
    ms_step = 1e3 * sec / steps
    nbytes = step_bytes(cfg1)
    total_bytes = sum(nbytes.values())
    kern = {}
    for name, phase in (("head_hidden", binding.PHASE_HEAD_HIDDEN), ("head_out", binding.PHASE_HEAD_OUT),
                        ("vocab", binding.PHASE_VOCAB), ("layers", binding.PHASE_LAYERS)):
        ms = profile_phase(ctx, phase, cfg1, src, n, max_len, sched, k, min(args.steps, 60), torch)
        kern[name] = {"ms": ms, "GBps": nbytes[name] / ms / 1e6}
    # what two events with nothing between them read on this stream: the part of every figure above that is the bracketing,
    # not the kernel (rocprofv3 reports kernel durations without it); `achieved` below keeps the raw event figure
    bracket_ms = profile_phase(ctx, binding.PHASE_EMPTY, cfg1, src, n, max_len, sched, k, min(args.steps, 60), torch)
    for name in ("head_hidden", "head_out", "vocab"):
        kern[name]["ms_minus_empty_bracket"] = kern[name]["ms"] - bracket_ms
    # the roofline entry is for the phase that takes most of the step: the decoder layers (42 kernels, each a small
    # weight stream), not for the best-behaved kernel; the three big single-kernel streams stay under "kernels"
    dom = max(("layers", "head_hidden", "head_out", "vocab"), key=lambda q: kern[q]["ms"])
    # HBM bytes per step of that phase measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of
    # known size), written by `python -m paper_1811_03115_amd.profsum` from the runs named in profiles/
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f).get("C2", {}).get(dom)
    # step latency distribution (HIP events around every bpd_step of a few sessions)
    ctx.bpd_profile_enable(binding.PHASE_STEP)
    run_sessions(ctx, cfg1, src, n, max_len, sched, k, min(args.steps, 200), torch)
    samples, _, _ = ctx.bpd_profile_samples(4096)
    ctx.bpd_profile_enable(0)
    lat = {"p50_ms": float(np.percentile(samples, 50)), "p95_ms": float(np.percentile(samples, 95)),
           "min_ms": float(samples.min()), "n": int(samples.size)}
    # end to end: one bpd_decode of the sentence (encoder, first invocation, all steps, host syncs)
    ctx.bpd_encode(src, n, max_len)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ctx.bpd_encode(src, n, max_len)
    ids_e2e, len_e2e, st_e2e = ctx.bpd_decode(k, sched)
    torch.cuda.synchronize()
    e2e = {"ms": 1e3 * (time.perf_counter() - t0), "tokens": int(len_e2e.sum()), "steps": int(st_e2e.steps)}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(5):
        ctx.bpd_encode(src, n, max_len)
    torch.cuda.synchronize()
    e2e["encode_ms"] = 1e3 * (time.perf_counter() - t0) / 5      # encoder + cross K/V + first invocation
    # the machine's own ceilings next to the published peaks
    peaks = None
    if not args.no_peaks:
        peaks = {"hbm_read_GBps": binding.Context.bpd_measure_hbm_read(1 << 30, 4),
                 "mfma_bf16_TFLOPs": binding.Context.bpd_measure_mfma_bf16(20000)}
    roofline = {"bound": "hbm", "kernel": dom if dom != "layers" else "layers (the 42 kernels of the 6 decoder layers)",
                "share_of_step": kern[dom]["ms"] / ms_step,
                "achieved": kern[dom]["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": kern[dom]["GBps"] / HBM_PEAK_GBS, "traffic": traffic,
                "frac_of_measured_peak": (kern[dom]["GBps"] / peaks["hbm_read_GBps"]) if peaks else None,
                "step_achieved": total_bytes / (ms_step * 1e6), "step_frac": total_bytes / (ms_step * 1e6) / HBM_PEAK_GBS,
                "kernels": kern, "empty_event_bracket_ms": bracket_ms}

    out = {
        "metric": "accepted tokens/s (bpd_step, Transformer-big k=10, batch 1)",
        "value": accepted / sec, "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "C2: Transformer-big 6+6 layers d=1024 F=4096 V=32768, k=10, batch 1, "
                               "imposed acceptance schedule mean 5", "batch": 1, "k": k,
                   "scored_positions_per_s": k / (ms_step * 1e-3), "mean_accepted": accepted / steps},
        "roofline": roofline,
        "step_latency": lat,
        "end_to_end_decode": e2e,
        "measured_peaks": peaks,
    }

    if not args.no_k_sweep:
        out["k_sweep"] = k_sweep(ctx, cfg1, src, n, max_len, torch)

    # ---------------------------------------------------------------- batch 32
    if not args.no_batch32:
        src32, n32 = wl.make_sources(cfg32)
        max32 = wl.make_max_len(cfg32, n32)
        sched32 = wl.make_schedule(cfg32, 3, cfg32.max_out)
        steps32 = max(20, args.steps // 4)
        run_sessions(ctx, cfg32, src32, n32, max32, sched32, k, max(4, args.warmup // 4), torch)
        sec32, acc32, st32 = run_sessions(ctx, cfg32, src32, n32, max32, sched32, k, steps32, torch)
        ms32 = 1e3 * sec32 / st32
        fl = step_flops(cfg32, cfg32.batch, 32.0, float(n32.mean()))
        vocab_ms = profile_phase(ctx, binding.PHASE_VOCAB, cfg32, src32, n32, max32, sched32, k, min(steps32, 30), torch)
        out["batch32"] = {
            "workload": "C3: same model, batch 32, ragged source lengths and budgets, imposed schedule mean 3",
            "value": acc32 / sec32, "unit": "tokens/s", "ms_per_step": ms32, "steps": st32,
            "scored_positions_per_s": cfg32.batch * k / (ms32 * 1e-3),
            "roofline": {"bound": "mfma", "kernel": "vocab", "achieved": fl["vocab"] / (vocab_ms * 1e9),
                         "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": fl["vocab"] / (vocab_ms * 1e9) / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                         "kernel_ms": vocab_ms,
                         "step_achieved": sum(fl.values()) / (ms32 * 1e9),
                         "step_frac": sum(fl.values()) / (ms32 * 1e9) / MFMA_BF16_PEAK_TFLOPS},
        }

        # the same workload with two-phase scoring (p_1 at all block rows, other heads at row k-hat only):
        # same tokens, 2k - 1 instead of k^2 vocabulary-projection rows per sequence
        ctx.bpd_set_two_phase(True)
        run_sessions(ctx, cfg32, src32, n32, max32, sched32, k, max(4, args.warmup // 4), torch)
        sec2, acc2, st2 = run_sessions(ctx, cfg32, src32, n32, max32, sched32, k, steps32, torch)
        ctx.bpd_set_two_phase(False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            ctx.bpd_encode(src32, n32, max32)
        torch.cuda.synchronize()
        out["batch32"]["encode_ms"] = 1e3 * (time.perf_counter() - t0) / 3
        out["batch32_two_phase"] = {"value": acc2 / sec2, "unit": "tokens/s", "ms_per_step": 1e3 * sec2 / st2, "steps": st2,
                                    "speedup_vs_full_table": (acc2 / sec2) / (acc32 / sec32)}

    if not args.no_other_configs:
        out["other_configs"] = other_configs(torch, binding)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg1, weights, src, n, sched[:, 0])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
