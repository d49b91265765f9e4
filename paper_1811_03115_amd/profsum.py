"""Summaries of rocprofv3 runs of bench.py: writes the text tables under profiles/ and profiles/traffic.json.

    python -m paper_1811_03115_amd.profsum --trace DIR --fetch DIR --write DIR [--sq DIR] [--c4-fetch DIR --c4-write DIR]

Each DIR is the `-d` output directory of one rocprofv3 run (a rocpd sqlite database somewhere below it).  The commands
that produce the runs are printed into the headers of the files written, so that every number can be reproduced from
committed files only.  Nothing here touches the GPU.
"""
from __future__ import annotations

import argparse
import glob
import json
import os
import sqlite3

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILES = os.path.join(ROOT, "profiles")

BENCH_TRACE = "python3 bench.py --steps 60 --warmup 10 --no-cpu-baseline --no-other-configs --no-k-sweep"
BENCH_PMC = "python3 bench.py --steps 30 --warmup 5 --no-cpu-baseline --no-batch32 --no-other-configs --no-k-sweep --no-peaks --copy-calibration"
BENCH_SQ = "python3 bench.py --steps 10 --warmup 3 --no-cpu-baseline --no-other-configs --no-k-sweep --no-peaks"
BENCH_C4 = "python3 bench.py --only C4 --copy-calibration"

# kernels of one C2 step (batch 1, 10 block rows) by phase: (substring of the kernel name, grid x, launches per step)
C2_STEP = {
    "layers": [("skinny_gemm_kernel<1, 1, true, false, 8, 4, 0, false>", 98304, 6),        # LayerNorm + QKV
               ("attention_mfma_kernel<false, false, 0>", 4096, 6),                       # self-attention
               ("skinny_gemm_kernel<1, 1, false, false, 4, 8, 0, false>", 16384, 12),      # attention output projections
               ("attention_mfma_kernel<false, false, 8>", 4096, 6),                       # LayerNorm + query projection + cross-attention
               ("skinny_gemm_kernel<1, 1, true, false, 8, 4, 0, false>", 131072, 6),       # LayerNorm + FFN in
               ("skinny_gemm_kernel<1, 1, false, false, 8, 16, 0, false>", 32768, 6)],     # FFN out
    "head_hidden": [("skinny_gemm_kernel<1, 2, true, false, 8, 4, 2, true>", 131072, 1)],
    "head_out": [("stream_gemm_kernel<16, true>", 12800, 1)],
    "vocab": [("stream_vocab_kernel<4, 1, 2, false>", 65536, 1)],
    "accept": [("accept_embed_kernel", 1024, 1)],
}
COPY_KERNEL = "vectorized_elementwise_kernel<4, at::native::AUnaryFunctor"     # torch.mul(a, 1.0, out=b): 256 MiB in, 256 MiB out
COPY_KIB = 262144.0
CLOCK_GHZ = 2.4        # the clock the published MFMA peak is quoted at
SIMDS = 1024           # 256 compute units x 4


def db_of(d):
    f = glob.glob(os.path.join(d, "**", "*.db"), recursive=True)
    if not f:
        raise SystemExit(f"no rocprofv3 database under {d}")
    return sqlite3.connect(f[0]).cursor()


def short(name, n):
    return name if len(name) <= n else name[:n - 3] + "..."


def trace_rows(cur):
    return cur.execute("select name, count(*), sum(end-start), avg(end-start), min(end-start), max(end-start), grid_x*1, workgroup_x "
                       "from kernels group by name, grid_x order by sum(end-start) desc").fetchall()


def trace_table(rows, top):
    tot = sum(r[2] for r in rows)
    out = [f"{'kernel':90s} {'calls':>6s} {'total_us':>10s} {'avg_us':>9s} {'min_us':>8s} {'max_us':>8s} {'pct':>6s} grid"]
    for r in rows[:top]:
        out.append(f"{short(r[0], 90):90s} {r[1]:6d} {r[2]/1e3:10.1f} {r[3]/1e3:9.2f} {r[4]/1e3:8.2f} {r[5]/1e3:8.2f} {100*r[2]/tot:6.2f} {r[6]}x{r[7]}")
    return "\n".join(out)


def pmc_rows(cur):
    return cur.execute("select kernel_name, grid_size_x, counter_name, count(*), avg(value), min(value), max(value), avg(end-start) "
                       "from counters_collection group by kernel_name, grid_size_x, counter_name order by avg(value)*count(*) desc").fetchall()


def pmc_table(rows, top):
    out = [f"{'kernel':80s} {'grid':>8s} {'counter':>11s} {'n':>5s} {'avg_KiB':>12s} {'min':>10s} {'max':>10s}"]
    for r in rows[:top]:
        out.append(f"{short(r[0], 80):80s} {r[1]:8d} {r[2]:>11s} {r[3]:5d} {r[4]:12.1f} {r[5]:10.1f} {r[6]:10.1f}")
    return "\n".join(out)


def avg_of(rows, sub, grid=None, col=4):
    m = [r for r in rows if sub in r[0] and (grid is None or r[1] == grid)]
    return sum(r[col] * r[3] for r in m) / max(1, sum(r[3] for r in m)) if m else 0.0


def phase_sum(rows, phase, col=4):
    """Per step: sum over the phase's kernels of (average per dispatch) x (launches per step)."""
    return sum(avg_of(rows, sub, grid, col) * n for sub, grid, n in C2_STEP[phase])


def write(name, text):
    os.makedirs(PROFILES, exist_ok=True)
    with open(os.path.join(PROFILES, name), "w") as f:
        f.write(text)
    print("wrote profiles/" + name)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--trace")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--sq")
    ap.add_argument("--c4-fetch")
    ap.add_argument("--c4-write")
    args = ap.parse_args()
    traffic = {}
    tpath = os.path.join(PROFILES, "traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f)

    if args.trace:
        rows = trace_rows(db_of(args.trace))
        def kavg(sub, grid):          # average duration (ns) over the dispatches of that kernel and grid
            m = [r for r in rows if sub in r[0] and r[6] == grid]
            return sum(r[2] for r in m) / max(1, sum(r[1] for r in m))
        per_step = {ph: sum(kavg(sub, grid) * n for sub, grid, n in ks) / 1e3 for ph, ks in C2_STEP.items()}
        hdr = [
            "# rocprofv3 kernel trace of bench.py (C2 batch-1 run and its per-phase timing passes, then the C3 batch-32 run in both",
            "# scoring modes; encoder runs and weight loading included)",
            f"# command: rocprofv3 --kernel-trace --stats -d prof_out/prof_trace -o bench -- {BENCH_TRACE}",
            "# summarised by: python -m paper_1811_03115_amd.profsum --trace prof_out/prof_trace",
            "# durations in microseconds, grouped by kernel and grid (grid = threads in x)",
            "# C2 step (batch 1, 10 block rows), average kernel durations x launches per step:",
        ] + [f"#   {ph:12s} {us:8.2f} us" for ph, us in per_step.items()] + [
            f"#   whole step   {sum(per_step.values()):8.2f} us (sum of kernel durations)",
            "# C2 kernels: skinny_gemm_kernel<1,..> = layer GEMMs and the heads' hidden layers (XLN variants apply LayerNorm from",
            "#   the partial statistics), stream_gemm_kernel<16,true> = heads' output layers, attention_mfma_kernel<..,0> self-attention,",
            "#   <..,8> cross-attention with its query projection, stream_vocab_kernel = vocabulary projection + arg-max (100 rows)",
            "# C3 step (batch 32, 320 block rows): gemm_ldsx_kernel<8,4,64,true,..> = vocabulary projection + arg-max (3200 rows),",
            "#   <7,4,64,false,..> = heads' hidden layers, <4,2,128,false> = heads' output layers (10 groups), <3,1,256> / <2,1,256> /",
            "#   <1,1,256> = layer GEMMs (the 4096-deep FFN output split 4 ways over K, summed by layernorm_kernel); two-phase mode adds",
            "#   gemm_ldsx_kernel<5,4,64,true> (320 and 288 rows), select_row_kernel, assemble_keys_kernel",
        ]
        write("bench_c2_c3_kernel_trace.txt", "\n".join(hdr) + "\n" + trace_table(rows, 48) + "\n")
        traffic.setdefault("C2", {})["kernel_us_per_step"] = per_step

    if args.fetch and args.write:
        fetch, wr = pmc_rows(db_of(args.fetch)), pmc_rows(db_of(args.write))
        copy_f, copy_w = avg_of(fetch, COPY_KERNEL), avg_of(wr, COPY_KERNEL)
        fs, ws = COPY_KIB / copy_f, COPY_KIB / copy_w
        c2 = {ph: int(1024 * (fs * phase_sum(fetch, ph) + ws * phase_sum(wr, ph))) for ph in ("layers", "head_hidden", "head_out", "vocab")}
        traffic.setdefault("C2", {}).update(c2)
        traffic["C2"]["fetch_scale"], traffic["C2"]["write_scale"] = fs, ws
        alg = {"layers": 176.2, "head_hidden": 83.9, "head_out": 83.9, "vocab": 67.1}
        hdr = [
            "# rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE (KiB per dispatch) for the kernels of the C2 batch-1 step",
            "# commands (one counter per run):",
            f"#   rocprofv3 --pmc FETCH_SIZE -d prof_out/pmc_fetch -o c2 -- {BENCH_PMC}",
            f"#   rocprofv3 --pmc WRITE_SIZE -d prof_out/pmc_write -o c2 -- {BENCH_PMC}",
            "#   python -m paper_1811_03115_amd.profsum --fetch prof_out/pmc_fetch --write prof_out/pmc_write",
            f"# calibration: the 256 MiB elementwise copy kernel (reads 262144 KiB, writes 262144 KiB) shows FETCH_SIZE {copy_f:.0f} and",
            f"# WRITE_SIZE {copy_w:.0f}, so FETCH_SIZE is scaled by {fs:.2f} and WRITE_SIZE by {ws:.2f} to get bytes.",
            "# per step (bytes = 1024 * (fetch scale * FETCH_SIZE + write scale * WRITE_SIZE), summed over the phase's launches),",
            "# against the algorithmic bytes (weights read once):",
        ] + [f"#   {ph:12s} {c2[ph] / 1e6:8.1f} MB measured, {alg[ph]:6.1f} MB algorithmic" for ph in c2] + [
            "# (FETCH_SIZE counts what the L2s request from the fabric: it sits in front of the Infinity Cache and cannot tell its hits",
            "#  from HBM reads.  The decoder layers' 42 kernels each fetch their activations once per XCD on top of the weights.)",
        ]
        write("c2_step_hbm_traffic_pmc.txt", "\n".join(hdr) + "\n\n" + pmc_table(fetch, 14) + "\n\n" + pmc_table(wr, 12) + "\n")

    if args.c4_fetch and args.c4_write:
        fetch, wr = pmc_rows(db_of(args.c4_fetch)), pmc_rows(db_of(args.c4_write))
        copy_f, copy_w = avg_of(fetch, COPY_KERNEL), avg_of(wr, COPY_KERNEL)
        fs, ws = COPY_KIB / copy_f, COPY_KIB / copy_w
        att = [r for r in fetch if "attention_mfma_kernel<true" in r[0]]
        # the dispatches with the longest cache (largest fetch): bytes and duration of the attention launch alone
        cur = db_of(args.c4_fetch)
        top = cur.execute("select value, end-start from counters_collection where kernel_name like '%attention_mfma_kernel<true%' "
                          "and counter_name = 'FETCH_SIZE' order by value desc limit 120").fetchall()
        hdr = [
            "# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE for the super-resolution workload C4 (batch 8, k = 10, 6 layers, d = 512):",
            "# bpd_step at cache lengths 256, 1536 and 3000 (bench.py --only C4 steps the decode to each length, then times 20 steps",
            "# that accept one token each)",
            f"#   rocprofv3 --pmc FETCH_SIZE -d prof_out/pmc_c4_fetch -o c4 -- {BENCH_C4}",
            f"#   rocprofv3 --pmc WRITE_SIZE -d prof_out/pmc_c4_write -o c4 -- {BENCH_C4}",
            "#   python -m paper_1811_03115_amd.profsum --c4-fetch prof_out/pmc_c4_fetch --c4-write prof_out/pmc_c4_write",
            f"# copy kernel: FETCH_SIZE {copy_f:.0f}, WRITE_SIZE {copy_w:.0f} for 262144 KiB each way: scales {fs:.2f} / {ws:.2f}",
            "# self-attention over the cache = attention_mfma_kernel<true, *, 0> (K/V fetched with non-temporal loads: the 303 MB of",
            "# caches would evict the weights from the Infinity Cache), its split-KV merge = attention_combine_kernel.",
            "# Algorithmic K/V bytes of one self-attention launch at cache length L: 2 * 8 sequences * L * 512 * 2 B = 16384 L",
            "# (the average below mixes all lengths the decode passes through; min / max are the ends).",
        ]
        for r in att:
            hdr.append(f"#   {short(r[0], 60)} grid {r[1]}: avg {1024 * fs * r[4] / 1e6:.1f} MB, max {1024 * fs * r[6] / 1e6:.1f} MB per launch "
                       f"(max: L = 3000+, algorithmic 49.5 MB), avg duration {r[7] / 1e3:.1f} us")
        if top:
            tb = 1024 * fs * sum(t[0] for t in top) / len(top)
            tus = sum(t[1] for t in top) / len(top) / 1e3
            hdr.append(f"#   the {len(top)} launches with the longest cache: {tb / 1e6:.1f} MB fetched in {tus:.1f} us per launch = {tb / tus / 1e3:.0f} GB/s "
                       f"({tb / tus / 1e3 / 8000:.2f} of 8 TB/s) for the attention launch alone (profiled run)")
            traffic["C4"] = {"attention_fetch_bytes_longest": int(tb), "attention_us_longest": tus, "attention_GBps_longest": tb / tus / 1e3,
                             "fetch_scale": fs}
        write("c4_attention_hbm_traffic_pmc.txt", "\n".join(hdr) + "\n\n" + pmc_table(fetch, 14) + "\n\n" + pmc_table(wr, 8) + "\n")

    if args.sq:
        cur = db_of(args.sq)
        rows = cur.execute("select kernel_name, grid_size_x, counter_name, count(*), avg(value), avg(end-start) from counters_collection "
                           "group by kernel_name, grid_size_x, counter_name").fetchall()
        d, n, dur = {}, {}, {}
        for k, g, c, cnt, v, t in rows:
            d.setdefault((k, g), {})[c] = v
            n[(k, g)] = cnt
            dur[(k, g)] = t
        names = ["SQ_WAVE_CYCLES", "SQ_BUSY_CYCLES", "SQ_WAIT_ANY", "SQ_WAIT_INST_ANY", "SQ_WAIT_INST_LDS", "SQ_ACTIVE_INST_LDS",
                 "SQ_ACTIVE_INST_VMEM", "SQ_VALU_MFMA_BUSY_CYCLES"]
        hdr = [
            "# rocprofv3 SQ counters per dispatch (averages) of the bench workloads: C2 step (batch 1) and C3 step (batch 32)",
            "# command: rocprofv3 --pmc " + " ".join(names) + f" -d prof_out/pmc_sq -o b -- {BENCH_SQ}",
            "# summarised by: python -m paper_1811_03115_amd.profsum --sq prof_out/pmc_sq",
            "# mfma_util = SQ_VALU_MFMA_BUSY_CYCLES / (kernel duration x 2.4 GHz x 1024 SIMDs): the share of the chip's matrix-pipe cycles",
            "# in use (the counter adds, over all SIMDs, the cycles an MFMA occupies its pipe: 16 per v_mfma_f32_16x16x32_bf16, which at",
            "# 16384 flop each is the published 2.5 PFLOP/s when every SIMD issues back to back; padded rows count as work here).",
            "# wait_inst = SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES: share of wave time spent waiting on an instruction's operands (memory, LDS).",
            "# The batch-32 (C3) GEMMs are the gemm_ldsx_kernel rows: <8,4,64,true> is the vocabulary projection + arg-max (3200 rows).",
        ]
        out = [f"{'kernel':74s} {'grid':>8s} {'n':>4s} {'dur_us':>8s} {'mfma_util':>9s} {'wait_inst':>9s} " + " ".join(f"{x[3:]:>18s}" for x in names)]
        keys = sorted(d, key=lambda x: -dur[x] * n[x])
        mf = {}
        for k in keys[:30]:
            c = d[k]
            util = c.get("SQ_VALU_MFMA_BUSY_CYCLES", 0) / max(1.0, dur[k] * CLOCK_GHZ * SIMDS)
            wi = c.get("SQ_WAIT_INST_ANY", 0) / max(1.0, c.get("SQ_WAVE_CYCLES", 1))
            mf[k] = util
            out.append(f"{short(k[0], 74):74s} {k[1]:8d} {n[k]:4d} {dur[k]/1e3:8.2f} {util:9.3f} {wi:9.3f} " + " ".join(f"{c.get(x, 0):18.0f}" for x in names))
        write("c2_c3_kernels_sq_counters_pmc.txt", "\n".join(hdr) + "\n" + "\n".join(out) + "\n")
        v = [u for k, u in mf.items() if "gemm_ldsx_kernel<8, 4, 64, true" in k[0]]
        if v:
            traffic.setdefault("C3", {})["vocab_mfma_util"] = v[0]

    with open(tpath, "w") as f:
        json.dump(traffic, f, indent=1, sort_keys=True)
    print("wrote profiles/traffic.json")


if __name__ == "__main__":
    main()
