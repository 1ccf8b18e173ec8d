#!/usr/bin/env python3
"""Benchmark of the all-gather -> GEMM pair on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input: plan (built once),
the piece transfers, the ready flags / signals and the piece GEMMs. In the all-gather direction the K
timed steps are taken in turn by two plans chained behind each other (ficco_plan_chain): a step's
transfers start on the device when the previous step's kernel has finished, the host never blocks
between steps, and both sides of the K steps are synchronised (the figure with a blocking statistics
query after every step is reported beside it). Prints ONE JSON line. Only one GPU is used; --gpus > 1
exits.

Legs (all on the same workload, default the 70B-class FFN-up share at TP=8, M=16384 K=8192 N=3584, the largest
all-gather configuration one GPU holds):
  pair      - K timed steps of the schedule the library itself picks (FICCO_AUTO_ANY) from the caller's
              row-major shards resident in HBM (device staging buffer): that is `value`. Beside it a screen of
              the other schedules and piece counts, and the serial and shard-level schedules for the speedups
  power     - (not run by default) board power and TFLOP/s of the timed plan's GEMM on the workload's data and on
              zeros, with the vendor library's GEMM beside it
  contend   - (for counter runs) the plan's GEMM with its transfers beside it, no dependency between them
  small     - the pair and pcie legs of the two smaller all-gather workloads (cfg1, cfg2), condensed
  pcie      - the same with the shards in pinned host memory (PCIe-inclusive; never `value`)
  roofline  - the GEMM launches of the timed plan in isolation, enqueued back to back between two
              HIP events on the compute stream -> achieved TFLOP/s against the bf16 dense MFMA peak
  losses    - decomposition / contention losses (DIL, CIL) through ficco_profile_losses
  cpu       - the CPU oracle timed on the host cores (a baseline, not a target)
  graph     - (not run by default) HIP-graph replays against call-by-call enqueue, stream backend
  reduce    - (not run by default) receiver side of the reduce-scatter on the workload's output block:
              serial / shard-level / finer-grain step times and the add kernel against the HBM roofline
              (reduce_kernel: the kernel part only, for profiling)
  calib     - (not in the default set) a plain device copy of 256 MiB, so that HBM counters read
              under rocprofv3 --pmc can be scaled by what they show for a known amount of traffic
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

MFMA_BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16
HBM_PEAK_GBPS = 8000.0

# HBM-side traffic per launch of the roofline kernel, from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# summaries kept under profiles/ (gemm_isolated_<workload>.md): KiB per dispatch as the counters
# read, and the factors by which a 256 MiB device copy's true traffic exceeds what they read for it.
PMC_SCALE = {"FETCH_SIZE": 262144.0 / 131086.7, "WRITE_SIZE": 262144.0 / 262144.0}
PMC_KIB = {
    ("cfg2_qkv8b", "gemm_resident_kernel<128x192>"): {"FETCH_SIZE": 57491.0, "WRITE_SIZE": 12288.0},
    ("cfg2_qkv8b", "gemm_blocks_kernel<128x192>"): {"FETCH_SIZE": 57458.0, "WRITE_SIZE": 12288.0},
    ("cfg3_ffn70b", "gemm_resident_kernel<256x256>"): {"FETCH_SIZE": 908479.1, "WRITE_SIZE": 115327.7},
    ("cfg3_ffn70b", "gemm_blocks_kernel<256x256>"): {"FETCH_SIZE": 825994.4, "WRITE_SIZE": 115201.6},
    ("cfg6_2d_proj", "gemm_resident2d_kernel<256x256>"): {"FETCH_SIZE": 394542.8, "WRITE_SIZE": 33777.8},
    ("cfg6_2d_proj", "gemm_blocks_kernel<256x256>"): {"FETCH_SIZE": 395433.1, "WRITE_SIZE": 33006.5},
    ("cfg4_gemm_rs", "rs_reduce_kernel"): {"FETCH_SIZE": 131151.5, "WRITE_SIZE": 32768.0},      # profiles/rs_reduce_cfg4_gemm_rs.md
}


def bench_grouped(args, cfg, legs, torch, np, fi, F, dev) -> int:
    """Expert-parallel workload: unequal token counts from G peers to E local experts, dispatch over the
    copy engines, one resident grouped kernel. Same JSON contract; legs pair, roofline, cpu."""
    K, N, G, E = cfg["K"], cfg["N"], cfg["shards"], cfg["experts"]
    rows = fi.make_token_counts(cfg["seed"], G, E, cfg["tokens"], cfg["skew"])
    M = int(rows.sum())
    en = rows.sum(axis=0)
    A = fi.normal_bf16(cfg["seed"], fi.TENSOR_A, M, K)
    W = np.stack([fi.normal_bf16(cfg["seed"] + 100 + e, fi.TENSOR_W, K, N, float(K) ** -0.5) for e in range(E)])
    A_stage = torch.from_numpy(A.view(np.int16)).to(dev)
    A_dev = torch.zeros((M, K), dtype=torch.int16, device=dev)
    W_dev = torch.from_numpy(W.view(np.int16)).to(dev)
    C_dev = torch.zeros((M, N), dtype=torch.int16, device=dev)
    cs, xs = torch.cuda.Stream(), torch.cuda.Stream()
    flops = 2 * M * N * K

    def make(sched, c, opts=()):
        plan = F.ficco_plan_grouped(K, N, rows.tolist(), c, sched)
        for o, v in opts:
            F.ficco_plan_set(plan, o, v)
        F.ficco_pack_weight(plan, W_dev, cs)
        return plan

    def timed(plan, steps, warmup):
        for _ in range(warmup):
            F.ficco_run(plan, A_stage, A_dev, W_dev, C_dev, None, cs, xs)
            F.ficco_query_stats(plan)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            F.ficco_run(plan, A_stage, A_dev, W_dev, C_dev, None, cs, xs)
            st = F.ficco_query_stats(plan)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps, st

    def timed_chained(sched, c, steps, warmup):
        """ms per step with two plans chained behind each other taking the steps in turn (no host wait between
        steps; synchronize on both sides)."""
        pa, pb = make(sched, c), make(sched, c)
        try:
            F.ficco_plan_chain(pa, pb)
            F.ficco_plan_chain(pb, pa)
            turn = [pa, pb]
            for i in range(warmup + warmup % 2):
                F.ficco_run(turn[i % 2], A_stage, A_dev, W_dev, C_dev, None, cs, xs)
            F.ficco_query_stats(pa), F.ficco_query_stats(pb)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(steps):
                F.ficco_run(turn[i % 2], A_stage, A_dev, W_dev, C_dev, None, cs, xs)
            F.ficco_query_stats(pa), F.ficco_query_stats(pb)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / steps
        finally:
            F.ficco_destroy(pa)
            F.ficco_destroy(pb)

    out = {"metric": "EP dispatch + grouped expert GEMM effective TFLOP/s (overlapped pair, best finer-grain schedule)",
           "value": None, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": None,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": args.workload, "tokens": M, "K": K, "N": N, "peers": G, "experts": E,
                      "tokens_per_peer_min_max": [int(rows.sum(axis=1).min()), int(rows.sum(axis=1).max())],
                      "source": "device staging buffer (HBM-resident), one SDMA engine per peer as its link"}}
    best = (F.FICCO_FINE_PERSISTENT, cfg["pieces"][0])
    if "pair" in legs:
        res = {}
        p_warm = make(F.FICCO_SERIAL, 1)             # bring the clocks up before the first (serial) case is timed
        t_warm = time.perf_counter()
        while time.perf_counter() - t_warm < 0.05:
            F.ficco_run(p_warm, A_stage, A_dev, W_dev, C_dev, None, cs, xs)
            F.ficco_query_stats(p_warm)
        F.ficco_destroy(p_warm)
        for name, sched, c in [("serial", F.FICCO_SERIAL, 1), ("shard_level", F.FICCO_SHARD, 1)] + \
                              [(f"fine:{c}", F.FICCO_FINE_PERSISTENT, c) for c in cfg["pieces"]]:
            plan = make(sched, c)
            ms, st = timed(plan, args.steps, args.warmup)
            info = F.ficco_plan_info(plan)
            F.ficco_destroy(plan)
            res[name] = round(ms, 4)
        bname = min((k for k in res if k.startswith("fine")), key=res.get)
        best = (F.FICCO_FINE_PERSISTENT, int(bname.split(":")[1]))
        # the figures that count: steps back to back through two chained plans (the table above, with a blocking
        # query after every step, ranks the piece counts and stays in the output)
        chained = {"serial": round(timed_chained(F.FICCO_SERIAL, 1, args.steps, args.warmup), 4),
                   "shard_level": round(timed_chained(F.FICCO_SHARD, 1, args.steps, args.warmup), 4),
                   bname: round(timed_chained(best[0], best[1], args.steps, args.warmup), 4)}
        out["value"] = round(flops / chained[bname] * 1e-9, 3)
        out["ms_per_step"] = chained[bname]
        out["pair"] = {"ms_per_step": chained, "ms_per_step_host_synced": res, "best": bname, "tile": f"{info.tile_m}x{info.tile_n}",
                       "stepping": "two plans chained behind each other take the steps in turn; the host runs one step ahead",
                       "speedup_vs_serial": round(chained["serial"] / chained[bname], 4),
                       "speedup_vs_shard_level": round(chained["shard_level"] / chained[bname], 4), "copy_backend": "engines", "links": info.links}
    if "roofline" in legs:
        plan = make(best[0], best[1], [(F.FICCO_OPT_MODE, F.FICCO_MODE_GEMM_ONLY)])
        spans = []
        for it in range(args.warmup + args.steps):
            F.ficco_run(plan, None, A_stage, W_dev, C_dev, None, cs, xs)
            st = F.ficco_query_stats(plan)
            if it >= args.warmup:
                spans.append(st.wall_us)
        info = F.ficco_plan_info(plan)
        F.ficco_destroy(plan)
        us = float(np.mean(spans))              # HIP events on the compute stream around the one launch of a run
        out["roofline"] = {"bound": "mfma", "achieved": round(flops / us * 1e-6, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                           "frac": round(flops / us * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                           "algorithmic_bytes": 2 * (M * K + E * K * N + M * N), "kernel": f"gemm_grouped_kernel<{info.tile_m}x{info.tile_n}>",
                           "launches_per_step": 1, "avg_launch_us": round(us, 3), "flops_per_launch": flops}
    if "cpu" in legs:
        from oracle import gemm as og
        rng = np.random.default_rng(0)
        sample = np.sort(rng.choice(M, size=min(M, 4096), replace=False)).astype(np.int64)
        expert_of = np.repeat(np.arange(E), en)
        t0 = time.perf_counter()
        ref = np.empty((sample.size, N))
        for e in range(E):
            sel = sample[expert_of[sample] == e]
            if sel.size:
                ref[expert_of[sample] == e] = og.ag_gemm_rows([A], W[e], sel)
        dt = time.perf_counter() - t0
        got = C_dev.cpu().numpy().view(np.uint16)[sample]
        err = og.rel_err(fi.bf16_bits_to_f32(got).astype(np.float64), ref) if ("pair" in legs or "roofline" in legs) else None
        out["cpu_baseline"] = {"value": round(2 * sample.size * N * K / dt * 1e-12, 6), "unit": "TFLOP/s", "cores": og.num_threads(),
                               "kind": "oracle", "sample": f"{sample.size} random token rows, all {N} columns, {dt:.1f} s",
                               "gpu_vs_oracle_rel_err": err}
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg3_ffn70b")
    ap.add_argument("--legs", default="pair,pcie,roofline,losses,small,cpu")
    ap.add_argument("--candidates", default="", help="schedule:chunks list, e.g. 3:2,4:4,5:3072+1024 (default: a small sweep)")
    ap.add_argument("--backend", default="auto", choices=["auto", "stream", "engines"],
                    help="transfer backend for every plan (default: the library's choice)")
    ap.add_argument("--plan-opts", default="", help="measuring aid: option:value pairs (ficco_option numbers) set on every plan, e.g. 13:4,14:2")
    ap.add_argument("--roofline-plan", default="", help="schedule:chunks (or schedule:w1+w2+... for column pieces of those widths) for the roofline leg when the pair leg is not run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every box here has one); "
              "run with --gpus 1 (across GPUs every GPU computes its own column share and only the gather of "
              "A is exchanged, one copy engine per peer link).", file=sys.stderr)
        return 2
    legs = set(args.legs.split(","))

    import numpy as np
    import torch

    import ficco_inputs as fi
    import paper_2512_10236_amd as F

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    F.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = fi.CONFIGS[args.workload]
    if cfg["direction"] == "ep_grouped":
        return bench_grouped(args, cfg, legs, torch, np, fi, F, dev)
    M, K, N, G = cfg["M"], cfg["K"], cfg["N"], cfg["shards"]
    shards, W = fi.config_inputs(args.workload)
    A_host = torch.from_numpy(np.concatenate(shards, 0).view(np.int16))
    A_pinned = A_host.pin_memory()
    A_stage = A_host.to(dev)                              # device staging buffer ("peers' memory")
    W_dev = torch.from_numpy(W.view(np.int16)).to(dev)
    A_dev = torch.zeros((M, K), dtype=torch.int16, device=dev)
    C_dev = torch.zeros((M, N), dtype=torch.int16, device=dev)
    cs, xs = torch.cuda.Stream(), torch.cuda.Stream()
    flops = 2 * M * N * K
    ms_shard = M // G

    rs = cfg["direction"] == "gemm_rs"
    if rs:
        # GEMM -> reduce-scatter (data movement): A is resident, row block p of C goes to peer buffer p
        A_dev.copy_(A_stage)
        peers_dev = [torch.zeros((ms_shard, N), dtype=torch.int16, device=dev) for _ in range(G)]
        peers_pin = [torch.zeros((ms_shard, N), dtype=torch.int16).pin_memory() for _ in range(G)]
        torch.cuda.synchronize()

    sliced = {}

    def source(tag, sched, c, layout="rm"):
        """Shard source for a plan: the row-major staging buffer (the caller's layout, also for column pieces),
        or its K-sliced copy (same bytes) for column pieces whose sender holds them that way (layout "ks").
        `tag` is "hbm" or "pcie"."""
        if rs:
            return peers_dev if tag == "hbm" else peers_pin
        base = A_stage if tag == "hbm" else A_pinned
        if sched != F.FICCO_FINE_2D or layout != "ks":
            return base
        if (tag, c) not in sliced:
            if isinstance(c, tuple):                      # slices of unequal width, block after block
                edges = [sum(c[:i]) for i in range(len(c) + 1)]
                t = torch.cat([base[:, edges[i]:edges[i + 1]].reshape(-1) for i in range(len(c))]).view(M, K)
            else:
                t = base.view(M, c, K // c).permute(1, 0, 2).contiguous().view(M, K)
            sliced[(tag, c)] = t if tag == "hbm" else t.pin_memory()
            torch.cuda.synchronize()
        return sliced[(tag, c)]

    def run_once(plan, src):
        """One step. `src` is the shard source (all-gather direction) or the peer list (reduce-scatter)."""
        if rs:
            F.ficco_run(plan, None, A_dev, W_dev, C_dev, src, cs, xs)
        else:
            F.ficco_run(plan, src, A_dev, W_dev, C_dev, None, cs, xs)
        return F.ficco_query_stats(plan)                  # the step's last stage; blocks until the step is done

    def timed_steps(plan, src, steps, warmup, warm_seconds=0.0):
        """ms per step over `steps` back-to-back steps, synchronize on both sides. `warm_seconds`: keep
        warming up (untimed) until that much time has passed."""
        t_warm = time.perf_counter()
        for _ in range(warmup):
            run_once(plan, src)
        while time.perf_counter() - t_warm < warm_seconds:
            run_once(plan, src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run_once(plan, src)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    def timed_steps_chained(sc, src, steps, warmup, opts=()):
        """ms per step when the host does not wait between steps: two plans of the same kind, chained behind
        each other (ficco_plan_chain), take the steps in turn on the same buffers; the transfers of a step
        start on the device when the previous step's kernel has finished, and the host only ever waits for
        the step before the previous one. Synchronize on both sides of the timed steps."""
        pa, pb = make(*sc, opts=opts), make(*sc, opts=opts)
        try:
            F.ficco_plan_chain(pa, pb)
            F.ficco_plan_chain(pb, pa)
            turn = [pa, pb]
            for i in range(warmup + warmup % 2):
                F.ficco_run(turn[i % 2], src, A_dev, W_dev, C_dev, None, cs, xs)
            F.ficco_query_stats(pa), F.ficco_query_stats(pb)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(steps):
                F.ficco_run(turn[i % 2], src, A_dev, W_dev, C_dev, None, cs, xs)
            F.ficco_query_stats(pa), F.ficco_query_stats(pb)       # the last two steps' last stage
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / steps
        finally:
            F.ficco_destroy(pa)
            F.ficco_destroy(pb)

    def sched_name(sched):
        return F.SCHEDULE_NAMES[sched % PACKED] + ("+gather_scatter" if sched >= PACKED else "")

    def make(sched, c, layout="rm", opts=()):
        if sched >= PACKED:
            sched, opts = sched - PACKED, list(opts) + [(F.FICCO_OPT_PACKING, 1)]
        plan = F.ficco_plan(M, K, N, G, len(c) if isinstance(c, tuple) else c, sched)
        if isinstance(c, tuple):
            F.ficco_plan_set_slice_widths(plan, c)
        if sched == F.FICCO_FINE_2D and layout == "ks":
            F.ficco_plan_set(plan, F.FICCO_OPT_SOURCE_LAYOUT, F.FICCO_LAYOUT_K_SLICED)
        if rs:
            F.ficco_plan_set(plan, F.FICCO_OPT_DIRECTION, F.FICCO_DIR_GEMM_RS)
        for o, v in opts:
            F.ficco_plan_set(plan, o, v)
        for pair in filter(None, args.plan_opts.split(",")):
            o, v = pair.split(":")
            F.ficco_plan_set(plan, int(o), int(v))
        if args.backend != "auto":
            F.ficco_plan_set(plan, F.FICCO_OPT_COPY_BACKEND, {"stream": F.FICCO_COPY_STREAM, "engines": F.FICCO_COPY_ENGINES}[args.backend])
        F.ficco_pack_weight(plan, W_dev, cs)
        return plan

    # a candidate is (schedule, pieces per shard, source layout); the fused schedule with explicit Gather/Scatter
    # copies ("3p:4" on the command line) is schedule FICCO_FINE_FUSED + PACKED; column pieces of unequal width
    # ("5:3072+1024") carry the tuple of widths in place of the count; column pieces leave the caller's row-major
    # matrix (layout "rm": the step pays for the sender-side re-layout) unless the candidate says the sender
    # holds them K-sliced ("5k:2", layout "ks")
    PACKED = 1000
    def pieces_of(c):
        return len(c) if isinstance(c, tuple) else c
    def label(sc):
        return f"{sched_name(sc[0])}" + ("_presliced" if sc[2] == "ks" else "") + ":" + \
            ("+".join(str(w) for w in sc[1]) if isinstance(sc[1], tuple) else str(sc[1]))
    def parse_plan(t):
        a, b = t.split(":")
        b = tuple(int(w) for w in b.split("+")) if "+" in b else int(b)
        if a.endswith("p"):
            return (int(a[:-1]) + PACKED, b, "rm")
        if a.endswith("k"):
            return (int(a[:-1]), b, "ks")
        return (int(a), b, "rm")
    def library_pick(host_resident=False):
        """What the library's rule builds for this shape, as a candidate: a FICCO_AUTO_ANY plan for shards in device
        memory; for shards in pinned host memory the caller says so (ficco_pick_schedule_layout, ROW_MAJOR_HOST)."""
        if host_resident:
            s_h, c_h = F.ficco_pick_schedule_layout(M, K, N, G, F.FICCO_LAYOUT_ROW_MAJOR_HOST)
            return (s_h, c_h, "rm")
        plan = F.ficco_plan(M, K, N, G, 1, F.FICCO_AUTO_ANY)
        try:
            info = F.ficco_plan_info(plan)
            c = info.chunks
            if info.schedule == F.FICCO_FINE_2D:
                w = tuple(F.ficco_plan_slices(plan)[1])
                if len(set(w)) > 1:
                    c = w
            return (info.schedule, c, "rm")
        finally:
            F.ficco_destroy(plan)
    if rs:
        s_rs, c_rs = F.ficco_pick_schedule_rs(M, K, N, G)
        pick = (s_rs, c_rs, "rm")
        pick_host = None           # peers in pinned host memory: no rule (everything is bound by the host link); the screen decides
    else:
        pick = library_pick()
        pick_host = library_pick(host_resident=True)
    if args.candidates:
        cands = [parse_plan(t) for t in args.candidates.split(",")]
    else:
        cands = []
        for rows in cfg["chunk_rows"]:
            c = ms_shard // rows
            for s in (F.FICCO_FINE_FUSED, F.FICCO_FINE_PERSISTENT, F.FICCO_FINE_UNFUSED):
                if (s, c, "rm") not in cands:
                    cands.append((s, c, "rm"))
        for lay in ("rm", "ks"):
            cands += [(F.FICCO_FINE_2D, c, lay) for c in cfg.get("k_slices", [])]
            cands += [(F.FICCO_FINE_2D, tuple(w), lay) for w in cfg.get("k_widths", [])]
    for pk in (pick, pick_host):
        if pk is not None and pk not in cands:
            cands.append(pk)
            if pk[0] == F.FICCO_FINE_2D:
                cands.append((pk[0], pk[1], "ks"))

    out = {"metric": ("GEMM+RS(data movement)" if cfg["direction"] == "gemm_rs" else "AG+GEMM")
                     + " effective TFLOP/s (overlapped pair, the schedule the library picks)",
           "value": None, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16", "data": "synthetic",
           "config": {"workload": args.workload, "M": M, "K": K, "N": N, "shards": G,
                      "source": "device staging buffer (HBM-resident), one SDMA engine per shard as its link"}}

    def leg_pair(tag):
        res = {}
        A_src = source(tag, F.FICCO_SERIAL, 1)
        chain = not rs
        # short screening of the candidates. The first plan of a process reads 5-10 % slow for its first 30 ms or
        # so (clocks, first use of everything), so the first candidate warms up that long before it is timed.
        screen = {}
        for i, sc in enumerate(cands):
            plan = make(*sc)
            screen[sc] = timed_steps(plan, source(tag, *sc), max(5, args.steps // 5), 3, warm_seconds=0.06 if i == 0 else 0.02)
            F.ficco_destroy(plan)
        # The schedule of this run is the library's own pick. It is timed in full, with a blocking query
        # after every step and - the figure that counts - with steps back to back through two chained plans.
        # The best of the screen is timed the same way beside it.
        screen_best = min(screen, key=screen.get)
        my_pick = pick_host if tag == "pcie" else pick
        timed = my_pick if my_pick is not None else screen_best
        def full(sc):
            p_f = make(*sc)
            synced = timed_steps(p_f, source(tag, *sc), args.steps, args.warmup)
            info_f, st_f = F.ficco_plan_info(p_f), F.ficco_query_stats(p_f)
            F.ficco_destroy(p_f)
            ms_f = timed_steps_chained(sc, source(tag, *sc), args.steps, args.warmup) if chain and sc[0] < PACKED else synced
            return ms_f, synced, info_f, st_f
        ms, ms_synced, info, st = full(timed)
        ms_best, ms_best_synced = (ms, ms_synced) if screen_best == timed else full(screen_best)[:2]
        # the best row-piece schedule, when column pieces were timed
        rows_best, ms_rows = None, None
        if timed[0] % PACKED == F.FICCO_FINE_2D:
            rows_best = min((k for k in screen if k[0] % PACKED != F.FICCO_FINE_2D), key=screen.get, default=None)
            if rows_best is not None:
                ms_rows = full(rows_best)[0]
        p_ser = make(F.FICCO_SERIAL, 1)
        ms_ser_synced = timed_steps(p_ser, A_src, args.steps, args.warmup)
        st_ser = F.ficco_query_stats(p_ser)
        F.ficco_destroy(p_ser)
        ms_ser = timed_steps_chained((F.FICCO_SERIAL, 1, "rm"), A_src, args.steps, args.warmup) if chain else ms_ser_synced
        p_sh = make(F.FICCO_SHARD, 1)
        ms_sh = timed_steps(p_sh, A_src, args.steps, args.warmup)
        F.ficco_destroy(p_sh)
        if chain:
            ms_sh = timed_steps_chained((F.FICCO_SHARD, 1, "rm"), A_src, args.steps, args.warmup)
        # shard-sized pieces over all links at once: what shard granularity gives when the links are not the
        # difference (the shard-level schedule above moves one shard at a time over one link, Fig. 3(c))
        all_links_c1 = {label(k): round(v, 4) for k, v in screen.items() if k[1] == 1 and k[0] % PACKED != F.FICCO_FINE_2D}
        # the paper's "hetero" start, for information (never `value`): shard 0 is this GPU's own and already in
        # place, so seven shards travel and the GEMM starts on local rows at once
        ms_het = None
        if not rs and timed[0] % PACKED != F.FICCO_FINE_2D:
            ms_shard_rows = M // G
            A_dev[:ms_shard_rows].copy_(A_stage[:ms_shard_rows])
            torch.cuda.synchronize()
            het = [(F.FICCO_OPT_LOCAL_SHARD, 0)]
            ms_het = timed_steps_chained(timed, source(tag, *timed), args.steps, args.warmup, opts=het)
        res.update(copy_backend={1: "stream", 2: "engines"}.get(info.copy_backend), links=info.links,
                   ms_per_step=ms, eff_tflops=flops / ms * 1e-9,
                   picked_by=("the screen" if my_pick is None else
                              "the library (ficco_pick_schedule_rs)" if rs else
                              "the library (ficco_pick_schedule_layout, shards in pinned host memory)" if tag == "pcie" else
                              "the library (FICCO_AUTO_ANY)"),
                   stepping=("two plans chained behind each other take the steps in turn; the host runs one step ahead"
                             if chain else "a blocking query after every step"),
                   ms_per_step_host_synced=ms_synced, ms_serial_host_synced=ms_ser_synced,
                   schedule=sched_name(timed[0]), chunks_per_shard=pieces_of(timed[1]),
                   source_layout=("row-major (the caller's)" if timed[2] == "rm" else "K-sliced by the sender"),
                   chunk_rows=ms_shard if timed[0] % PACKED == F.FICCO_FINE_2D else ms_shard // timed[1],
                   slice_widths=(list(timed[1]) if isinstance(timed[1], tuple) else None),
                   tile=f"{info.tile_m}x{info.tile_n}", ms_serial=ms_ser, ms_shard_level=ms_sh,
                   speedup_vs_serial=ms_ser / ms, speedup_vs_shard_level=ms_sh / ms,
                   speedup_vs_shard_level_note="the shard-level schedule sends one shard after the other over one link while the finer "
                                               "schedules use all links at once: the ratio is dominated by the link count; "
                                               "shard_granularity_all_links has shard-sized pieces over all links",
                   shard_granularity_all_links_ms_host_synced=all_links_c1,
                   copy_gbps_serial=st_ser.copy_gbps, copy_span_us=st.copy_span_us,
                   ms_local_shard_resident=ms_het,
                   screen_best=label(screen_best), ms_screen_best=ms_best, ms_screen_best_host_synced=ms_best_synced,
                   pick_vs_screen_best=ms / ms_best,
                   best_row_pieces=(label(rows_best) if rows_best else None), ms_best_row_pieces=ms_rows,
                   screen_ms_host_synced={label(k): round(v, 4) for k, v in screen.items()})
        if not rs:
            s_rows, c_rows = F.ficco_pick_schedule(M, K, N, G)
            res["row_piece_rule"] = label((s_rows, c_rows, "rm"))
        return res, timed

    best = None
    if "pair" in legs:
        res, best = leg_pair("hbm")
        out["value"] = round(res["eff_tflops"], 3)
        out["ms_per_step"] = round(res["ms_per_step"], 5)
        out["pair"] = {k: (round(v, 4) if isinstance(v, float) else v) for k, v in res.items()}
        out["config"].update(schedule=res["schedule"], chunks_per_shard=res["chunks_per_shard"], tile=res["tile"],
                             picked_by=res["picked_by"], source_layout=res["source_layout"])
        if res["slice_widths"]:
            out["config"]["slice_widths"] = res["slice_widths"]
    if "roofline" in legs:
        if best:
            s, c, lay = best
        elif args.roofline_plan:
            s, c, lay = parse_plan(args.roofline_plan)
        else:
            s, c, lay = pick if pick is not None else (F.FICCO_FINE_PERSISTENT, 1, "rm")
        s %= PACKED                                    # Gather/Scatter only exists in the overlapped pair
        def launch_time(sched, chunks, A_res):
            """Average duration of the plan's GEMM launches, operands resident: one run that enqueues them
            `steps` times back to back between the two HIP events it records on the compute stream
            (FICCO_OPT_REPEAT), so the figure holds the kernels and the gaps between them, nothing else."""
            plan = make(sched, chunks, opts=[(F.FICCO_OPT_MODE, F.FICCO_MODE_GEMM_ONLY)])
            for _ in range(args.warmup):
                F.ficco_run(plan, None, A_res, W_dev, C_dev, None, cs, xs)
            st1 = F.ficco_query_stats(plan)
            F.ficco_plan_set(plan, F.FICCO_OPT_REPEAT, args.steps)
            # After an idle spell the shader clock needs some tens of milliseconds of load to settle, which
            # a handful of warm-up runs do not give (brackets of 20 launches of 55 us read 56, 64, 68, 65, 63,
            # 60 us in a row, then 54 us for good): brackets are repeated until 40 ms of them have run,
            # and the one after that counts.
            settled_us = 0.0
            while True:
                F.ficco_run(plan, None, A_res, W_dev, C_dev, None, cs, xs)
                st = F.ficco_query_stats(plan)
                if settled_us >= 40e3:
                    break
                settled_us += st.wall_us
            info = F.ficco_plan_info(plan)
            F.ficco_destroy(plan)
            return st.wall_us / args.steps, st1.n_launches, info

        us_step, launches, info = launch_time(s, c, A_stage if rs else source("hbm", s, c, "ks"))   # operands resident in the layout the kernel reads (column pieces: K-sliced)
        achieved = flops / us_step * 1e-6
        # the monolithic GEMM of the same shape, for reference
        whole_us, _, winfo = launch_time(F.FICCO_SERIAL, 1, A_stage)
        whole = [whole_us]
        kname = {F.FICCO_FINE_PERSISTENT: "gemm_resident_kernel", F.FICCO_FINE_2D: "gemm_resident2d_kernel"}.get(s, "gemm_blocks_kernel") \
            + f"<{info.tile_m}x{info.tile_n}>"
        pmc = PMC_KIB.get((args.workload, kname)) if launches == 1 else None
        traffic = int(sum(pmc[k] * PMC_SCALE[k] for k in pmc) * 1024) if pmc else None
        out["roofline"] = {"bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                           "unit": "TFLOP/s", "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": traffic,
                           "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled; see profiles/)",
                           "algorithmic_bytes": 2 * (M * K + K * N + M * N),
                           "kernel": kname,
                           "launches_per_step": launches, "avg_launch_us": round(us_step / max(launches, 1), 3),
                           "flops_per_launch": flops // max(launches, 1),
                           "monolithic_us": round(float(np.mean(whole)), 3),
                           "monolithic_tflops": round(flops / float(np.mean(whole)) * 1e-6, 2),
                           "monolithic_tile": f"{winfo.tile_m}x{winfo.tile_n}"}
        if "pair" in out and traffic:
            # memory side of the overlapped pair: what the GEMM moves beyond its L2s (counters above) plus what the
            # copy engines read and write (the staging buffer and A_dev both live in HBM), over the step time
            step_bytes = traffic + 2 * (M * N * 2 if rs else M * K * 2)
            out["pair"]["hbm_side_bytes_per_step"] = step_bytes
            out["pair"]["hbm_side_frac_of_peak"] = round(step_bytes / (out["ms_per_step"] * 1e-3) / (HBM_PEAK_GBPS * 1e9), 4)

    if "power" in legs and not rs:
        # (not in the default set) board power while the timed plan's GEMM launches loop for about a second, on the
        # workload's own data and on zeros: the chip holds its power limit by lowering the shader clock, and how
        # far depends on how many bits toggle, so the same kernel is faster on zeros. Beside it the vendor
        # library's GEMM (torch.matmul on the same operands, weight in the k-contiguous layout it is fastest in),
        # as the practical ceiling of the machine at that power.
        import glob
        import threading
        pw_files = glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") or \
            glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average")

        def looped(fn, seconds=1.2):
            samples, stop = [], [False]

            def sample():
                while not stop[0]:
                    try:
                        samples.append(max(float(open(f).read()) for f in pw_files))
                    except (OSError, ValueError):
                        pass
                    time.sleep(0.004)
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            th = threading.Thread(target=sample, daemon=True)
            th.start()
            t0, n = time.perf_counter(), 0
            while time.perf_counter() - t0 < seconds:
                fn()
                n += 1
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            stop[0] = True
            th.join()
            tail = samples[len(samples) // 3:]
            return dt / n, (sum(tail) / len(tail) * 1e-6 if tail else None)

        s, c, lay = parse_plan(args.roofline_plan) if args.roofline_plan else (pick if pick is not None else (F.FICCO_FINE_PERSISTENT, 1, "rm"))
        s %= PACKED
        REP = 20
        res = {}
        for kind in ("workload", "zeros"):
            A_k = source("hbm", s, c, "ks") if kind == "workload" else torch.zeros_like(A_stage)
            W_k = W_dev if kind == "workload" else torch.zeros_like(W_dev)
            plan = make(s, c, "ks", opts=[(F.FICCO_OPT_MODE, F.FICCO_MODE_GEMM_ONLY)])
            F.ficco_pack_weight(plan, W_k, cs)
            F.ficco_plan_set(plan, F.FICCO_OPT_REPEAT, REP)

            def ours():
                F.ficco_run(plan, None, A_k, W_k, C_dev, None, cs, xs)
                F.ficco_query_stats(plan)
            t, watts = looped(ours)
            F.ficco_destroy(plan)
            Ab = (A_stage if kind == "workload" else torch.zeros_like(A_stage)).view(torch.bfloat16)
            Wt_b = W_k.view(torch.bfloat16).t().contiguous()

            def vendor():
                for _ in range(REP):
                    torch.matmul(Ab, Wt_b.t())
            tv, wv = looped(vendor)
            res[kind] = {"tflops": round(flops / (t / REP) * 1e-12, 1), "watts": round(watts, 0) if watts else None,
                         "vendor_library_tflops": round(flops / (tv / REP) * 1e-12, 1), "vendor_library_watts": round(wv, 0) if wv else None}
        out["power"] = res

    if "contend" in legs and not rs:
        # counter runs only: the plan's GEMM launches with the plan's transfers running beside them and no
        # dependency between the two (FICCO_MODE_INDEPENDENT), so that rocprofv3 --pmc reads the kernel's
        # counters under the copy engines' traffic; the roofline leg gives the same kernel alone
        s, c, lay = parse_plan(args.roofline_plan) if args.roofline_plan else (pick if pick is not None else (F.FICCO_FINE_PERSISTENT, 1, "rm"))
        s %= PACKED
        plan = make(s, c, "ks", opts=[(F.FICCO_OPT_MODE, F.FICCO_MODE_INDEPENDENT)])
        src = source("hbm", s, c, "ks")
        A_dev.copy_(src if isinstance(src, torch.Tensor) else A_stage)     # the kernel reads resident operands
        torch.cuda.synchronize()
        ms = timed_steps(plan, src, args.steps, args.warmup)
        st = F.ficco_query_stats(plan)
        F.ficco_destroy(plan)
        out["contend"] = {"ms_per_step": round(ms, 4), "gemm_span_us": round(st.gemm_span_us, 2), "copy_span_us": round(st.copy_span_us, 2)}

    # after the roofline leg: half a second of host-link-bound steps leaves the chip in a lower clock state than
    # the settling loop of that leg brings back (its launches read 5 % longer behind this leg than in front of it)
    if "pcie" in legs:
        res, _ = leg_pair("pcie")
        out["pcie_inclusive"] = {k: (round(v, 4) if isinstance(v, float) else v) for k, v in res.items()}

    if "losses" in legs and not rs:
        sc = best if best else (pick if pick is not None else (F.FICCO_FINE_FUSED, 2, "rm"))
        sc = (sc[0] % PACKED, sc[1], sc[2])
        losses = {}
        for tag in ("hbm", "pcie"):
            src = source(tag, *sc)
            plan = make(*sc)
            L = F.ficco_profile_losses(plan, src, A_dev, W_dev, C_dev, cs, xs, 10, 5)
            F.ficco_destroy(plan)
            losses[tag] = {k: round(v, 4) for k, v in L.as_dict().items()}
            losses[tag]["gemm_dil_pct"] = round((L.gemm_dil - 1) * 100, 2)
            losses[tag]["gemm_cil_pct"] = round((L.gemm_cil - 1) * 100, 2)
            losses[tag]["comm_dil_pct"] = round((L.comm_dil - 1) * 100, 2)
            losses[tag]["comm_cil_pct"] = round((L.comm_cil - 1) * 100, 2)
        out["losses"] = losses

    if "small" in legs and not rs and args.workload == "cfg3_ffn70b":
        # the two smaller all-gather workloads, each by a run of this script of its own (pair and pcie legs),
        # condensed to: serial, shard-level, the library's pick, the best of the screen; both source kinds
        import subprocess
        small = {}
        for w in ("cfg1_tiny", "cfg2_qkv8b"):
            r = subprocess.run([sys.executable, os.path.abspath(__file__), "--workload", w, "--legs", "pair,pcie",
                                "--steps", str(min(args.steps, 30)), "--warmup", str(min(args.warmup, 5))],
                               stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
            if r.returncode != 0:
                small[w] = {"error": r.stderr[-400:]}
                continue
            d = json.loads(r.stdout.strip().splitlines()[-1])
            row = {"shape": [d["config"]["M"], d["config"]["K"], d["config"]["N"]]}
            for key, leg in (("hbm_staging", "pair"), ("pinned_host", "pcie_inclusive")):
                q = d[leg]
                row[key] = {"ms_serial": q["ms_serial"], "ms_shard_level": q["ms_shard_level"],
                            "library_pick": f'{q["schedule"]}:' + ("+".join(map(str, q["slice_widths"])) if q["slice_widths"] else str(q["chunks_per_shard"])),
                            "ms_library_pick": q["ms_per_step"], "eff_tflops": q["eff_tflops"],
                            "speedup_vs_serial": q["speedup_vs_serial"], "speedup_vs_shard_level": q["speedup_vs_shard_level"],
                            "screen_best": q["screen_best"], "ms_screen_best": q["ms_screen_best"],
                            "best_row_pieces": q["best_row_pieces"], "ms_best_row_pieces": q["ms_best_row_pieces"],
                            "shard_granularity_all_links_ms_host_synced": q["shard_granularity_all_links_ms_host_synced"]}
            small[w] = row
        out["small_workloads"] = small

    if "graph" in legs and not rs:
        # HIP-graph replay of one run against the same run enqueued call by call (stream backend, shards in
        # pinned host memory): mean step time, and the host time one enqueue takes
        res = {}
        for sname, sched, c in (("serial", F.FICCO_SERIAL, 1), ("fine_fused", F.FICCO_FINE_FUSED, 4), ("fine_unfused", F.FICCO_FINE_UNFUSED, 4)):
            plan = make(sched, c, opts=[(F.FICCO_OPT_COPY_BACKEND, F.FICCO_COPY_STREAM)])
            row = {}
            for how in ("eager", "graph"):
                if how == "graph":
                    F.ficco_graph_capture(plan, A_pinned, A_dev, W_dev, C_dev, None)

                def step():
                    if how == "eager":
                        F.ficco_run(plan, A_pinned, A_dev, W_dev, C_dev, None, cs, xs)
                    else:
                        F.ficco_graph_launch(plan, cs)
                for _ in range(args.warmup):
                    step()
                    F.ficco_query_stats(plan)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(args.steps):
                    step()
                    F.ficco_query_stats(plan)
                torch.cuda.synchronize()
                ms = (time.perf_counter() - t0) * 1e3 / args.steps
                h0 = time.perf_counter()
                step()
                h1 = time.perf_counter()
                F.ficco_query_stats(plan)
                row[how] = {"ms_per_step": round(ms, 4), "host_enqueue_us": round((h1 - h0) * 1e6, 1)}
            F.ficco_destroy(plan)
            res[f"{sname}:{c}"] = row
        out["graph"] = res

    if "reduce" in legs or "reduce_kernel" in legs:
        # receiver side of the reduce-scatter: G-1 partial blocks [M/G, N] arrive over the links and are added
        # to this GPU's own; serial (receive, then add) against pieces added as they land
        from oracle import reduce as orr
        rows = M // G
        x = fi.make_partials(cfg["seed"], G, rows, N)
        P_stage = torch.from_numpy(x.view(np.int16)).to(dev)
        P_land = torch.zeros((G, rows, N), dtype=torch.int16, device=dev)
        own = P_stage[0].clone()
        red = torch.zeros((rows, N), dtype=torch.int16, device=dev)
        torch.cuda.synchronize()

        def reduce_plan(sched, c, opts=()):
            plan = F.ficco_plan(M, K, N, G, c, sched)
            for o, v in opts:
                F.ficco_plan_set(plan, o, v)
            return plan

        def reduce_steps(plan, steps, warmup):
            for _ in range(warmup):
                F.ficco_rs_reduce(plan, 0, P_stage, P_land, own, red, cs)
                F.ficco_query_stats(plan)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                F.ficco_rs_reduce(plan, 0, P_stage, P_land, own, red, cs)
                st = F.ficco_query_stats(plan)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / steps, st

        rres = {}
        cases = [("serial", F.FICCO_SERIAL, 1), ("shard_level", F.FICCO_SHARD, 1)] + \
                [(f"fine:{c}", F.FICCO_FINE_FUSED, c) for c in (2, 4, 8, 16) if rows % c == 0]
        if "reduce" in legs:                         # bring the clocks up before the first (serial) case is timed
            p_warm = reduce_plan(F.FICCO_SERIAL, 1)
            t_warm = time.perf_counter()
            while time.perf_counter() - t_warm < 0.05:
                F.ficco_rs_reduce(p_warm, 0, P_stage, P_land, own, red, cs)
                F.ficco_query_stats(p_warm)
            F.ficco_destroy(p_warm)
        for name, sched, c in (cases if "reduce" in legs else cases[2:3]):      # reduce_kernel: one pass, for the parity check
            plan = reduce_plan(sched, c)
            ms, st = reduce_steps(plan, args.steps if "reduce" in legs else 1, args.warmup if "reduce" in legs else 0)
            F.ficco_destroy(plan)
            rres[name] = round(ms, 4)
        best_name = min((k for k in rres if k.startswith("fine")), key=rres.get)
        got = red.cpu().numpy().view(np.uint16)
        # the kernel alone, landing buffer resident: HIP events recorded on the stream around each launch
        plan = reduce_plan(F.FICCO_FINE_FUSED, int(best_name.split(":")[1]), [(F.FICCO_OPT_MODE, F.FICCO_MODE_GEMM_ONLY)])
        spans = []
        for it in range(args.warmup + args.steps):
            F.ficco_rs_reduce(plan, 0, P_stage, P_land, own, red, cs)
            st = F.ficco_query_stats(plan)
            if it >= args.warmup:
                spans.append(st.wall_us)
        F.ficco_destroy(plan)
        us = float(np.mean(spans))
        alg_bytes = (G + 1) * rows * N * 2
        t0 = time.perf_counter()
        want = orr.rs_reduce(list(x))
        dt = time.perf_counter() - t0
        out["reduce"] = {"block": [rows, N], "peers": G, "ms_per_step": rres if "reduce" in legs else None, "best": best_name,
                         "speedup_vs_serial": round(rres["serial"] / rres[best_name], 4) if "reduce" in legs else None,
                         "speedup_vs_shard_level": round(rres["shard_level"] / rres[best_name], 4) if "reduce" in legs else None,
                         "bits_equal_oracle": bool(np.array_equal(got, want)),
                         "roofline": {"bound": "hbm", "achieved": round(alg_bytes / us * 1e-3, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                      "frac": round(alg_bytes / us * 1e-3 / HBM_PEAK_GBPS, 4),
                                      "traffic": (lambda t: int(sum(t[k] * PMC_SCALE[k] for k in t) * 1024) if t else None)(
                                          PMC_KIB.get((args.workload, "rs_reduce_kernel"))),
                                      "algorithmic_bytes": alg_bytes, "kernel": "rs_reduce_kernel", "avg_launch_us": round(us, 3)},
                         "cpu_baseline": {"value": round(alg_bytes / dt * 1e-9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
                                          "sample": f"the whole block, {dt:.2f} s"}}

    if "calib" in legs:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["calib"] = {"kernel": "torch elementwise copy", "bytes_read": 256 << 20, "bytes_written": 256 << 20, "launches": 3}

    if "cpu" in legs:
        from oracle import gemm as og
        # bounded sample of the same workload: the whole product when it is small, otherwise as many
        # random rows as about 20 s of CPU work allow (rate calibrated on 64 rows first)
        rng = np.random.default_rng(0)
        if flops <= 2e11:
            rows = np.arange(M, dtype=np.int64)
        else:
            probe = np.sort(rng.choice(M, size=64, replace=False)).astype(np.int64)
            t0 = time.perf_counter()
            og.ag_gemm_rows(shards, W, probe)
            per_row = (time.perf_counter() - t0) / 64
            rows_n = int(min(M, max(64, 20.0 / per_row)))
            rows = np.sort(rng.choice(M, size=rows_n, replace=False)).astype(np.int64)
        rows_n = int(rows.size)
        t0 = time.perf_counter()
        ref = og.ag_gemm(shards, W) if rows_n == M else og.ag_gemm_rows(shards, W, rows)
        dt = time.perf_counter() - t0
        got = C_dev.cpu().numpy().view(np.uint16)[rows]
        err = og.rel_err(fi.bf16_bits_to_f32(got).astype(np.float64), ref) if "pair" in legs or "roofline" in legs else None
        out["cpu_baseline"] = {"value": round(2 * rows_n * N * K / dt * 1e-12, 6), "unit": "TFLOP/s",
                               "cores": og.num_threads(), "kind": "oracle",
                               "sample": (f"the whole {M}x{K}x{N} product, {dt:.1f} s" if rows_n == M else
                                          f"{rows_n} random rows of the {M}x{K}x{N} product, all {N} columns, {dt:.1f} s"),
                               "gpu_vs_oracle_rel_err": err}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
