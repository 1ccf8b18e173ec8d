#!/usr/bin/env python3
"""Heuristic sweep (paper Sec. V-C, Sec. VI-D): measure every schedule and piece count on a grid of
all-gather -> GEMM shapes on this GPU, fit the thresholds of the static schedule rule, and report
how often the rule picks the measured best.

    python -m paper_2512_10236_amd.sweep --out sweep.jsonl            # measure
    python -m paper_2512_10236_amd.sweep --fit sweep.jsonl            # fit + accuracy

Shapes default to the grid M in {4096,16384,65536} x K in {4096,8192} x N in {512,1024,3584,14336},
8 shards, pieces per shard in {1,2,4,8,16,32}; shards are moved from a device staging buffer by one
SDMA engine per shard. Inputs are seeded normal bf16 (A ~ N(0,1), W ~ N(0,1/K)) generated on the
device; every schedule's output is compared bitwise with the serial schedule's.
PyTorch is used for device memory and streams only.
"""
from __future__ import annotations

import argparse
import json
import math
import sys

from . import binding as F

FINE = (F.FICCO_FINE_UNFUSED, F.FICCO_FINE_FUSED, F.FICCO_FINE_PERSISTENT)


def measure(args) -> int:
    import torch

    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    cs, xs = torch.cuda.Stream(), torch.cuda.Stream()
    G = args.shards
    out = open(args.out, "w")
    for M in args.M:
        for K in args.K:
            gen = torch.Generator(device=dev)
            gen.manual_seed(4)
            A_stage = torch.randn((M, K), device=dev, generator=gen).to(torch.bfloat16).view(torch.int16)
            A_dev = torch.zeros((M, K), dtype=torch.int16, device=dev)
            for N in args.N:
                W = (torch.randn((K, N), device=dev, generator=gen) * K ** -0.5).to(torch.bfloat16).view(torch.int16)
                C = torch.zeros((M, N), dtype=torch.int16, device=dev)
                C_ref = None
                cases = [(F.FICCO_SERIAL, 1, None), (F.FICCO_SHARD, 1, None)]
                cases += [(s, c, None) for c in args.chunks for s in FINE if (M // G) % c == 0 and c * G <= 4096]
                # the 2D schedule (k slices) wherever the slices are whole k-tiles; its source is the K-sliced copy
                cases += [(F.FICCO_FINE_2D, c, None) for c in args.chunks if c > 1 and K % (64 * c) == 0 and c * G <= 4096]
                # what ficco_pick_schedule_any answers, when that is column pieces in a cut of its own
                ps, pc = F.ficco_pick_schedule_any(M, K, N, G)
                if ps == F.FICCO_FINE_2D:
                    pw = F.ficco_pick_slice_widths(M, K, N, G, pc)
                    if len(set(pw)) > 1:
                        cases.append((ps, pc, pw))
                for sched, c, widths in cases:
                    src = A_stage
                    if widths is not None:
                        edges = [sum(widths[:i]) for i in range(len(widths) + 1)]
                        src = torch.cat([A_stage[:, edges[i]:edges[i + 1]].reshape(-1) for i in range(len(widths))]).view(M, K)
                        torch.cuda.synchronize()
                    elif sched == F.FICCO_FINE_2D:
                        src = A_stage.view(M, c, K // c).permute(1, 0, 2).contiguous().view(M, K)
                        torch.cuda.synchronize()
                    plan = F.ficco_plan(M, K, N, G, c, sched)
                    try:
                        if widths is not None:
                            F.ficco_plan_set_slice_widths(plan, widths)
                        F.ficco_pack_weight(plan, W, cs)
                        ts, cps = [], []
                        for it in range(args.warmup + args.iters):
                            if it == 0:
                                C.zero_()
                                torch.cuda.synchronize()
                            F.ficco_run(plan, src, A_dev, W, C, None, cs, xs)
                            st = F.ficco_query_stats(plan)
                            if it >= args.warmup:
                                ts.append(st.wall_us)
                                cps.append(st.copy_span_us)
                        info = F.ficco_plan_info(plan)
                    finally:
                        F.ficco_destroy(plan)
                    torch.cuda.synchronize()
                    if C_ref is None:
                        C_ref = C.clone()
                        same = True
                    else:
                        same = bool(torch.equal(C, C_ref))
                    row = dict(M=M, K=K, N=N, shards=G, schedule=F.SCHEDULE_NAMES[sched], sched_id=sched, chunks=c,
                               wall_us=round(sum(ts) / len(ts), 2), min_us=round(min(ts), 2),
                               copy_span_us=round(sum(cps) / len(cps), 2), tile=f"{info.tile_m}x{info.tile_n}",
                               bits_equal_serial=same)
                    if widths is not None:
                        row["widths"] = widths
                    out.write(json.dumps(row) + "\n")
                    out.flush()
                    print(json.dumps(row), flush=True)
                    if not same:
                        print("sweep: output differs bitwise from the serial schedule", file=sys.stderr)
                        return 1
                del W, C, C_ref
            del A_stage, A_dev
            torch.cuda.empty_cache()
    return 0


def rule(M, K, N, G, piece_flops, min_rows, max_pieces):
    """The static rule of ficco_pick_schedule with free constants: the resident schedule, and as many
    pieces per shard as keep one piece's GEMM (OTB x MT = its flops) above ``piece_flops``."""
    ms = M // G
    t = piece_flops / (2.0 * N * K)
    m = 1
    while m * 2 <= t:
        m *= 2
    m = max(min_rows, min(m, ms))
    c = max(1, min(max_pieces, ms // m))
    while c > 1 and ms % c:
        c //= 2
    return F.FICCO_FINE_PERSISTENT, c


def fit(args) -> int:
    rows = [json.loads(l) for l in open(args.fit) if l.startswith("{")]
    shapes = {}
    for r in rows:
        shapes.setdefault((r["M"], r["K"], r["N"], r["shards"]), []).append(r)
    keys = sorted(shapes)
    table = []
    for k in keys:
        rs = shapes[k]
        serial = next(r for r in rs if r["schedule"] == "serial")["wall_us"]
        shard = next(r for r in rs if r["schedule"] == "shard")["wall_us"]
        fine = [r for r in rs if r["sched_id"] in FINE]
        best = min(fine, key=lambda r: r["wall_us"])
        two_d = [r for r in rs if r["sched_id"] == F.FICCO_FINE_2D and "widths" not in r]
        cut = [r for r in rs if r["sched_id"] == F.FICCO_FINE_2D and "widths" in r]
        if two_d:
            b2 = min(two_d, key=lambda r: r["wall_us"])
            note_2d = f"  best 2D x{b2['chunks']} {b2['wall_us']:9.1f} us ({best['wall_us'] / b2['wall_us']:.3f}x of best 1D)"
        else:
            note_2d = ""
        table.append(dict(key=k, serial=serial, shard=shard, best=best, fine={(r["sched_id"], r["chunks"]): r["wall_us"] for r in fine},
                          best_2d=min((r["wall_us"] for r in two_d), default=None),
                          two_d={r["chunks"]: r["wall_us"] for r in two_d},
                          rule_cut={(r["chunks"], tuple(r["widths"])): r["wall_us"] for r in cut}))
        print(f"M={k[0]:6d} K={k[1]:5d} N={k[2]:6d}: serial {serial:9.1f} us  shard-level {shard:9.1f} us  best {best['schedule']} x{best['chunks']} "
              f"{best['wall_us']:9.1f} us  speedup {serial / best['wall_us']:.3f}x (vs shard-level {shard / best['wall_us']:.2f}x){note_2d}")

    def score(consts, subset):
        hit = near = 0
        loss = []
        for t in subset:
            M, K, N, G = t["key"]
            s, c = rule(M, K, N, G, *consts)
            got = t["fine"].get((s, c))
            if got is None:
                continue
            bw = t["best"]["wall_us"]
            hit += (s, c) == (t["best"]["sched_id"], t["best"]["chunks"])
            near += got <= 1.03 * bw
            if got > 1.03 * bw:
                sp_best, sp_got = t["serial"] / bw, t["serial"] / got
                loss.append((sp_best - sp_got) / sp_best)
        return hit, near, loss

    train, test = table[0::2], table[1::2]
    best_c, best_s = None, (-1, -1)
    for piece_flops in (0.5e10, 1e10, 1.5e10, 2e10, 2.5e10, 3e10, 4e10, 6e10, 1e11):
        for min_rows in (128, 256, 512, 1024):
            for max_pieces in (8, 16, 32):
                consts = (piece_flops, min_rows, max_pieces)
                h, n, _ = score(consts, train)
                if (n, h) > best_s:
                    best_s, best_c = (n, h), consts
    for name, subset in (("fitted on (even shapes)", train), ("held out (odd shapes)", test), ("all", table)):
        h, n, loss = score(best_c, subset)
        ml = 100 * sum(loss) / len(loss) if loss else 0.0
        print(f"{name}: exact pick {h}/{len(subset)}, within 3% of best {n}/{len(subset)}, mean loss of optimal speedup on misses {ml:.1f}%")
    print("fitted constants: piece flops %.3g, min rows %d, max pieces %d" % best_c)
    # the shape rule of Sec. V-C: column pieces (2D) when M <= K, row pieces (1D) otherwise
    with_2d = [t for t in table if t["best_2d"] is not None]
    if with_2d:
        ok = near = 0
        for t in with_2d:
            M, K = t["key"][0], t["key"][1]
            picked, other = (t["best_2d"], t["best"]["wall_us"]) if M <= K else (t["best"]["wall_us"], t["best_2d"])
            ok += picked <= other
            near += picked <= 1.03 * other
        n_le = sum(1 for t in with_2d if t["key"][0] <= t["key"][1])
        print(f"shape rule (2D when M <= K, else 1D): picks the faster family at {ok}/{len(with_2d)} shapes, "
              f"within 3% of it at {near}/{len(with_2d)} ({n_le} shapes have M <= K)")
    h, n, loss = score((2.5e10, 256, 16), table)
    print(f"constants compiled into ficco_pick_schedule (2.5e10, 256, 16): exact {h}/{len(table)}, within 3% {n}/{len(table)}")
    # ficco_pick_schedule_any (column pieces allowed) against the best of both families
    if with_2d:
        hit = near = fam = 0
        worst = 0.0
        for t in with_2d:
            M, K, N, G = t["key"]
            s, c = F.ficco_pick_schedule_any(M, K, N, G)
            got = t["two_d"].get(c) if s == F.FICCO_FINE_2D else t["fine"].get((s, c))
            if s == F.FICCO_FINE_2D:           # the rule's own cut, where the sweep measured it
                got = t["rule_cut"].get((c, tuple(F.ficco_pick_slice_widths(M, K, N, G, c))), got)
            if got is None:
                continue
            best = min([t["best"]["wall_us"], t["best_2d"]] + list(t["rule_cut"].values()))
            hit += got <= 1.001 * best
            near += got <= 1.03 * best
            worst = max(worst, got / best)
            fam += (s == F.FICCO_FINE_2D) == (t["best_2d"] <= t["best"]["wall_us"])
        n_cut = sum(1 for t in with_2d if t["rule_cut"])
        print(f"(column pieces in the rule's own unequal cut were measured at {n_cut} shapes and count among the candidates)")
        print(f"ficco_pick_schedule_any against the best of row and column pieces: exact {hit}/{len(with_2d)}, within 3% {near}/{len(with_2d)}, "
              f"worst {100 * (worst - 1):.1f}% off, faster family picked at {fam}/{len(with_2d)} shapes")
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default="")
    ap.add_argument("--fit", default="")
    ap.add_argument("--M", type=int, nargs="+", default=[4096, 16384, 65536])
    ap.add_argument("--K", type=int, nargs="+", default=[4096, 8192])
    ap.add_argument("--N", type=int, nargs="+", default=[512, 1024, 3584, 14336])
    ap.add_argument("--chunks", type=int, nargs="+", default=[1, 2, 4, 8, 16, 32])
    ap.add_argument("--shards", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--iters", type=int, default=5)
    args = ap.parse_args()
    if args.fit:
        return fit(args)
    if not args.out:
        ap.error("give --out FILE to measure or --fit FILE to fit")
    return measure(args)


if __name__ == "__main__":
    sys.exit(main())
