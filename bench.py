#!/usr/bin/env python3
"""Benchmark of the RBE retrieval hot path on one MI355X.

Workload (default): 1,000,000,000 items, d = 64, 3 bit-planes + 3 fp32 scales
per item (36 B/item, 36 GB resident in HBM), clustered synthetic corpus, exact
top-1000.  A step is one whole search -- stage the query, score every item,
select, copy the k results to the host -- for ONE query (the paper's latency
experiment); `value` is items scored and selected per second over the timed
steps.  Further legs in the same line: the same searches with every plane read,
the near-lossless selector, fp32 queries, 16 queries per call, the paper's own
operating point, and the two other large configurations of the workload table
(1e9 near-duplicate items with 8 queries and k = 4000; 1e8 items of d = 128 with
4 planes and 64 queries), each with its own roofline figures.  `--only` runs a
subset (for profiling one kernel under rocprofv3).

Prints exactly one JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E
VALU_PEAK_TLANEOPS = 39.3216     # 256 CU x 4 SIMD x 16 lanes x 2.4 GHz, one 32-bit lane-op per lane per clock
MFMA_F16_PEAK_TFLOPS = 2500.0    # dense fp16 matrix-core peak
MFMA_I8_PEAK_TOPS = 5000.0       # dense int8 matrix-core peak (binary queries on general scales are contracted in int8)


def log(msg: str):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def measured_traffic(workload: str):
    """HBM bytes per finest-level scan launch from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE scaled by the plain-copy yardstick), if it covers this workload.
    Hardware counters cannot be read from inside this process; the figure is the profile's."""
    path = os.path.join(ROOT, "profiles", "scan_exact_1e9_d64_p3_q1.json")
    try:
        with open(path) as f:
            rec = json.load(f)
        if rec.get("workload") == workload:
            return rec.get("traffic_bytes_per_launch")
    except (OSError, ValueError):
        pass
    return None


def oracle_all_cores(oracle, np, planes, scales, qp, qs, k, n_threads):
    """oracle.topk of one query from n_threads host threads over disjoint item ranges (the C call
    releases the interpreter lock), per-range results merged with oracle.topk_of_scores."""
    from concurrent.futures import ThreadPoolExecutor
    n = planes.shape[1]
    edges = np.linspace(0, n, n_threads + 1).astype(np.int64)
    with ThreadPoolExecutor(n_threads) as pool:
        jobs = [pool.submit(oracle.topk, planes, scales, qp, qs, k, int(a), int(b)) for a, b in zip(edges[:-1], edges[1:]) if b > a]
        got = [j.result() for j in jobs]
    ids = np.concatenate([g[0][g[0] >= 0] for g in got])
    sc = np.concatenate([g[1][g[0] >= 0] for g in got])
    return oracle.topk_of_scores(sc, ids, k)


def finest_level_roofline(np, r, W, P, Q, d, kernel):
    """Roofline figures of the finest-level scan of a leg from its search statistics: bytes the method has to
    move per pass (every plane and scale of every item), matrix-core flops of the dense contraction, 32-bit lane
    operations of the XOR/popcount arithmetic, each over the HIP-event time of that launch."""
    items = r["last_items"]
    ms = float(r["scan_ms"].mean())
    bytes_per_item = P * (8 * W + 4)
    passes = -(-Q // 32) if kernel == "scan_batch_mfma" else 1
    out = {"kernel": f"{kernel} (finest level)", "kernel_ms": ms, "items": items,
           "algorithmic_bytes_per_item_per_pass": bytes_per_item, "passes_over_the_level": passes,
           "hbm_gbs": items * bytes_per_item * passes / (ms * 1e-3) / 1e9}
    out["hbm_frac"] = out["hbm_gbs"] / HBM_PEAK_GBS
    deep = float(r["deep_units"].mean()) * 8.0 if r["deep_units"].size else 0.0
    if kernel == "scan_batch_mfma" and Q <= 16 and P >= 2 and deep > 0:
        # the lean stream: planes 0 .. P-2 and one-byte scale copies, plus what the library counted beyond them
        asked = items * (8 * W * (P - 1) + (P - 1)) + deep
        out["bytes_asked_for"] = asked
        out["hbm_gbs_asked_for"] = asked / (ms * 1e-3) / 1e9
    if kernel == "scan_batch_mfma":
        ach = 2.0 * Q * items * d * P / (ms * 1e-3) / 1e12
        out.update({"bound": "mfma", "achieved": ach, "peak": MFMA_I8_PEAK_TOPS, "unit": "TOP/s",
                    "frac": ach / MFMA_I8_PEAK_TOPS, "flops_per_pair": 2 * d * P, "traffic": None,
                    "note": "priced against the int8 matrix-core peak as a dense contraction (the kernel contracts "
                            "eight-bit integer operands); it is held by vector-instruction issue (bits to operand "
                            "bytes, scale multiply-adds, thresholds) at the clock the chip sustains, see profiles/"})
    elif Q >= 3:
        ops = lane_ops_per_pair(W, P, P)
        ach = ops * Q * items / (ms * 1e-3) / 1e12
        out.update({"bound": "alu", "achieved": ach, "peak": VALU_PEAK_TLANEOPS, "unit": "T lane-ops/s",
                    "frac": ach / VALU_PEAK_TLANEOPS, "lane_ops_per_pair": ops, "traffic": None})
    else:
        out.update({"bound": "hbm", "achieved": out["hbm_gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": out["hbm_frac"], "traffic": None})
    return out


def lane_ops_per_pair(W: int, P: int, Pq: int) -> int:
    """32-bit vector lane-operations the scoring arithmetic needs per (query, item)
    pair: per plane pair 2W xor + 2W popcount-accumulate + 1 convert + 1 fma, per
    corpus plane 1 fma, plus 1 compare."""
    return P * Pq * (4 * W + 2) + P + 1


def build_corpus(rbe, rbe_synth, torch, n_items, d, P, n_clusters, sigma, chunk_items, keep_host_items, flags=0):
    dev = torch.device("cuda:0")
    centres = rbe_synth.centres_torch(n_clusters, d, dev)
    ix = rbe.rbe_index_create(n_items, d, P, flags)
    dyadic = bool(flags & rbe.RBE_DYADIC)
    host_planes, host_scales, kept = [], [], 0
    t0 = time.time()
    done, chunk = 0, 0
    while done < n_items:
        n = min(chunk_items, n_items - done)
        x = rbe_synth.vectors_torch(n, centres, sigma, rbe_synth.SEED_ITEMS, chunk)
        planes, scales = rbe_synth.pack_planes_torch(x, P)
        rbe.rbe_load_chunk(ix, done, planes, None if dyadic else scales)
        if kept < keep_host_items:
            take = min(n, keep_host_items - kept)
            host_planes.append(planes[:, :take].cpu().numpy())
            host_scales.append(scales[:, :take].cpu().numpy())
            kept += take
        done += n
        chunk += 1
        if chunk % 16 == 0:
            log(f"corpus {done / 1e6:.0f}M / {n_items / 1e6:.0f}M items, {time.time() - t0:.1f}s")
        del x, planes, scales
    rbe.rbe_finalize(ix)
    torch.cuda.empty_cache()
    log(f"corpus of {n_items} items resident after {time.time() - t0:.1f}s")
    import numpy as np
    hp = np.concatenate(host_planes, axis=1).view(np.uint64) if host_planes else None
    hs = np.concatenate(host_scales, axis=1) if host_scales else None
    return ix, centres, hp, hs


def settle(rbe, rbe_synth, torch, ix, centres, sigma, Pq, k, seconds, binary_scales=True):
    """Untimed searches for `seconds` after a corpus has been built (part of the set-up, before any warm-up step):
    for the first 0.2 s after the build -- generation and encoding of 1e9 items on the GPU -- searches run about
    4 % slower than the rate they then settle at.  Returns the number of searches made."""
    if seconds <= 0:
        return 0
    qp, qs = make_queries(rbe, rbe_synth, torch, centres, 8, sigma, Pq, 99)
    n, t0 = 0, time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        rbe.rbe_search(ix, qp[n % 8:n % 8 + 1], qs[n % 8:n % 8 + 1] if binary_scales else None, k)
        n += 1
    return n


def make_queries(rbe, rbe_synth, torch, centres, n, sigma, P, seed_chunk):
    import numpy as np
    x = rbe_synth.vectors_torch(n, centres, sigma, rbe_synth.SEED_QUERIES, seed_chunk).cpu().numpy()
    enc = [rbe.rbe_encode_query(x[i], P) for i in range(n)]
    return np.stack([e[0] for e in enc]), np.stack([e[1] for e in enc])


def timed_searches(rbe, torch, ix, qp, qs, Q, k, steps, warmup, mode=0, group_size_I=0):
    if qs is None:
        class _NoScales:
            def __getitem__(self, _):
                return None
        qs = _NoScales()
    """Runs warmup + steps searches of Q queries each (different queries per call)."""
    import numpy as np
    per_step, scan_ms, select_ms, total_gpu, all_ids, deep_rows, deep_units, last_items, split_steps = [], [], [], [], [], [], [], [], 0
    stats = None
    fallbacks = 0
    # (the interpreter's cyclic collector stays out of the timed steps: with torch imported a full collection takes
    # about 40 ms, a dozen steps' worth, and comes about once in a thousand searches.  It is run before the warm-up
    # steps, not between them and the timed ones: 40 ms of idling there and the first timed steps run at the
    # clocks of an idle chip, 15 % slower for a batch)
    gc.collect()
    gc.disable()
    for s in range(warmup):
        sl = slice(s * Q, (s + 1) * Q)
        rbe.rbe_search(ix, qp[sl], qs[sl], k, mode, group_size_I)
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for s in range(warmup, warmup + steps):
        sl = slice(s * Q, (s + 1) * Q)
        t0 = time.perf_counter()
        ids, _ = rbe.rbe_search(ix, qp[sl], qs[sl], k, mode, group_size_I)
        per_step.append((time.perf_counter() - t0) * 1e3)
        all_ids.append(ids)
        stats = rbe.rbe_get_search_stats(ix)
        fallbacks += int(stats["fallback"])
        if stats["n_levels"] and not stats["fallback"]:
            # the last (largest) level of the plan: one launch, or two when the library takes it in two parts
            parts = stats["last_level_parts"]
            scan_ms.append(sum(stats["scan_ms"][-parts:]))
            last_items.append(sum(stats["items_scanned"][-parts:]))
            split_steps += int(parts == 2)
            select_ms.append(sum(stats["select_ms"]))
            total_gpu.append(stats["total_gpu_ms"])
            deep_rows.append(stats["deep_rows"])
            deep_units.append(stats["deep_units"])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_begin
    gc.enable()
    return {
        "wall_s": wall, "per_step_ms": np.array(per_step), "scan_ms": np.array(scan_ms),
        "select_ms": np.array(select_ms), "total_gpu_ms": np.array(total_gpu), "stats": stats,
        "ids": all_ids, "deep_rows": np.array(deep_rows), "deep_units": np.array(deep_units), "fallbacks": fallbacks,
        "last_items": int(last_items[-1]) if last_items else 0, "split_steps": split_steps,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--settle-seconds", type=float, default=0.4,
                    help="untimed one-query searches after each corpus build, before the warm-up steps (0 = none)")
    ap.add_argument("--items", type=int, default=1_000_000_000)
    ap.add_argument("--dim", type=int, default=64)
    ap.add_argument("--planes", type=int, default=3)
    ap.add_argument("--k", type=int, default=1000)
    ap.add_argument("--batch", type=int, default=16, help="queries per call of the batch leg (0 = skip)")
    ap.add_argument("--batch-steps", type=int, default=10)
    ap.add_argument("--clusters", type=int, default=4096)
    ap.add_argument("--sigma", type=float, default=0.3)
    ap.add_argument("--chunk-items", type=int, default=4_000_000)
    ap.add_argument("--cpu-sample-items", type=int, default=100_000_000)
    ap.add_argument("--cpu-sample-queries", type=int, default=8)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-nearlossless", action="store_true")
    ap.add_argument("--no-paper-point", action="store_true")
    ap.add_argument("--no-hybrid", action="store_true")
    ap.add_argument("--paper-items", type=int, default=136 * 136 * 256 * 256)
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="also launch the plain copy kernel of this size 5 times (yardstick for rocprofv3 counters)")
    ap.add_argument("--no-config5", action="store_true", help="skip the 1e9 near-duplicate leg (8 queries, k=4000)")
    ap.add_argument("--no-config3", action="store_true", help="skip the 1e8 d=128 4-plane leg (64 queries)")
    ap.add_argument("--config-steps", type=int, default=6, help="timed calls of the config-3 and config-5 legs")
    ap.add_argument("--only", default="", help="comma list of legs to run instead of all: headline, all_planes, near, "
                    "mixed, hybrid, small_batch, batch, batch_popcount, cpu, paper, config5, config3 (headline alone = the contract's steps)")
    args = ap.parse_args()
    only = {x for x in args.only.split(",") if x}
    known = {"headline", "all_planes", "near", "mixed", "hybrid", "small_batch", "batch", "batch_popcount", "cpu", "paper", "config5", "config3"}
    if only - known:
        print(f"bench.py: unknown legs {sorted(only - known)}", file=sys.stderr)
        sys.exit(2)

    def want(leg: str) -> bool:
        return leg in only if only else True
    main_corpus = not only or bool(only & {"headline", "all_planes", "near", "mixed", "hybrid", "batch", "batch_popcount", "cpu"})

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the whole 1e9-item corpus fits one MI355X); "
              "--gpus must be 1: item-range sharding across GPUs is not built.",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_1802_06466_amd as rbe
    import rbe_synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    rbe.load_library()  # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)

    N, d, P, k = args.items, args.dim, args.planes, args.k
    W = d // 64
    bytes_per_item = P * (8 * W + 4)
    cpu_items = 0 if (args.no_cpu_baseline or not want("cpu")) else min(args.cpu_sample_items, N)

    if not main_corpus:
        out = {"metric": "candidates scored+selected/sec and p50 query latency at 1B items, k=1000", "value": None,
               "unit": "candidates/s", "n_gpus": 1, "steps": 0, "warmup": 0, "data": "synthetic",
               "config": {"workload": "subset run (--only %s): no headline steps" % args.only}}
        extra_legs(out, args, want, rbe, rbe_synth, torch, np)
        print(json.dumps(out), flush=True)
        return

    ix, centres, host_planes, host_scales = build_corpus(
        rbe, rbe_synth, torch, N, d, P, args.clusters, args.sigma, args.chunk_items, cpu_items)
    rbe.rbe_set_profiling(ix, True)
    settled = settle(rbe, rbe_synth, torch, ix, centres, args.sigma, P, k, args.settle_seconds)

    # ---------------- single-query leg (the timed steps of the contract)
    n_q1 = args.warmup + args.steps
    qp1, qs1 = make_queries(rbe, rbe_synth, torch, centres, n_q1, args.sigma, P, 0)
    r1 = timed_searches(rbe, torch, ix, qp1, qs1, 1, k, args.steps, args.warmup)
    ms_per_step = r1["wall_s"] * 1e3 / args.steps
    value = N * args.steps / r1["wall_s"]
    st = r1["stats"]
    last_items = r1["last_items"] if st["n_levels"] else N
    scan_avg_ms = float(r1["scan_ms"].mean()) if r1["scan_ms"].size else float("nan")
    # The finest-level scan of one query is progressive.  In two stages (three or more planes): of every item it
    # streams plane 0 and one-byte copies of all its scales; for the items that a bound from those cannot rule out
    # (gathered 64 at a time) a lane reads the planes 1 .. P-2, and for what a second bound still lets through the
    # last plane and the P fp32 scales.  With two planes (or the first stage switched off): every plane but the
    # last and the copies of the matching scales are streamed (plus one fp32 per row of 256 items, the row's largest
    # last scale).  The library counts the bytes asked for beyond the stream (`deep_units` x 8).  `achieved` is
    # priced on the bytes moved; the rate on the bytes of all planes is reported beside it.
    deep_avg = float(r1["deep_rows"].mean()) if r1["deep_rows"].size else 0.0
    deep_bytes = float(r1["deep_units"].mean()) * 8.0 if r1["deep_units"].size else 0.0
    deep_row_bytes = 256 * (8 * W + 4)        # (fp32-query scan: whole rows of the last plane and last scale)
    two_stage = bool(st["n_levels"]) and st["scan_kernel"][-1] == "scan_exact_prog2_hint"
    if P >= 2:
        # (three hint bytes travel as four; the two-stage scan streams plane 0 alone and counts what its lanes ask
        # for beyond that -- the other planes of the items its first bound lets through -- in deep_units)
        stream_bytes_per_item = ((2 if P >= 4 else 1) if two_stage else P - 1) * 8 * W + (4 if P == 4 else P - 1) + (1 if two_stage else 0)
        bytes_read = last_items * stream_bytes_per_item + (last_items // 256) * 4 + deep_bytes
    else:
        stream_bytes_per_item = bytes_per_item
        bytes_read = last_items * bytes_per_item
    achieved_gbs = bytes_read / (scan_avg_ms * 1e-3) / 1e9
    all_planes_gbs = last_items * bytes_per_item / (scan_avg_ms * 1e-3) / 1e9
    log(f"Q=1: {ms_per_step:.3f} ms/step, p50 {np.percentile(r1['per_step_ms'], 50):.3f} ms, "
        f"scan kernel {scan_avg_ms:.3f} ms -> {achieved_gbs:.0f} GB/s read "
        f"({bytes_read / last_items:.2f} B/item; {all_planes_gbs:.0f} GB/s if every plane counted)")

    out = {
        "metric": "candidates scored+selected/sec and p50 query latency at 1B items, k=1000",
        "value": value,
        "unit": "candidates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle": {"seconds": args.settle_seconds, "searches": settled,
                   "note": "untimed one-query searches between the corpus build and the warm-up steps (set-up): the first 0.2 s "
                           "of searches after the build run about 4 % slower than the rate they settle at"},
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u64 xor/popcount + f32 combine",
        "data": "synthetic",
        "config": {
            "workload": f"{N} items, d={d}, {P} bit-planes + {P} fp32 scales ({bytes_per_item} B/item), "
                        f"{args.clusters}-cluster Gaussian mixture sigma={args.sigma}, exact top-{k}, 1 query per step",
            "n_items": N, "dim": d, "n_planes": P, "k": k, "queries_per_step": 1, "mode": "exact",
        },
        "p50_ms": float(np.percentile(r1["per_step_ms"], 50)),
        "p95_ms": float(np.percentile(r1["per_step_ms"], 95)),
        "gpu_ms_per_search": float(r1["total_gpu_ms"].mean()) if r1["total_gpu_ms"].size else None,
        "levels": st["n_levels"],
        "candidates_max": st["candidates_max"],
        "select_ms_total": float(r1["select_ms"].mean()) if r1["select_ms"].size else None,
        "last_search_level_ms": {"scan": st["scan_ms"], "select": st["select_ms"]},
        "roofline": {
            "kernel": (st["scan_kernel"][-1] if st["n_levels"] else "scan_exact") + " (finest level)",
            "bound": "hbm",
            "achieved": achieved_gbs,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved_gbs / HBM_PEAK_GBS,
            "traffic": None,
            "bytes_per_launch": bytes_read,
            "bytes_per_item_streamed": stream_bytes_per_item,
            "rows_with_items_read_in_full": deep_avg,
            "bytes_beyond_the_stream": deep_bytes,
            "rows": -(-last_items // 256),
            "bytes_per_launch_all_planes": last_items * bytes_per_item,
            "gbs_if_all_planes_counted": all_planes_gbs,
            "kernel_ms": scan_avg_ms,
            "launches": "kernel_ms, bytes_per_launch and rows cover the last level of the plan: one launch of the kernel, or, in the "
                        "steps where the library takes that level in two parts, its two launches together (same bytes, times added)",
            "steps_with_the_level_in_two_launches": r1["split_steps"],
            "grid_blocks": st["grid_blocks"],
            "algorithmic_bytes_per_item": bytes_per_item,
            "algorithmic_bytes_per_launch": last_items * bytes_per_item,
            "frac_of_algorithmic": all_planes_gbs / HBM_PEAK_GBS,
            "note": "achieved/frac price the bytes this kernel MOVES (it prunes: of every item it streams plane 0 and one-byte "
                    "copies of its scales; the other planes are read, lane by lane, only for items whose upper bound "
                    "reaches the threshold, and the fp32 scales only for those that pass a second bound), not the method's %d B/item; "
                    "frac_of_algorithmic prices all %d B/item over the same time and can exceed 1 for that reason. "
                    "The share pruned depends on the corpus: on one with no cluster structure the library falls back "
                    "to the all-planes scan, whose fraction is worst_case." % (bytes_per_item, bytes_per_item),
            "worst_case": None,
        },
    }
    if st["n_levels"]:
        out["scan_kernel_per_level"] = st["scan_kernel"]

    # ---------------- the same searches with every plane of every item read (progressive scan off)
    if P >= 2 and want("all_planes"):
        rbe.rbe_debug_set_progressive(ix, False)
        steps_a = max(2, args.steps // 4)
        ra = timed_searches(rbe, torch, ix, qp1, qs1, 1, k, steps_a, args.warmup)
        rbe.rbe_debug_set_progressive(ix, True)
        a_scan = float(ra["scan_ms"].mean())
        a_gbs = last_items * bytes_per_item / (a_scan * 1e-3) / 1e9
        same = all(np.array_equal(x, y) for x, y in zip(ra["ids"], r1["ids"]))
        out["all_planes_scan"] = {
            "steps": steps_a, "ms_per_step": ra["wall_s"] * 1e3 / steps_a, "scan_kernel_ms": a_scan,
            "hbm_gbs": a_gbs, "hbm_frac": a_gbs / HBM_PEAK_GBS, "bytes_per_launch": last_items * bytes_per_item,
            "same_ids_as_progressive": bool(same),
        }
        out["roofline"]["worst_case"] = {"kernel": "scan_exact (finest level, every plane of every item read)",
                                         "achieved": a_gbs, "frac": a_gbs / HBM_PEAK_GBS, "kernel_ms": a_scan,
                                         "ms_per_step": ra["wall_s"] * 1e3 / steps_a}
        log(f"Q=1, every plane read: {ra['wall_s'] * 1e3 / steps_a:.3f} ms/step, scan kernel {a_scan:.3f} ms -> {a_gbs:.0f} GB/s, "
            f"same ids: {same}")

    # ---------------- the same searches on the one-stage progressive scan (planes 0 .. P-2 and their scale copies in
    # the stream): more bytes, moved at a higher rate, in more time
    if two_stage and want("all_planes"):
        rbe.rbe_debug_set_progressive(ix, 3)
        steps_o = max(2, args.steps // 2)
        ro = timed_searches(rbe, torch, ix, qp1, qs1, 1, k, steps_o, args.warmup)
        rbe.rbe_debug_set_progressive(ix, True)
        o_scan = float(ro["scan_ms"].mean())
        o_bytes = (last_items * ((P - 1) * 8 * W + (4 if P == 4 else P - 1)) + (last_items // 256) * 4
                   + float(ro["deep_units"].mean()) * 8.0)
        out["roofline"]["one_stage_scan"] = {
            "kernel": ro["stats"]["scan_kernel"][-1] + " (finest level; planes 0 .. P-2 streamed)", "kernel_ms": o_scan,
            "bytes_per_launch": o_bytes, "achieved": o_bytes / (o_scan * 1e-3) / 1e9, "frac": o_bytes / (o_scan * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "ms_per_step": ro["wall_s"] * 1e3 / steps_o,
            "same_ids": bool(all(np.array_equal(x, y) for x, y in zip(ro["ids"], r1["ids"]))),
            "note": "the two-stage scan asks for fewer bytes and needs less time, but its lane-wise reads bring whole lines, so "
                    "its fraction on the bytes asked for is the lower one",
        }
        log(f"Q=1, one-stage progressive scan: {ro['wall_s'] * 1e3 / steps_o:.3f} ms/step, scan kernel {o_scan:.3f} ms -> "
            f"{o_bytes / (o_scan * 1e-3) / 1e9:.0f} GB/s")

    # ---------------- near-lossless selector (Algorithm 1, queue length 1, I = 256) on the same queries
    if not args.no_nearlossless and want("near"):
        I = 256
        rn = timed_searches(rbe, torch, ix, qp1, qs1, 1, k, args.steps, args.warmup, rbe.RBE_SELECT_NEARLOSSLESS, I)
        recalls = [len(set(a[0].tolist()) & set(b[0].tolist()) - {-1}) / k for a, b in zip(rn["ids"], r1["ids"])]
        groups = -(-N // (256 * I)) * 256
        slots = groups * I
        # Appendix A: E[M]/N = (T/N) (1 - prod_{i<I} (1 - N/(C-i))) ~ 1 - (N-1)(I-1)/(2(C-1))
        predicted = 1.0 - (k - 1) * (I - 1) / (2.0 * (slots - 1))
        n_ms = rn["wall_s"] * 1e3 / args.steps
        out["near_lossless"] = {
            "group_size_I": I, "ms_per_step": n_ms, "p50_ms": float(np.percentile(rn["per_step_ms"], 50)),
            "value": N * args.steps / rn["wall_s"], "unit": "candidates/s",
            "scan_kernel_ms": float(rn["scan_ms"].mean()) if rn["scan_ms"].size else None,
            "recall_vs_exact_mean": float(np.mean(recalls)), "recall_vs_exact_min": float(np.min(recalls)),
            "recall_predicted_appendix_a": predicted, "queries": len(recalls),
        }
        out["near_lossless"]["scan_kernel_per_level"] = rn["stats"]["scan_kernel"]
        log(f"near-lossless I={I}: {n_ms:.3f} ms/step, recall {np.mean(recalls):.5f} (Appendix A: {predicted:.5f})")
        # the same searches on the scan that keeps one queue per thread as Algorithm 1 is written (every plane read)
        rbe.rbe_debug_set_nearlossless_path(ix, 1)
        steps_q = max(2, args.steps // 4)
        rq = timed_searches(rbe, torch, ix, qp1, qs1, 1, k, steps_q, args.warmup, rbe.RBE_SELECT_NEARLOSSLESS, I)
        rbe.rbe_debug_set_nearlossless_path(ix, 0)
        out["near_lossless"]["per_thread_queue_scan"] = {
            "steps": steps_q, "ms_per_step": rq["wall_s"] * 1e3 / steps_q,
            "scan_kernel_ms": float(rq["scan_ms"].mean()) if rq["scan_ms"].size else None,
            "same_ids": bool(all(np.array_equal(x, y) for x, y in zip(rq["ids"], rn["ids"])))}
        log(f"near-lossless I={I}, per-thread-queue scan: {rq['wall_s'] * 1e3 / steps_q:.3f} ms/step")
        # the same selector with priority queues of length 2 (Algorithm 1 leaves the length open)
        steps2 = max(2, args.steps // 2)
        rn2 = timed_searches(rbe, torch, ix, qp1, qs1, 1, k, steps2, args.warmup, rbe.RBE_SELECT_NEARLOSSLESS_Q2, I)
        rec2 = [len(set(a[0].tolist()) & set(b[0].tolist()) - {-1}) / k for a, b in zip(rn2["ids"], r1["ids"])]
        out["near_lossless_queue2"] = {
            "group_size_I": I, "ms_per_step": rn2["wall_s"] * 1e3 / steps2, "steps": steps2,
            "recall_vs_exact_mean": float(np.mean(rec2)), "recall_vs_exact_min": float(np.min(rec2)),
        }
        log(f"near-lossless I={I}, queue length 2: {rn2['wall_s'] * 1e3 / steps2:.3f} ms/step, recall {np.mean(rec2):.5f}")

    # ---------------- mixed workload: one query per call, a share of the queries far from every cluster (their
    # k-th best score is so low that the last level's bound prunes nothing and the scan reads every plane).  The
    # one thing a one-query search takes from earlier searches is whether its last level goes in one launch or two,
    # so the latency of the ordinary queries is reported for the mix, by class.
    if want("mixed"):
        n_mix, share = 200, 0.1
        rng_mix = np.random.default_rng(12345)
        far = rng_mix.random(n_mix) < share
        qn_p, qn_s = make_queries(rbe, rbe_synth, torch, centres, n_mix, args.sigma, P, 11)
        qf_p, qf_s = make_queries(rbe, rbe_synth, torch, centres, n_mix, 10.0, P, 12)      # sigma 10: no cluster left
        lat, rows_full, lv = [], [], []
        for i in range(n_mix):
            qp_i, qs_i = (qf_p, qf_s) if far[i] else (qn_p, qn_s)
            t0 = time.perf_counter()
            rbe.rbe_search(ix, qp_i[i:i + 1], qs_i[i:i + 1], k)
            lat.append((time.perf_counter() - t0) * 1e3)
            st = rbe.rbe_get_search_stats(ix)
            rows_full.append(st["deep_rows"]); lv.append(st["last_level_parts"])
        lat = np.array(lat); lv = np.array(lv)
        def dist(x):
            return {"n": int(x.size), "p50_ms": float(np.percentile(x, 50)), "p95_ms": float(np.percentile(x, 95)),
                    "p99_ms": float(np.percentile(x, 99)), "max_ms": float(x.max()), "mean_ms": float(x.mean())}
        out["mixed_workload"] = {"queries": n_mix, "share_far_from_every_cluster": share,
                                 "ordinary": dist(lat[~far][2:]), "far": dist(lat[far]),
                                 "searches_with_the_last_level_in_two_parts": int((lv == 2).sum())}
        rbe.rbe_debug_set_plan_split(ix, 0)          # forget what this leg taught the index
        log(f"mixed workload ({share:.0%} of {n_mix} queries far from every cluster): ordinary queries p50 "
            f"{out['mixed_workload']['ordinary']['p50_ms']:.3f} p95 {out['mixed_workload']['ordinary']['p95_ms']:.3f} p99 "
            f"{out['mixed_workload']['ordinary']['p99_ms']:.3f} ms; far queries p50 {out['mixed_workload']['far']['p50_ms']:.3f} ms; "
            f"{out['mixed_workload']['searches_with_the_last_level_in_two_parts']} searches took the last level in two parts")

    # ---------------- hybrid scoring: fp32 query against the binary items (the paper's model m_5)
    if not args.no_hybrid and want("hybrid"):
        xq = rbe_synth.vectors_torch(args.warmup + args.steps, centres, args.sigma, rbe_synth.SEED_QUERIES, 0).cpu().numpy()
        for s_ in range(args.warmup):
            rbe.rbe_search_float(ix, xq[s_:s_ + 1], k)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        h_scan, h_deep, h_units = [], [], []
        for s_ in range(args.warmup, args.warmup + args.steps):
            rbe.rbe_search_float(ix, xq[s_:s_ + 1], k)
            h_stats = rbe.rbe_get_search_stats(ix)
            h_scan.append(sum(h_stats["scan_ms"][-h_stats["last_level_parts"]:])); h_deep.append(h_stats["deep_rows"]); h_units.append(h_stats["deep_units"])
        torch.cuda.synchronize()
        h_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        # progressive like the binary-query scan: bytes read = streamed planes and scales + the last plane of some rows
        h_two = h_stats["scan_kernel"][-1] == "scan_exact_fq_prog2_hint"      # plane 0 and the copies of all scales in the stream
        h_bytes = (last_items * ((1 if h_two else P - 1) * 8 * W + (4 if P == 4 else P - 1) + (1 if h_two else 0))
                   + (last_items // 256) * 4 + float(np.mean(h_units)) * 8.0
                   if P >= 2 else last_items * bytes_per_item)
        h_gbs = h_bytes / (float(np.mean(h_scan)) * 1e-3) / 1e9
        out["hybrid_float_query"] = {"ms_per_step": h_ms, "value": N / (h_ms * 1e-3), "unit": "candidates/s",
                                     "scan_kernel_ms": float(np.mean(h_scan)), "hbm_gbs": h_gbs,
                                     "hbm_frac": h_gbs / HBM_PEAK_GBS, "bytes_per_launch": h_bytes,
                                     "rows_with_items_read_in_full": float(np.mean(h_deep)),
                                     "scan_kernel": h_stats["scan_kernel"][-1]}
        log(f"hybrid fp32 query: {h_ms:.3f} ms/step, scan kernel {np.mean(h_scan):.3f} ms -> {h_gbs:.0f} GB/s read")
        if args.batch >= 3:
            B = args.batch
            xb = rbe_synth.vectors_torch(B * 4, centres, args.sigma, rbe_synth.SEED_QUERIES, 5).cpu().numpy()
            rbe.rbe_search_float(ix, xb[:B], k)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for s_ in range(1, 4):
                rbe.rbe_search_float(ix, xb[s_ * B:(s_ + 1) * B], k)
            torch.cuda.synchronize()
            hb_ms = (time.perf_counter() - t0) * 1e3 / 3
            out["hybrid_float_query"]["batch"] = {"queries_per_step": B, "ms_per_step": hb_ms,
                                                  "value": N * B / (hb_ms * 1e-3), "unit": "candidates/s"}
            log(f"hybrid fp32 queries, Q={B}: {hb_ms:.3f} ms/step")

    # ---------------- batch leg
    # ---------------- a few queries per call (below the batch size from which the matrix cores take over): the
    # XOR/popcount scans with a loop over the queries, two-stage from three planes on
    if want("small_batch"):
        sb = {}
        for B in (2, 4):
            steps_s, warm_s = 12, 6
            qps, qss = make_queries(rbe, rbe_synth, torch, centres, (warm_s + steps_s) * B, args.sigma, P, 5)
            rs = timed_searches(rbe, torch, ix, qps, qss, B, k, steps_s, warm_s)
            s_ms = rs["wall_s"] * 1e3 / steps_s
            s_scan = float(rs["scan_ms"].mean()) if rs["scan_ms"].size else float("nan")
            sb[f"Q{B}"] = {"queries_per_step": B, "steps": steps_s, "ms_per_step": s_ms,
                           "p50_ms": float(np.percentile(rs["per_step_ms"], 50)),
                           "value": N * B / (s_ms * 1e-3), "unit": "candidates/s",
                           "last_level_ms": s_scan, "last_level_kernel": rs["stats"]["scan_kernel"][-1]}
            log(f"Q={B}: {s_ms:.3f} ms/step, last level {s_scan:.3f} ms on {rs['stats']['scan_kernel'][-1]}")
        out["small_batch"] = sb

    if args.batch > 0 and want("batch"):
        B = args.batch
        bw = 16      # (the first dozen batch calls after the one-query legs run up to 15 % slower: the clock settles)
        qpb, qsb = make_queries(rbe, rbe_synth, torch, centres, (bw + args.batch_steps) * B, args.sigma, P, 1)
        rb = timed_searches(rbe, torch, ix, qpb, qsb, B, k, args.batch_steps, bw)
        b_ms = rb["wall_s"] * 1e3 / args.batch_steps
        b_scan = float(rb["scan_ms"].mean()) if rb["scan_ms"].size else float("nan")
        b_items = rb["last_items"]
        matrix_cores = B >= 5 and W <= 2     # the library's own choice of kernel for a batch (binary queries, general scales)
        # bytes the finest-level launches ask for: whole rows, or (up to 16 queries per launch, an index with one-byte
        # scale copies) planes 0 .. P-2 and the copies, plus what the second looks read
        b_deep = float(rb["deep_units"].mean()) * 8.0 if rb["deep_units"].size else 0.0
        b_bytes = b_items * (8 * W * (P - 1) + (P - 1)) + b_deep if (matrix_cores and b_deep > 0) else b_items * bytes_per_item
        if matrix_cores:
            # dense contraction [B x d] . [d x items] per corpus plane (one eight-bit integer per query component:
            # the contraction filters, survivors are rescored bitwise).  `achieved` prices the whole contraction;
            # the kernel issues less of it -- the last plane is contracted only for the blocks of items that the
            # other planes cannot rule out -- and more of it, by padding the batch to a multiple of 16 queries.
            flops = 2.0 * B * b_items * d * P
            issued = 2.0 * 16 * -(-B // 16) * b_items * d * (P - 1 if P >= 2 else P)
            ach = flops / (b_scan * 1e-3) / 1e12
            roof = {"kernel": "scan_batch_mfma (finest level)", "bound": "mfma", "achieved": ach,
                    "peak": MFMA_I8_PEAK_TOPS, "unit": "TOP/s", "frac": ach / MFMA_I8_PEAK_TOPS,
                    "frac_of_f16_peak": ach / MFMA_F16_PEAK_TFLOPS,
                    "kernel_ms": b_scan, "flops_per_pair": 2 * d * P,
                    "issued_tops_first_look": issued / (b_scan * 1e-3) / 1e12, "traffic": None,
                    "hbm_gbs": b_bytes / (b_scan * 1e-3) / 1e9, "bytes_per_launch": b_bytes,
                    "lean_stream": bool(b_deep > 0)}
        else:
            lane_ops = lane_ops_per_pair(W, P, P) * B * b_items
            ach = lane_ops / (b_scan * 1e-3) / 1e12
            roof = {"kernel": "scan_exact_batch_prog (finest level)" if P >= 2 else "scan_exact (finest level)", "bound": "alu", "achieved": ach,
                    "peak": VALU_PEAK_TLANEOPS, "unit": "T lane-ops/s", "frac": ach / VALU_PEAK_TLANEOPS,
                    "kernel_ms": b_scan, "lane_ops_per_pair": lane_ops_per_pair(W, P, P), "traffic": None,
                    "note": "the op model prices every plane of every pair; the progressive scan skips the last "
                            "plane of most pairs, so this figure can exceed the modelled peak",
                    "hbm_gbs": b_items * bytes_per_item / (b_scan * 1e-3) / 1e9}
        out["batch"] = {
            "queries_per_step": B, "steps": args.batch_steps, "warmup": bw, "ms_per_step": b_ms,
            "p50_ms": float(np.percentile(rb["per_step_ms"], 50)),
            "value": N * B * args.batch_steps / rb["wall_s"], "unit": "candidates/s",
            "dtype": "i8 x i8 -> i32 filter, u64 xor/popcount + f32 scores" if matrix_cores else "u64 xor/popcount + f32",
            "last_search_level_ms": {"scan": rb["stats"]["scan_ms"], "select": rb["stats"]["select_ms"]},
            "gpu_ms_per_search": float(rb["total_gpu_ms"].mean()) if rb["total_gpu_ms"].size else None,
            "roofline": roof,
        }
        log(f"Q={B}: {b_ms:.3f} ms/step (per step {np.round(rb['per_step_ms'], 2).tolist()}, "
            f"{rb['fallbacks']} on the bounded-segment path), scan kernel {b_scan:.3f} ms")
        if matrix_cores and want("batch_popcount"):
            # the same calls on the XOR/popcount kernel (what one query uses), against the vector-ALU roofline
            # (progressive scan off for the roofline figure: the 58-op model prices every plane of every pair)
            rbe.rbe_debug_set_batch_path(ix, 3)                 # matrix cores with half operands (v_mfma_f32_16x16x32_f16)
            rh = timed_searches(rbe, torch, ix, qpb, qsb, B, k, args.batch_steps, bw)
            out["batch"]["half_operands"] = {"ms_per_step": rh["wall_s"] * 1e3 / args.batch_steps, "scan_kernel_ms": float(rh["scan_ms"].mean()),
                                             "same_ids": bool(all(np.array_equal(x, y) for x, y in zip(rh["ids"], rb["ids"])))}
            log(f"Q={B}, matrix cores with half operands: {rh['wall_s'] * 1e3 / args.batch_steps:.3f} ms/step, scan kernel {rh['scan_ms'].mean():.3f} ms")
            rbe.rbe_debug_set_batch_path(ix, 1)
            steps_v = max(2, args.batch_steps // 2)
            rvp = timed_searches(rbe, torch, ix, qpb, qsb, B, k, steps_v, 1)
            rbe.rbe_debug_set_progressive(ix, False)
            rv = timed_searches(rbe, torch, ix, qpb, qsb, B, k, steps_v, 1)
            rbe.rbe_debug_set_progressive(ix, True)
            rbe.rbe_debug_set_batch_path(ix, 0)
            v_ms = rv["wall_s"] * 1e3 / steps_v
            v_scan = float(rv["scan_ms"].mean())
            v_ach = lane_ops_per_pair(W, P, P) * B * rv["last_items"] / (v_scan * 1e-3) / 1e12
            out["batch_popcount_kernel"] = {
                "queries_per_step": B, "steps": steps_v, "ms_per_step": v_ms,
                "ms_per_step_progressive": rvp["wall_s"] * 1e3 / steps_v,
                "scan_kernel_ms_progressive": float(rvp["scan_ms"].mean()),
                "p50_ms": float(np.percentile(rv["per_step_ms"], 50)),
                "gpu_ms_per_search": float(rv["total_gpu_ms"].mean()) if rv["total_gpu_ms"].size else None,
                "last_search_level_ms": {"scan": rv["stats"]["scan_ms"], "select": rv["stats"]["select_ms"]},
                "value": N * B / (v_ms * 1e-3), "unit": "candidates/s", "dtype": "u64 xor/popcount + f32",
                "roofline": {"kernel": "scan_exact (finest level)", "bound": "alu", "achieved": v_ach,
                             "peak": VALU_PEAK_TLANEOPS, "unit": "T lane-ops/s", "frac": v_ach / VALU_PEAK_TLANEOPS,
                             "kernel_ms": v_scan, "lane_ops_per_pair": lane_ops_per_pair(W, P, P), "traffic": None},
            }
            log(f"Q={B}, XOR/popcount kernel, progressive: {rvp['wall_s'] * 1e3 / steps_v:.3f} ms/step, scan kernel {rvp['scan_ms'].mean():.3f} ms")
            log(f"Q={B}, XOR/popcount kernel, every plane: {v_ms:.3f} ms/step (per step {np.round(rv['per_step_ms'], 2).tolist()}), scan kernel {v_scan:.3f} ms "
                f"-> {v_ach:.1f} T lane-ops/s")

    # ---------------- what instruction issue alone allows the two batch kernels (no memory traffic: every tile is
    # gone over 200 times from registers / LDS), as the ceiling their rooflines are priced against
    if args.batch >= 3 and want("batch"):
        B = args.batch
        qpi, qsi = make_queries(rbe, rbe_synth, torch, centres, B, args.sigma, P, 9)
        ceil = {}
        for kernel, name in ((0, "scan_exact"), (1, "scan_batch_mfma")):
            if kernel == 1 and not (B >= 5 and W <= 2):
                continue
            rbe.rbe_debug_issue_rate(ix, qpi, qsi, kernel, 20)                      # warm-up
            runs = [rbe.rbe_debug_issue_rate(ix, qpi, qsi, kernel, 200) for _ in range(3)]
            ms_i, pairs_i = min(runs)
            ceil[name] = {"ms": ms_i, "pairs": pairs_i, "pairs_per_s": pairs_i / (ms_i * 1e-3)}
        if "scan_exact" in ceil:
            c0 = ceil["scan_exact"]
            c0["lane_ops_per_pair"] = lane_ops_per_pair(W, P, P)
            c0["t_lane_ops_per_s"] = c0["pairs_per_s"] * c0["lane_ops_per_pair"] / 1e12
            c0["modelled_peak_t_lane_ops_per_s"] = VALU_PEAK_TLANEOPS
            log(f"issue ceiling, XOR/popcount batch scan: {c0['t_lane_ops_per_s']:.2f} T lane-ops/s "
                f"({c0['pairs_per_s'] / 1e9:.1f} G pairs/s; modelled {VALU_PEAK_TLANEOPS:.2f})")
            if "batch_popcount_kernel" in out:
                rf = out["batch_popcount_kernel"]["roofline"]
                rf["issue_ceiling_t_lane_ops_per_s"] = c0["t_lane_ops_per_s"]
                rf["frac_of_issue_ceiling"] = rf["achieved"] / c0["t_lane_ops_per_s"]
        if "scan_batch_mfma" in ceil:
            c1 = ceil["scan_batch_mfma"]
            c1["tflops_algorithmic"] = c1["pairs_per_s"] * 2 * d * P / 1e12
            log(f"issue ceiling, matrix-core scan (first look): {c1['pairs_per_s'] / 1e9:.1f} G pairs/s = "
                f"{c1['tflops_algorithmic']:.0f} TOP/s algorithmic")
            if "batch" in out and out["batch"]["roofline"].get("bound") == "mfma":
                rf = out["batch"]["roofline"]
                rf["issue_ceiling_tflops"] = c1["tflops_algorithmic"]
                rf["frac_of_issue_ceiling"] = rf["achieved"] / c1["tflops_algorithmic"]
        out["issue_ceilings"] = ceil

    # ---------------- CPU baseline: the oracle, as it stands, on a bounded sample: one thread, then one thread per
    # host core over disjoint item ranges (the oracle's own code is unchanged and single-threaded)
    if cpu_items > 0:
        import oracle
        nq = min(args.cpu_sample_queries, n_q1)
        t0 = time.perf_counter()
        single = [oracle.topk(host_planes, host_scales, qp1[i], qs1[i], k) for i in range(nq)]
        dt = time.perf_counter() - t0
        n_threads = max(1, min(16, os.cpu_count() or 1))      # a one-GPU machine has a share of 16 host cores
        t0 = time.perf_counter()
        multi = [oracle_all_cores(oracle, np, host_planes, host_scales, qp1[i], qs1[i], k, n_threads) for i in range(nq)]
        dt_all = time.perf_counter() - t0
        agree = all(np.array_equal(a[0], b[0]) for a, b in zip(single, multi))
        out["cpu_baseline"] = {
            "value": cpu_items * nq / dt_all, "unit": "candidates/s", "cores": n_threads, "kind": "oracle",
            "sample": f"first {cpu_items} items of the same corpus x {nq} of the same queries, exact top-{k}: "
                      f"{dt_all:.1f} s with one oracle call per host thread over disjoint item ranges "
                      f"({n_threads} threads), {dt:.1f} s single-threaded",
            "single_thread": {"value": cpu_items * nq / dt, "unit": "candidates/s", "cores": 1, "seconds": dt},
            "all_cores_seconds": dt_all, "same_ids_as_single_thread": bool(agree),
            "host_cpus": os.cpu_count(),
        }
        log(f"oracle: {cpu_items * nq / dt / 1e6:.1f} M candidates/s on 1 core ({dt:.1f}s), "
            f"{cpu_items * nq / dt_all / 1e6:.1f} M candidates/s on {n_threads} threads ({dt_all:.1f}s)")

    rbe.rbe_free(ix)
    ix = None
    host_planes = host_scales = None
    if args.calibrate_copy > 0:
        calibrate(out, args, rbe, torch)
    extra_legs(out, args, want, rbe, rbe_synth, torch, np)
    out["roofline"]["traffic"] = measured_traffic(out["config"]["workload"])
    out["roofline"]["traffic_source"] = ("profiles/scan_exact_1e9_d64_p3_q1.md: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE of "
                                         "this kernel on this workload, scaled by the plain-copy yardstick; not measured in this run")
    if out["roofline"]["traffic"] and out["roofline"].get("kernel_ms"):
        # what the memory system moved for those bytes (the lane-wise reads bring whole lines), over this run's time
        t_gbs = out["roofline"]["traffic"] / (out["roofline"]["kernel_ms"] * 1e-3) / 1e9
        out["roofline"]["traffic_gbs"] = t_gbs
        out["roofline"]["traffic_frac"] = t_gbs / HBM_PEAK_GBS
    print(json.dumps(out), flush=True)


def calibrate(out, args, rbe, torch):
    """Yardsticks for hardware-counter readings and for the practical read ceiling of the box."""
    nbytes = args.calibrate_copy << 20
    src = torch.full((nbytes // 4,), 1.0, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    rbe.rbe_debug_copy(dst, src)
    ev0.record()
    for _ in range(5):
        rbe.rbe_debug_copy(dst, src)
    ev1.record()
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / 5
    out["calib_copy"] = {"bytes_read": nbytes, "bytes_written": nbytes, "kernel_ms": ms,
                         "gbs_read_plus_write": 2 * nbytes / (ms * 1e-3) / 1e9}
    log(f"calib_copy {args.calibrate_copy} MiB: {ms:.3f} ms -> {2 * nbytes / (ms * 1e-3) / 1e9:.0f} GB/s (r+w)")
    # read-only yardstick over a buffer several times the 256 MB last-level cache
    del dst
    big = torch.full((max(nbytes, 16 << 30) // 4,), 1.0, dtype=torch.float32, device="cuda:0")
    sink = torch.empty(8 << 20, dtype=torch.uint8, device="cuda:0")
    rbe.rbe_debug_read(big, sink)
    ev0.record()
    for _ in range(5):
        rbe.rbe_debug_read(big, sink)
    ev1.record()
    torch.cuda.synchronize()
    rms = ev0.elapsed_time(ev1) / 5
    rbytes = big.numel() * 4
    out["calib_read"] = {"bytes_read": rbytes, "kernel_ms": rms, "gbs_read": rbytes / (rms * 1e-3) / 1e9}
    log(f"calib_read {rbytes >> 20} MiB: {rms:.3f} ms -> {rbytes / (rms * 1e-3) / 1e9:.0f} GB/s")



def extra_legs(out, args, want, rbe, rbe_synth, torch, np):
    """Legs on corpora of their own: the paper's operating point and configurations 3 and 5 of the workload table."""
    k = args.k
    n_q1 = args.warmup + args.steps
    # ---------------- the paper's own operating point: 2 keyword bits, 3 query bits per dimension,
    # residual weights 2^-t by shift-adds, one stored inverse norm per keyword (20 B/item)
    if not args.no_paper_point and want("paper"):
        Np, Pk, Pq = args.paper_items, 2, 3
        ixp, centres_p, _, _ = build_corpus(rbe, rbe_synth, torch, Np, 64, Pk, args.clusters, args.sigma,
                                            args.chunk_items, 0, rbe.RBE_DYADIC | rbe.RBE_COSINE)
        rbe.rbe_set_profiling(ixp, True)
        settle(rbe, rbe_synth, torch, ixp, centres_p, args.sigma, Pq, k, args.settle_seconds, binary_scales=False)
        qpp, _ = make_queries(rbe, rbe_synth, torch, centres_p, n_q1, args.sigma, Pq, 2)
        rp = timed_searches(rbe, torch, ixp, qpp, None, 1, k, args.steps, args.warmup)
        rpn = timed_searches(rbe, torch, ixp, qpp, None, 1, k, args.steps, args.warmup, rbe.RBE_SELECT_NEARLOSSLESS, 256)
        p_items = rp["last_items"]
        p_scan = float(rp["scan_ms"].mean())
        p_deep = float(rp["deep_rows"].mean()) if rp["deep_rows"].size else 0.0
        # plane 0 of every item, one fp32 per row, and what the lanes asked for beyond that (plane 1 + inverse norm)
        p_bytes = p_items * 8 + (p_items // 256) * 4 + (float(rp["deep_units"].mean()) * 8.0 if rp["deep_units"].size else 0.0)
        p_gbs = p_bytes / (p_scan * 1e-3) / 1e9
        rec = [len(set(a[0].tolist()) & set(b[0].tolist()) - {-1}) / k for a, b in zip(rpn["ids"], rp["ids"])]
        out["paper_operating_point"] = {
            "workload": f"{Np} items (136*136 blocks x 256 threads x 256 keywords), d=64, 2 keyword planes + 1 fp32 inverse "
                        f"norm (20 B/item), 3 query planes, dyadic weights, top-{k}, 1 query per step",
            "exact": {"ms_per_step": rp["wall_s"] * 1e3 / args.steps, "p50_ms": float(np.percentile(rp["per_step_ms"], 50)),
                      "scan_kernel_ms": p_scan, "hbm_gbs": p_gbs, "hbm_frac": p_gbs / HBM_PEAK_GBS,
                      "bytes_per_launch": p_bytes, "rows_with_items_read_in_full": p_deep, "rows": -(-p_items // 256),
                      "gbs_if_all_planes_counted": p_items * 20 / (p_scan * 1e-3) / 1e9},
            "near_lossless_I256": {"ms_per_step": rpn["wall_s"] * 1e3 / args.steps,
                                   "p50_ms": float(np.percentile(rpn["per_step_ms"], 50)),
                                   "recall_vs_exact_mean": float(np.mean(rec))},
            "paper": {"avg_latency_ms": 31.17, "hardware": "4 x GeForce GTX 1080, 1.2e9 keywords, recall@1000 99.99%"},
        }
        log(f"paper point: exact {rp['wall_s'] * 1e3 / args.steps:.3f} ms/step ({p_gbs:.0f} GB/s), "
            f"near-lossless {rpn['wall_s'] * 1e3 / args.steps:.3f} ms/step, recall {np.mean(rec):.5f}")
        if args.batch >= 7:
            B = args.batch
            qpb, _ = make_queries(rbe, rbe_synth, torch, centres_p, (16 + args.batch_steps) * B, args.sigma, Pq, 3)
            rpb = timed_searches(rbe, torch, ixp, qpb, None, B, k, args.batch_steps, 16)
            pb_scan = float(rpb["scan_ms"].mean())
            pb_items = rpb["last_items"]
            pb_ms = rpb["wall_s"] * 1e3 / args.batch_steps
            pb_ach = 2.0 * B * pb_items * 64 * Pk / (pb_scan * 1e-3) / 1e12
            out["paper_operating_point"]["batch"] = {
                "queries_per_step": B, "ms_per_step": pb_ms, "value": Np * B / (pb_ms * 1e-3), "unit": "candidates/s",
                "dtype": "i8 x i8 -> i32 (3 query and 2 keyword planes with dyadic weights are exact in eight-bit integers)",
                "roofline": {"kernel": "scan_batch_mfma (finest level)", "bound": "mfma", "achieved": pb_ach,
                             "peak": MFMA_I8_PEAK_TOPS, "unit": "TOP/s", "frac": pb_ach / MFMA_I8_PEAK_TOPS,
                             "kernel_ms": pb_scan, "traffic": None,
                             "hbm_gbs": pb_items * 20 / (pb_scan * 1e-3) / 1e9},
            }
            log(f"paper point Q={B}: {pb_ms:.3f} ms/step, scan kernel {pb_scan:.3f} ms")
        rbe.rbe_free(ixp)

    # ---------------- configuration 5: 1e9 near-duplicate items (sigma 0.05), 8 queries per call, k = 4000:
    # stresses pruning (cluster-mates share bit planes and have nearly equal scales) and the merge
    if not args.no_config5 and want("config5"):
        out["config5_near_duplicates"] = config_leg(
            rbe, rbe_synth, torch, np, args, N=1_000_000_000, d=64, P=3, clusters=4096, sigma=0.05, Q=8, k=4000,
            seed_chunk=11, label="config 5", near_lossless=True)
    # ---------------- configuration 3: 1e8 items, d = 128, 4 planes (80 B/item), 64 queries per call, k = 1000
    if not args.no_config3 and want("config3"):
        out["config3_d128_4planes"] = config_leg(
            rbe, rbe_synth, torch, np, args, N=100_000_000, d=128, P=4, clusters=4096, sigma=0.3, Q=64, k=1000,
            seed_chunk=12, label="config 3", near_lossless=False)


def config_leg(rbe, rbe_synth, torch, np, args, *, N, d, P, clusters, sigma, Q, k, seed_chunk, label, near_lossless):
    """One more configuration of the workload table on a corpus of its own: Q queries per call, exact top-k, timed
    like the headline steps (different queries per call, results in host memory), with the roofline figures of its
    finest-level scan; optionally the near-lossless selector's time and recall against the exact result."""
    W = d // 64
    ix, centres, _, _ = build_corpus(rbe, rbe_synth, torch, N, d, P, clusters, sigma, args.chunk_items, 0)
    rbe.rbe_set_profiling(ix, True)
    settle(rbe, rbe_synth, torch, ix, centres, sigma, P, k, args.settle_seconds)
    steps, warm = args.config_steps, 16
    qp, qs = make_queries(rbe, rbe_synth, torch, centres, (warm + steps) * Q, sigma, P, seed_chunk)
    r = timed_searches(rbe, torch, ix, qp, qs, Q, k, steps, warm)
    ms = r["wall_s"] * 1e3 / steps
    st = r["stats"]
    leg = {
        "workload": f"{N} items, d={d}, {P} bit-planes + {P} fp32 scales ({P * (8 * W + 4)} B/item), {clusters}-cluster "
                    f"Gaussian mixture sigma={sigma}, exact top-{k}, {Q} queries per call",
        "queries_per_step": Q, "k": k, "steps": steps, "warmup": warm, "ms_per_step": ms,
        "p50_ms": float(np.percentile(r["per_step_ms"], 50)), "value": N * Q * steps / r["wall_s"], "unit": "candidates/s",
        "levels": st["n_levels"], "scan_kernel_per_level": st["scan_kernel"], "candidates_max": st["candidates_max"],
        "last_search_level_ms": {"scan": st["scan_ms"], "select": st["select_ms"]},
        "gpu_ms_per_search": float(r["total_gpu_ms"].mean()) if r["total_gpu_ms"].size else None,
        "fallbacks": r["fallbacks"],
        "roofline": finest_level_roofline(np, r, W, P, Q, d, st["scan_kernel"][-1]) if st["n_levels"] and r["scan_ms"].size else None,
    }
    log(f"{label}: Q={Q}, k={k}: {ms:.3f} ms/step (per step {np.round(r['per_step_ms'], 2).tolist()}), "
        f"levels {st['scan_kernel']}, scan {np.round(st['scan_ms'], 3).tolist()} ms, select {np.round(st['select_ms'], 3).tolist()} ms")
    if near_lossless:
        I = 256
        rn = timed_searches(rbe, torch, ix, qp, qs, Q, k, steps, warm, rbe.RBE_SELECT_NEARLOSSLESS, I)
        rec = [len(set(a[q].tolist()) & set(b[q].tolist()) - {-1}) / k for a, b in zip(rn["ids"], r["ids"]) for q in range(Q)]
        slots = -(-N // (256 * I)) * 256 * I
        predicted = 1.0 - (k - 1) * (I - 1) / (2.0 * (slots - 1))      # Appendix A, expected recall
        leg["near_lossless"] = {"group_size_I": I, "ms_per_step": rn["wall_s"] * 1e3 / steps,
                                "recall_vs_exact_mean": float(np.mean(rec)), "recall_vs_exact_min": float(np.min(rec)),
                                "recall_predicted_appendix_a": predicted, "queries": len(rec)}
        log(f"{label}: near-lossless I={I}: {rn['wall_s'] * 1e3 / steps:.3f} ms/step, recall {np.mean(rec):.5f} "
            f"(Appendix A: {predicted:.5f})")
    rbe.rbe_free(ix)
    torch.cuda.empty_cache()
    return leg


if __name__ == "__main__":
    main()
