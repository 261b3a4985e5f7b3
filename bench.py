#!/usr/bin/env python3
"""Decode-step sparse-attention benchmark on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload batched_16] [--no-per-config]

One step = one decode step of one layer: append the new token's key/value (Session.update), then
the sparse-attention query (Session.attention): score every cached key, select top-k (or DIPR),
gather the selected value rows, softmax-weighted sum, merge.  Both through one alaya_decode_step
call (--separate-append: through alaya_append_kv_step and alaya_sparse_attn, one launch more).
Inputs are resident in HBM before the timed region.  Prints ONE JSON line whose headline fields
(value, ms_per_step, roofline, cpu_baseline, config) are those of --workload - by default the
largest configuration, 16 requests of 32K..256K tokens in one call - and whose per_config block
repeats the measurement on the other configurations (128K, 256K at beta = 2 and 4, 1M).

  value       keys scored per second over the whole step  (a key-score = one (query head, token) pair)
  roofline    the main scoring kernel against the 8 TB/s HBM peak.  Algorithmic bytes per launch =
              256 B (one bf16 K row, read once) x the K rows that the launch has to read: those of the
              call (tokens rounded up to pages x KV heads) less the pages that the sample pass has
              scored already and hands over as scores (every 8th to 32nd page); the handed-over scores
              and the few survivors it writes are not counted.  Duration = the kernel's
              average over a profiled repeat of the timed loop, taken with HIP events attached to
              the kernel's own dispatch on the launch stream (the library's profiling mode; events
              between kernels would lengthen the timed steps themselves, so the timed loop runs
              without them).  When the keys of the call are smaller than 512 MB they partly survive
              in the 256 MB last-level cache from step to step, which no model with many layers
              would see: `frac` is then taken from the cold loop (cache flushed before every step)
              and the warm figure is reported beside it.  scoring_pass_frac = every K row of the
              call, once, over sample pass + bound + main pass.
  gather      the gather + attend kernel: one V row (256 B) per selected (head, token), same clock
  cpu_baseline  the CPU oracle on the same step, on this host's cores (a reported baseline only)
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

HBM_PEAK_GBS = 8000.0
LLC_BYTES = 512e6          # below this the keys of a call partly stay in the last-level cache


def measure(name, args, steps, warmup, cold_steps, cpu_baseline, beta=None, dense=True, coarse_div=0):
    """One workload: timed loop, profiled loop, cold-cache loop, optional oracle timing.  Returns a dict.
    coarse_div > 0: the top-k query goes through the coarse index with 1 / coarse_div of each request's pages
    per head (the cache then keeps block representatives, and the append is not fused into the query)."""
    import numpy as np
    import torch

    import paper_2504_10326_amd as A
    import workloads as wl

    w = wl.config(name)
    beta = args.beta if beta is None else beta
    t0 = time.time()
    g = wl.generate(w)
    print(f"[bench] generated {w.name}: {w.total_tokens} tokens in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)

    # Each step appends one token per request, so leave room for every step of all passes.
    extra = 2 * (warmup + steps) + cold_steps + 16
    n_phys = g["n_phys_pages"] + w.batch * ((extra + 63) // 64 + 1)
    order = g["page_order"]
    if len(order) < n_phys:
        order = np.concatenate([order, np.arange(len(order), n_phys, dtype=np.int32)])
    c = A.Cache(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, max_seqs=w.batch, max_batch=w.batch,
                max_tokens_per_seq=max(w.lens) + extra, max_batch_tokens=w.total_tokens + w.batch * extra,
                n_phys_pages=n_phys, phys_page_order=order if w.permute_pages else None, coarse_index=coarse_div > 0)
    tdt = torch.bfloat16

    def dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).cuda().view(tdt)

    # The cache starts one token short; the first step's append brings it to the stated length.
    for r, n in enumerate(w.lens):
        c.append_kv(r, dev(g["K"][r][:n - 1]), dev(g["V"][r][:n - 1]))
    q = dev(g["q"])
    # What the steps append: the workload's own last token first, then fresh random rows - a new
    # key and value for every step and request, as a decoding model would emit them.
    n_new = extra + 1
    ek = np.empty((n_new, w.batch, w.n_kv_heads, w.head_dim), dtype=np.uint16)
    ev = np.empty_like(ek)
    for r in range(w.batch):
        k2, v2 = wl.extra_tokens(w, r, n_new - 1)
        ek[0, r], ev[0, r] = g["K"][r][w.lens[r] - 1], g["V"][r][w.lens[r] - 1]
        ek[1:, r], ev[1:, r] = k2, v2
    step_k, step_v = dev(ek), dev(ev)                        # [step][batch][H_kv][d]
    cursor = [0]
    seqs = list(range(w.batch))
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    window = tuple(int(x) for x in args.window.split(","))
    if w.mode == "topk":
        mode, kw = A.ALAYA_TOPK, dict(topk=list(w.topk), window=window)
        if coarse_div > 0:
            kw["coarse_pages"] = [max(1, (n + 63) // 64 // coarse_div) for n in w.lens]
    else:
        mode, kw = A.ALAYA_DIPR, dict(beta=[beta] * w.batch, window=window)
    c.set_tuning(args.pages_per_wave, args.attend_splits, 0, args.write_all_scores)
    torch.cuda.synchronize()

    if args.separate_append:
        def step():
            i = cursor[0] = cursor[0] + 1
            c.append_step(seqs, step_k[i - 1], step_v[i - 1])  # Session.update for the whole batch, one launch
            c.sparse_attn(seqs, q, mode, out=out, **kw)        # Session.attention
    else:
        def step():                                            # both in one call: the first scoring kernel
            i = cursor[0] = cursor[0] + 1                      # writes the new rows itself
            c.decode_step(seqs, step_k[i - 1], step_v[i - 1], q, mode, out=out, **kw)

    def run(n_steps):
        """n_steps steps bracketed by synchronisation; returns (seconds, key-scores, K rows scored)."""
        before = sum(c.seq_len(r) for r in seqs)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(n_steps):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t
        # step i (1-based) scores before + i * batch tokens in total
        toks = n_steps * before + w.batch * n_steps * (n_steps + 1) // 2
        return dt, w.n_q_heads * toks, w.n_kv_heads * toks

    run(warmup)
    c.debug_repairs()
    secs, keys, rows = run(steps)
    ms_per_step = secs / steps * 1e3
    repairs = c.debug_repairs()
    recall = None
    if coarse_div > 0:
        # what the approximation costs: the share of the exact query's tokens that the coarse query returns
        kmax = max(w.topk) + sum(window)
        ex = c.sparse_attn(seqs, q, mode, topk=list(w.topk), window=window, ids_stride=kmax)
        co = c.sparse_attn(seqs, q, mode, ids_stride=kmax, **kw)
        e_ids, c_ids, cnts = ex[1].cpu().numpy(), co[1].cpu().numpy(), ex[2].cpu().numpy()
        hits = sum(len(np.intersect1d(e_ids[r, h, :cnts[r, h]], c_ids[r, h])) for r in range(w.batch) for h in range(w.n_q_heads))
        recall = hits / float(cnts.sum())

    # Profiled repeat of the same loop: per-kernel durations from HIP events on the launch stream.
    c.set_profiling(True)
    run(steps)
    kt = c.kernel_times()
    c.set_profiling(False)
    pages_sampled, pages_main = c.debug_pages()              # of the last step (the context grows by one token a step)
    survivors = c.debug_survivors()
    bytes_per_row = w.head_dim * 2                            # one bf16 K row, read once
    bytes_per_launch = pages_main * 64 * w.n_kv_heads * bytes_per_row   # the pages whose keys the main pass reads
    pages_call = sum((c.seq_len(r) + 63) // 64 for r in seqs)
    bytes_per_call = pages_call * 64 * w.n_kv_heads * bytes_per_row     # every K row of the call, once

    def per_kernel(k):
        us = {n: round(v["sum_ms"] / v["launches"] * 1e3, 2) for n, v in k.items() if v["launches"]}
        main_s = k["score"]["sum_ms"] / max(1, k["score"]["launches"]) * 1e-3
        pass_s = main_s + k["sample"]["sum_ms"] / max(1, k["sample"]["launches"]) * 1e-3
        return us, bytes_per_launch / main_s / 1e9, bytes_per_call / pass_s / 1e9, main_s

    kernels_us, warm_gbs, warm_pass_gbs, warm_main_s = per_kernel(kt)
    # The gather + attend kernel reads one V row per selected (head, token).
    stride = int(max(w.topk) + sum(window)) if w.mode == "topk" else 0
    if stride:
        _, sel, counts = c.sparse_attn(seqs, q, mode, out=out, ids_stride=stride, **kw)
    else:
        _, counts = c.sparse_attn(seqs, q, mode, out=out, want_counts=True, **kw)
    selected_rows = int(counts.sum().item())
    # How many of those rows the G query heads of a KV group share (they read the same V rows): the heads
    # select on their own, so a row that two heads of a group pick is fetched twice.
    distinct_rows = None
    if stride:
        sel_h, cnt_h, G = sel.cpu().numpy(), counts.cpu().numpy(), w.n_q_heads // w.n_kv_heads
        distinct_rows = sum(len(np.unique(np.concatenate([sel_h[r, h, :cnt_h[r, h]] for h in range(g0, g0 + G)])))
                            for r in range(w.batch) for g0 in range(0, w.n_q_heads, G))
    attend_ms = kt["attend"]["sum_ms"] / max(1, kt["attend"]["launches"])
    gather_bytes = selected_rows * bytes_per_row
    gather = {"kernel": "attend_kernel", "selected_rows": selected_rows, "distinct_rows_per_kv_group": distinct_rows,
              "bytes_per_launch": gather_bytes,
              "avg_us": attend_ms * 1e3, "achieved": gather_bytes / (attend_ms * 1e-3) / 1e9, "unit": "GB/s",
              "frac": gather_bytes / (attend_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}

    # The same steps with the last-level cache flushed before each one (a 1 GiB buffer is read, which
    # leaves no dirty lines behind to be written back during the step): in a model with many layers
    # every layer's keys arrive cold.  Only the per-kernel event times of this loop are used; its wall
    # clock includes the flushes.
    cold = None
    if cold_steps > 0:
        scratch = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        c.set_profiling(True)
        for _ in range(cold_steps):
            scratch.sum()
            step()
        torch.cuda.synchronize()
        ktc = c.kernel_times()
        c.set_profiling(False)
        del scratch
        cold_us, cold_gbs, cold_pass_gbs, cold_main_s = per_kernel(ktc)
        gather_cold_ms = ktc["attend"]["sum_ms"] / max(1, ktc["attend"]["launches"])
        cold = {"steps": cold_steps, "kernels_us": cold_us, "step_kernel_sum_us": round(sum(cold_us.values()), 2),
                "main_pass_achieved": cold_gbs, "unit": "GB/s", "main_pass_frac": cold_gbs / HBM_PEAK_GBS,
                "scoring_pass_frac": cold_pass_gbs / HBM_PEAK_GBS,
                "gather_frac": gather_bytes / (gather_cold_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}

    # Dense attention over the same cache, for context (reads K and V once each).
    full_ms = None
    if dense:
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(10):
            c.full_attn(seqs, q, out=out)
        torch.cuda.synchronize()
        full_ms = (time.perf_counter() - t) / 10 * 1e3

    if args.calibration_copy_mb > 0:
        # A plain copy of known size: what FETCH_SIZE / WRITE_SIZE read for it gives the counters' scale.
        src = torch.ones(args.calibration_copy_mb << 18, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cpu = None
    if cpu_baseline:
        import oracle
        # One whole step of the first request on the oracle (scores, selection, attention; fp64).
        # Repeated until it has used about 20 s of CPU time (threads x wall), so that the figure is stable.
        n = w.lens[0]
        reps, cpu_s = 0, 0.0
        t0 = time.perf_counter()
        while True:
            res = oracle.sparse_attn(g["q"][0], g["K"][0], g["V"][0],
                                     oracle.TOPK if w.mode == "topk" else oracle.DIPR,
                                     k=w.topk[0] if w.topk else 0, beta=beta, want_ids=False, window=window)
            reps += 1
            dt = time.perf_counter() - t0
            cpu_s = dt * int(res["threads"])
            if cpu_s >= 20.0 or dt >= 30.0:
                break
        # ... and once on a single thread, on the first KV head's group (the groups are independent, equal work)
        G = w.n_q_heads // w.n_kv_heads
        t1 = time.perf_counter()
        oracle.sparse_attn(g["q"][0][:G], g["K"][0][:, :1], g["V"][0][:, :1],
                           oracle.TOPK if w.mode == "topk" else oracle.DIPR,
                           k=w.topk[0] if w.topk else 0, beta=beta, want_ids=False, threads=1, window=window)
        dt1 = time.perf_counter() - t1
        model = ""
        try:
            with open("/proc/cpuinfo") as f:
                model = next((ln.split(":", 1)[1].strip() for ln in f if ln.startswith("model name")), "")
        except OSError:
            pass
        cpu = {"value": w.n_q_heads * n * reps / dt, "unit": "keys/s", "cores": int(res["threads"]),
               "cpu_model": model, "host_cpus": os.cpu_count(),
               "kind": "oracle", "single_thread_value": G * n / dt1,
               "sample": f"{reps} full steps of request 0 ({n} tokens x {w.n_q_heads} heads each), "
                         f"{dt:.2f} s wall, about {cpu_s:.0f} s of CPU time"}

    total_n = sum(c.seq_len(r) for r in seqs)
    # Bytes the main pass moved as rocprofv3 counted them - from the committed summaries, not from this run.
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "measured_traffic.json")
    if os.path.exists(tpath):
        ent = json.load(open(tpath)).get(w.name)
        if ent:
            traffic, traffic_source = ent.get("main_pass_hbm_bytes_per_launch"), ent.get("source")
    k_bytes = bytes_per_launch
    use_cold = cold is not None and k_bytes < LLC_BYTES
    achieved = cold["main_pass_achieved"] if use_cold else warm_gbs
    res = {
        "value": keys / secs, "ms_per_step": ms_per_step,
        "config": {"workload": w.name, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim,
                   "batch": w.batch, "tokens": total_n, "mode": w.mode,
                   "topk": list(w.topk) if w.topk else None, "beta": beta if w.mode == "dipr" else None,
                   "paged": "64-token pages" + (", randomly permuted" if w.permute_pages else ""),
                   "accumulate": "fp32", "window": list(window),
                   "calls_per_step": "alaya_append_kv_step + alaya_sparse_attn" if args.separate_append
                   else "alaya_decode_step"},
        "latency_us_per_layer": ms_per_step * 1e3,
        "k_rows_per_s": rows / secs,
        "kernels_us": kernels_us,
        "full_attn_ms": full_ms,
        "survivor_fraction": survivors / (w.n_q_heads * total_n),
        "repaired_heads_per_step": repairs / steps,
        "coarse": None if coarse_div <= 0 else {"pages_per_head": kw["coarse_pages"], "recall_of_exact_topk": recall},
        "pages": {"call": pages_call, "sampled": pages_sampled, "main_pass_reads": pages_main},
        "roofline": {"bound": "hbm", "kernel": "main_kernel (main scoring pass)", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "cache": "cold (last-level cache flushed before every step)" if use_cold else
                              "as timed (the keys of one call are far larger than the last-level cache)",
                     "warm_frac": warm_gbs / HBM_PEAK_GBS,
                     "scoring_pass_frac": (cold["scoring_pass_frac"] if use_cold else warm_pass_gbs / HBM_PEAK_GBS),
                     "traffic": traffic, "traffic_source": traffic_source,
                     "bytes_per_launch": bytes_per_launch,
                     "avg_us": (bytes_per_launch / (achieved * 1e9)) * 1e6},
        "gather": gather,
        "cold_cache": cold,
        "cpu_baseline": cpu,
    }
    c.close()
    del c, g, q, step_k, step_v, ek, ev, out
    gc.collect()
    torch.cuda.empty_cache()
    return res


def measure_diprs(args, name="range_256k", degree=32, beta=2.0, l0s=(64, 1024), reps=20):
    """The approximate DIPR query on the graph index (Algorithm 1) beside the exact DIPR scan, same cache, same
    query, no append: build time and size of the index, time per query, length of the list C, size of the
    answer and the share of the exact answer that it holds."""
    import numpy as np
    import torch

    import paper_2504_10326_amd as A
    import workloads as wl

    w = wl.config(name)
    g = wl.generate(w)
    n = w.lens[0]
    c = A.Cache(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, max_seqs=1, max_batch=1, max_tokens_per_seq=n + 64,
                max_batch_tokens=n + 64, n_phys_pages=g["n_phys_pages"],
                phys_page_order=g["page_order"] if w.permute_pages else None)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda().view(torch.bfloat16)
    c.append_kv(0, dev(g["K"][0]), dev(g["V"][0]))
    q = dev(g["q"])
    torch.cuda.synchronize()
    t = time.perf_counter()
    gr = c.build_graph(0, degree)
    torch.cuda.synchronize()
    build_ms = (time.perf_counter() - t) * 1e3
    print(f"[bench] graph over {n} keys x {w.n_kv_heads} KV heads, degree {degree}: {build_ms:.0f} ms", file=sys.stderr, flush=True)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / reps * 1e6

    out = torch.empty((1, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    scan_us = timed(lambda: c.sparse_attn([0], q, A.ALAYA_DIPR, beta=[beta], out=out))
    ex = c.sparse_attn([0], q, A.ALAYA_DIPR, beta=[beta], ids_stride=n)
    e_ids, e_cnt = ex[1].cpu().numpy()[0], ex[2].cpu().numpy()[0]
    res = {"workload": name, "tokens": n, "degree": degree, "beta": beta, "graph_build_ms": build_ms,
           "index_bytes": int(gr.index_mem.numel()), "exact_scan_us": scan_us,
           "exact_answer_mean": float(e_cnt.mean()), "walks": []}
    for l0 in l0s:
        us = timed(lambda: c.diprs_attn(gr, q, beta, l0, out=out))
        _, ids, cnt = c.diprs_attn(gr, q, beta, l0, ids_stride=n)
        ids, cnt = ids.cpu().numpy()[0], cnt.cpu().numpy()[0]
        lens = [len(c.debug_diprs_list(h)) for h in range(w.n_q_heads)]
        rec = [len(np.intersect1d(ids[h, :cnt[h]], e_ids[h, :e_cnt[h]])) / max(1, int(e_cnt[h])) for h in range(w.n_q_heads)]
        res["walks"].append({"l0": l0, "us_per_query": us, "list_len_mean": float(np.mean(lens)), "list_len_max": int(max(lens)),
                             "answer_mean": float(cnt.mean()), "recall_of_exact_dipr": float(np.mean(rec)),
                             "neighbours_examined_mean": float(np.mean(lens)) * degree})
    gr.close()
    c.close()
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="batched_16",
                    choices=["llama8b_128k", "range_256k", "paged_1m", "batched_16", "clustered_128k"])
    ap.add_argument("--coarse-div", type=int, default=0,
                    help="answer --workload through the coarse index with 1 / this of the pages per head (0 = exact)")
    ap.add_argument("--beta", type=float, default=2.0, help="DIPR margin for range_256k")
    ap.add_argument("--window", default="0,0",
                    help="INIT,LAST tokens that are always attended (the paper's tables use 128,512)")
    ap.add_argument("--separate-append", action="store_true",
                    help="append and attend through two calls instead of one alaya_decode_step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="measure only --workload")
    ap.add_argument("--cold-steps", type=int, default=40,
                    help="extra steps with the last-level cache flushed before each (0 = skip)")
    ap.add_argument("--pages-per-wave", type=int, default=0)
    ap.add_argument("--attend-splits", type=int, default=0)
    ap.add_argument("--write-all-scores", action="store_true")
    ap.add_argument("--diprs-only", action="store_true",
                    help="run only the graph-index leg (build, walks, exact scan beside them) and print its block")
    ap.add_argument("--calibration-copy-mb", type=int, default=0,
                    help="also run a plain device copy of this many MiB (reference for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        return 2

    import torch

    import paper_2504_10326_amd as A

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 1
    A.lib()
    if args.diprs_only:
        print(json.dumps({"diprs_vs_scan": measure_diprs(args)}))
        return 0
    head = measure(args.workload, args, args.steps, args.warmup, args.cold_steps, not args.no_cpu_baseline,
                   coarse_div=args.coarse_div)
    per_config = {}
    if not args.no_per_config:
        # (workload, DIPR margin, share of the pages that the coarse index keeps per head: 1 / that)
        others = [("llama8b_128k", None, 0), ("range_256k", 2.0, 0), ("range_256k", 4.0, 0), ("paged_1m", None, 0),
                  ("batched_16", None, 0), ("clustered_128k", None, 0), ("clustered_128k", None, 16), ("paged_1m", None, 16)]
        for name, beta, cdiv in others:
            if name == args.workload and cdiv == 0 and (beta is None or beta == args.beta):
                continue
            r = measure(name, args, min(args.steps, 100), min(args.warmup, 10), min(args.cold_steps, 20), False,
                        beta=beta, dense=False, coarse_div=cdiv)
            key = name if beta is None else f"{name}_beta{beta:g}"
            if cdiv:
                key += f"_coarse_1_in_{cdiv}"
            per_config[key] = {"ms_per_step": r["ms_per_step"], "keys_per_s": r["value"], "tokens": r["config"]["tokens"],
                               "kernels_us": r["kernels_us"], "survivor_fraction": r["survivor_fraction"],
                               "repaired_heads_per_step": r["repaired_heads_per_step"], "coarse": r["coarse"],
                               # (through the coarse index the main pass skips the pages no head chose: the
                               # bytes of all keys say nothing about it, and no fraction is given)
                               "main_pass_frac": None if cdiv else r["roofline"]["frac"],
                               "main_pass_warm_frac": None if cdiv else r["roofline"]["warm_frac"],
                               "main_pass_cache": r["roofline"]["cache"],
                               "scoring_pass_frac": None if cdiv else r["roofline"]["scoring_pass_frac"],
                               "gather_frac": r["gather"]["frac"], "gather_rows": r["gather"]["selected_rows"],
                               "cold_kernels_us": r["cold_cache"]["kernels_us"] if r["cold_cache"] else None}
    line = {
        "metric": "keys scored/s (one layer, sparse decode step: append + score + select + gather + attend)",
        "value": head["value"], "unit": "keys/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
    }
    for k in ("config", "latency_us_per_layer", "k_rows_per_s", "kernels_us", "full_attn_ms", "survivor_fraction",
              "repaired_heads_per_step", "coarse", "pages", "roofline", "gather", "cold_cache", "cpu_baseline"):
        line[k] = head[k]
    line["per_config"] = per_config
    line["diprs_vs_scan"] = None if args.no_per_config else measure_diprs(args)
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
