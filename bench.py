#!/usr/bin/env python3
"""Throughput of the graph-ANN hot path on one MI355X.

A step is one pass of the whole hot path over one batch of queries: query
folding, best-first graph search with SQ8 traversal distances, and the fp32
rerank of the top 2k pool entries (index upload, encoding and ground truth are
set-up, outside the timed region; all inputs are resident in HBM).  The
workload is the 1M x 128 SQ8 configuration; ef is the smallest value of the
sweep {32, 64, 128, 256} whose recall@10 reaches 0.95.

Prints ONE JSON line with the metric, a roofline object for the search kernel
and the CPU oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import threading
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
sys.path.insert(0, str(ROOT))

HBM_PEAK_GBS = 8000.0

# Memory-side traffic of one search launch (bytes the L2 read from / wrote to the
# fabric: rocprofv3 FETCH_SIZE scaled by the factor a plain copy kernel of known
# size shows for the same counter, 2.0, plus WRITE_SIZE, factor 1.0; the summary
# is under profiles/).  A measurement belongs to the kernel sources it was taken
# with and to the default configuration of this script; any change voids it.
KERNEL_SOURCES = ("paper_2503_17911_amd/csrc/search_kernel.hpp", "paper_2503_17911_amd/csrc/device_utils.hpp",
                  "paper_2503_17911_amd/csrc/search.hip", "paper_2503_17911_amd/csrc/schedule.hip",
                  "paper_2503_17911_amd/csrc/entry.hip")
MEASURED_TRAFFIC = {
    # sha256 of KERNEL_SOURCES -> bytes per launch on c2, ef=128, multi-expansion, 10,000 queries scheduled by 256 pivots
    # (medians over the 140 launches of that grid in one run of this script under rocprofv3 --pmc, profiles/)
    "b598a5a99d45afe0bf1e877e0b72efeba591fa4907f40e1cceb52562de09619a": 836399.5 * 1024 * 2.0 + 5000.0 * 1024 * 1.0,
}


def kernel_source_hash():
    import hashlib
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        h.update((ROOT / rel).read_bytes())
    return h.hexdigest()


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def recall_at_k(found, truth):
    import numpy as np
    hits = 0
    for f, t in zip(found, truth):
        hits += len(np.intersect1d(f, t))
    return hits / truth.size


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--n", type=int, default=0, help="scale the base set down (debugging)")
    ap.add_argument("--nq", type=int, default=0)
    ap.add_argument("--ef", type=int, default=0, help="skip the sweep and use this ef")
    ap.add_argument("--ef-list", default="", help="comma-separated pool sizes to sweep instead of the workload's own list")
    ap.add_argument("--mode", type=int, default=-1, help="0 exact, 1 multi-expansion; -1: fastest that meets recall")
    ap.add_argument("--expansions", type=int, default=0, help="expansions per step in mode 1 (0 = library default)")
    ap.add_argument("--visited-slots", type=int, default=0, help="LDS visited-set slots (0 = library default)")
    ap.add_argument("--visited-kind", type=int, default=0, help="0 library default, 1 two-way cache, 2 probing table, 3 two-way cache with whole ids")
    ap.add_argument("--pivots", type=int, default=0,
                    help="entry-point stage: scan this many sampled base vectors per query (0 = start at the medoid)")
    ap.add_argument("--n-entry", type=int, default=1, help="initial nodes per query taken from the pivot scan")
    ap.add_argument("--layout", type=int, default=-1,
                    help="0: code rows and norm terms gathered; 1: redundant neighbour-code layout (PRS); 2: code rows gathered, "
                         "norm terms read with the adjacency rows; -1: time 0 and 2 (2 only where keys use a norm term) and take the faster")
    ap.add_argument("--prs-ratio", type=float, default=1.0, help="redundancy ratio of the PRS layout (share of a row's slots stored with the node)")
    ap.add_argument("--schedule-pivots", type=int, default=256,
                    help="order each batch so that similar queries share a die's L2: keys from a scan of this many "
                         "pivots (0 = natural order; with --pivots the entry scan's result is the key)")
    ap.add_argument("--coverage", type=float, default=1.0,
                    help="codebook range: 1 = per-dimension min/max, below 1 = truncated (symmetric order statistics)")
    ap.add_argument("--unit-norm-l2-keys", action="store_true",
                    help="inner-product workloads with unit-norm vectors: low-precision keys in the Euclidean form")
    ap.add_argument("--query-15bit", action="store_true", help="fold queries to 15 bits (two packed-dot passes per code row)")
    ap.add_argument("--rerank-gamma", type=float, default=-1.0,
                    help=">= 0: per-query rerank length from the key gap (ann_rerank_adaptive) instead of the fixed prefix")
    ap.add_argument("--rerank-max", type=int, default=0, help="longest reranked prefix with --rerank-gamma (0 = ef)")
    ap.add_argument("--rerank-mult", type=int, default=0, help="fixed rerank prefix in units of k (0 = the workload's own)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--bruteforce", action="store_true",
                    help="time the exact brute-force search alone (the ground-truth stage) on the workload's vectors "
                         "and queries, k = 10 on the whole batch and k = 100 on a fifth of it, print one JSON line, exit")
    ap.add_argument("--print-kernel-hash", action="store_true", help="print the hash MEASURED_TRAFFIC is keyed by, and exit")
    args = ap.parse_args()
    if args.print_kernel_hash:
        print(kernel_source_hash())
        return
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (queries are independent: more GPUs would each hold the "
                 "index and take a share of the batch, with no exchange); run with --gpus 1")

    import numpy as np
    import torch

    import inputs
    import paper_2503_17911_amd as ann

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    w = inputs.WORKLOADS[args.workload]
    if args.n:
        w = w.scaled(args.n, nq=args.nq or w.nq)
    elif args.nq:
        w = w.scaled(w.n, nq=args.nq, n_clusters=w.n_clusters)
    metric = ann.L2 if w.metric == "l2" else ann.IP
    bits = w.bits[0]
    k, n_rerank = w.k, (args.rerank_mult or w.rerank_mult) * w.k
    adaptive = args.rerank_gamma >= 0.0
    if args.bruteforce:
        bruteforce_only(w, metric)
        return

    t0 = time.time()
    X = inputs.base_vectors(w)
    Q = inputs.queries(w)
    log(f"[bench] inputs {w.name}: X {X.shape}, Q {Q.shape} in {time.time() - t0:.1f}s")
    t0 = time.time()
    adj, entry = inputs.graph(w, X)
    log(f"[bench] graph degree {adj.shape[1]} entry {entry} in {time.time() - t0:.1f}s")

    st = torch.cuda.current_stream().cuda_stream
    xd = torch.from_numpy(X).to(dev)
    qd = torch.from_numpy(Q).to(dev)
    n, d, nq = w.n, w.d, w.nq
    lo = torch.empty(d, dtype=torch.float32, device=dev)
    delta = torch.empty(d, dtype=torch.float32, device=dev)
    codes = torch.empty((n, d if bits == 8 else d // 2), dtype=torch.uint8, device=dev)
    norm = torch.empty(n, dtype=torch.float32, device=dev)
    if args.coverage < 1.0:
        ann.ann_sq_train_truncated(xd, n, d, bits, args.coverage, lo, delta, st)
    else:
        ann.ann_sq_train(xd, n, d, bits, lo, delta, st)
    ann.ann_sq_encode(xd, n, d, bits, lo, delta, codes, norm, st)
    levels = [(bits, codes, lo, delta, norm)]
    if len(w.bits) > 1:
        # second, finer code level for the rescore stage of the cascade (low -> higher -> full precision)
        b2 = w.bits[1]
        lo2 = torch.empty(d, dtype=torch.float32, device=dev)
        delta2 = torch.empty(d, dtype=torch.float32, device=dev)
        codes2 = torch.empty((n, d if b2 == 8 else d // 2), dtype=torch.uint8, device=dev)
        norm2 = torch.empty(n, dtype=torch.float32, device=dev)
        ann.ann_sq_train(xd, n, d, b2, lo2, delta2, st)
        ann.ann_sq_encode(xd, n, d, b2, lo2, delta2, codes2, norm2, st)
        levels.append((b2, codes2, lo2, delta2, norm2))
    adj_d = torch.from_numpy(adj.view(np.int32)).to(dev)
    index = ann.ann_upload_index(n=n, d=d, degree=adj.shape[1], metric=metric, vectors=xd,
                                 levels=levels, adjacency=adj_d, entry_point=entry,
                                 unit_norm_l2_keys=args.unit_norm_l2_keys, query_15bit=args.query_15bit, stream=st)
    del codes, adj_d, levels
    torch.cuda.synchronize()

    # exact ground truth (set-up)
    gt_ids = torch.empty((nq, k), dtype=torch.int32, device=dev)
    gt_dist = torch.empty((nq, k), dtype=torch.float32, device=dev)
    t0 = time.time()
    ann.ann_bruteforce_topk(xd, n, d, qd, nq, k, metric, gt_ids, gt_dist, st)
    torch.cuda.synchronize()
    bf_s = time.time() - t0
    log(f"[bench] brute-force ground truth {bf_s:.2f}s ({2 * n * nq * d / bf_s / 1e12:.1f} TFLOP/s)")
    gt = gt_ids.cpu().numpy()

    out_ids = torch.empty((nq, k), dtype=torch.int32, device=dev)
    out_dist = torch.empty((nq, k), dtype=torch.float32, device=dev)

    if args.layout == 1:
        ann.ann_build_prs_ratio(index, args.prs_ratio, st)
    keys_use_norms = metric == ann.L2 or args.unit_norm_l2_keys
    auto_layout = args.layout < 0
    layouts = [args.layout] if args.layout >= 0 else ([0, 2] if keys_use_norms else [0])
    if 2 in layouts:
        ann.ann_build_row_norms(index, st)
    args.layout = layouts[0]          # the layout of the searches below; set again once the sweep has chosen
    entries = None
    if args.pivots:
        ann.ann_build_entry_table(index, args.pivots, st)
        entries = torch.empty((nq, args.n_entry), dtype=torch.int32, device=dev)

    # processing order of a batch (a speed knob): one key per query from a pivot
    # scan, then ann_schedule_queries; part of every timed step
    scheduling = args.schedule_pivots > 0 or entries is not None
    if scheduling and entries is None:
        ann.ann_build_entry_table(index, args.schedule_pivots, st)
    sched_buf = {}

    def schedule(q_, nq_, entries_):
        """Returns the query_order tensor for this batch (None: natural order)."""
        if not scheduling:
            return None
        if nq_ not in sched_buf:
            sched_buf[nq_] = tuple(torch.empty(nq_, dtype=torch.int32, device=dev) for _ in range(2))
        keys, order = sched_buf[nq_]
        if entries_ is not None:
            keys = entries_[:, 0].contiguous() if entries_.shape[1] > 1 else entries_
        else:
            ann.ann_entry_scan(index, q_, nq_, 1, keys, st)
        ann.ann_schedule_queries(keys, nq_, n, order, st)
        return order

    key_bufs = {}

    def keys_of(t):
        """The key buffer that goes with an id buffer (only kept when the rerank length depends on the keys)."""
        if not adaptive:
            return None
        if t.data_ptr() not in key_bufs:
            key_bufs[t.data_ptr()] = torch.empty(t.shape, dtype=torch.float32, device=dev)
        return key_bufs[t.data_ptr()]

    n_reranked = {}

    def search(q_, nq_, ef, mode, pool, entries_, counts=None, complete_table=False):
        if entries_ is not None:
            ann.ann_entry_scan(index, q_, nq_, args.n_entry, entries_, st)
        order = schedule(q_, nq_, entries_)
        ann.ann_search_batch(index, q_, nq_, k=k, ef=ef, mode=mode, out_ids=pool, out_keys=keys_of(pool), out_counts=counts,
                             entry_ids=entries_, n_entry=args.n_entry if entries_ is not None else 0,
                             layout=args.layout, expansions_per_step=args.expansions if mode == 1 else 0,
                             visited_slots=8192 if complete_table else args.visited_slots,
                             visited_kind=ann.VISITED_TABLE if complete_table else args.visited_kind,
                             query_order=order, reuse_folded_queries=order is not None or entries_ is not None,
                             stream=st)

    def run_step(ef, mode, pool, counts=None, complete_table=False):
        search(qd, nq, ef, mode, pool, entries, counts, complete_table)
        finish(pool, ef)

    rescored = {}

    def finish(pool, ef, nq_=None, q_=None, ids_=None, dist_=None):
        """Rescore with the finer code level if the workload has one, then the fp32 rerank."""
        nq_ = nq if nq_ is None else nq_
        q_ = qd if q_ is None else q_
        src = pool
        if len(w.bits) > 1:
            key = (nq_, ef)
            if key not in rescored:
                rescored[key] = torch.empty((nq_, ef), dtype=torch.int32, device=dev)
            ann.ann_rescore(index, 1, q_, nq_, pool, ef, ef, rescored[key], keys_of(rescored[key]), None, st)
            src = rescored[key]
        if adaptive:
            if nq_ not in n_reranked:
                n_reranked[nq_] = torch.empty(nq_, dtype=torch.int32, device=dev)
            ann.ann_rerank_adaptive(index, q_, nq_, src, keys_of(src), min(n_rerank, ef), min(args.rerank_max or ef, ef), ef,
                                    args.rerank_gamma, k, out_ids if ids_ is None else ids_,
                                    out_dist if dist_ is None else dist_, n_reranked[nq_], st)
            return
        ann.ann_rerank(index, q_, nq_, src, min(n_rerank, ef), ef, k, out_ids if ids_ is None else ids_,
                       out_dist if dist_ is None else dist_, st)

    # recall sweep
    efs = [args.ef] if args.ef else ([int(e) for e in args.ef_list.split(",")] if args.ef_list else list(w.ef))
    modes = [args.mode] if args.mode >= 0 else [0, 1]
    # expansions per step of the multi-expansion mode: 4 and the library's maximum (8: fewer and
    # wider steps, more evaluations - faster where the batch does not fill the chip), unless one is asked for
    p_lists = {0: [0], 1: [args.expansions] if args.expansions else [4, 8]}
    p_of = lambda mode_, p_: 1 if mode_ == 0 else p_
    sweep = []
    sweep_counts = {}
    chosen = None
    meeting = []
    for ef in efs:
        pool = torch.empty((nq, ef), dtype=torch.int32, device=dev)
        counts = torch.empty((nq, 4), dtype=torch.int32, device=dev)
        for mode, p_ in [(m_, p_) for m_ in modes for p_ in p_lists[m_]]:
            args.expansions = p_
            # counting run with the largest visited table: no rebuilds, so the
            # evaluation counts are those of the algorithm itself
            run_step(ef, mode, pool, counts, complete_table=True)
            torch.cuda.synchronize()
            rec = recall_at_k(out_ids.cpu().numpy(), gt)
            c = counts.cpu().numpy().astype(np.int64)
            sweep_counts[(ef, mode, p_)] = c
            for lay in layouts:             # a storage choice: same results, so recall and counts are those above
                args.layout = lay
                run_step(ef, mode, pool)        # first launch of this kernel variant: not timed
                ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                reps_sw = 12 if rec >= 0.95 else 3      # the candidates for the headline are timed longer
                ev0.record()
                for _ in range(reps_sw):
                    run_step(ef, mode, pool)
                ev1.record()
                torch.cuda.synchronize()
                ms = ev0.elapsed_time(ev1) / reps_sw
                sweep.append(dict(ef=ef, mode=mode, expansions_per_step=p_of(mode, p_), layout=lay, recall=round(rec, 4),
                                  qps=round(nq / ms * 1e3), n_exp=float(c[:, 0].mean()), n_dist=float(c[:, 1].mean()),
                                  rebuilds=int(c[:, 3].sum())))
                log(f"[bench] ef={ef} mode={mode} P={p_of(mode, p_)} layout={lay} recall@{k}={rec:.4f} {ms:.3f} ms/batch "
                    f"n_exp={c[:, 0].mean():.1f} n_dist={c[:, 1].mean():.1f} rebuilds={int(c[:, 3].sum())}")
                if rec >= 0.95:
                    meeting.append((ef, mode, rec, c, ms, lay, p_))
            args.layout = layouts[0]
    if meeting:
        # the fastest configuration that meets the target; configurations within 2 % of it (a dozen launches each:
        # closer than the timing resolves) are ranked by the evaluations they need, then by time
        t_best = min(m_[4] for m_ in meeting)
        chosen = min((m_ for m_ in meeting if m_[4] <= 1.02 * t_best), key=lambda m_: (float(m_[3][:, 1].mean()), m_[4]))
    if chosen is None:          # target recall not reached inside the sweep: report the best point, say so
        best = max(sweep, key=lambda r: r["recall"])
        best = max((r for r in sweep if r["recall"] == best["recall"]), key=lambda r: r["qps"])
        ef, mode = best["ef"], best["mode"]
        p_ = next(p for (e_, m_, p) in sweep_counts if e_ == ef and m_ == mode and p_of(m_, p) == best["expansions_per_step"])
        chosen = (ef, mode, best["recall"], sweep_counts[(ef, mode, p_)], 0.0, best["layout"], p_)
    ef, mode, rec, c, _, args.layout, args.expansions = chosen
    n_expansions = p_of(mode, args.expansions)
    mode_name = "exact" if mode == 0 else f"multi-expansion ({n_expansions} per step)"
    pool = torch.empty((nq, ef), dtype=torch.int32, device=dev)

    # algorithmic bytes of one search launch: adjacency rows + code rows (+ norm
    # term for L2) actually needed, folded query in, pool out
    code_row = d if bits == 8 else d // 2
    per_eval = code_row + (4 if metric == ann.L2 else 0)

    def algorithmic_bytes(cnt, ef_):
        return int((cnt[:, 0] * 4 * adj.shape[1] + cnt[:, 1] * per_eval).sum() + cnt.shape[0] * (d + ef_ * 4))

    bytes_search = algorithmic_bytes(c, ef)
    bytes_rerank = nq * (min(n_rerank, ef) * (d * 4 + 4) + d * 4 + k * 8)

    # the configuration that is timed repeats some evaluations because its small
    # visited set forgets; report how many
    counts = torch.empty((nq, 4), dtype=torch.int32, device=dev)
    run_step(ef, mode, pool, counts)
    torch.cuda.synchronize()
    ca = counts.cpu().numpy().astype(np.int64)
    evals_timed, rebuilds_timed = float(ca[:, 1].mean()), float(ca[:, 3].mean())
    log(f"[bench] timed configuration: {evals_timed:.1f} evaluations/query ({float(c[:, 1].mean()):.1f} needed), "
        f"{rebuilds_timed:.2f} table rebuilds/query")

    # timed region
    for _ in range(args.warmup):
        run_step(ef, mode, pool)
    torch.cuda.synchronize()
    e_begin = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    e_mid = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    e_start, e_end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_wall = time.perf_counter()
    e_start.record()
    for i in range(args.steps):
        if entries is not None:
            ann.ann_entry_scan(index, qd, nq, args.n_entry, entries, st)
        order = schedule(qd, nq, entries)
        e_begin[i].record()
        ann.ann_search_batch(index, qd, nq, k=k, ef=ef, mode=mode, out_ids=pool, out_keys=keys_of(pool),
                             entry_ids=entries, n_entry=args.n_entry if entries is not None else 0, layout=args.layout,
                             expansions_per_step=args.expansions if mode == 1 else 0,
                             visited_slots=args.visited_slots, visited_kind=args.visited_kind,
                             query_order=order, reuse_folded_queries=order is not None or entries is not None,
                             stream=st)
        e_mid[i].record()
        finish(pool, ef)
    e_end.record()
    torch.cuda.synchronize()
    wall_s = time.perf_counter() - t_wall
    ref_ids = out_ids.clone()        # the timed configuration's results, for the variants below to be checked against
    total_ms = e_start.elapsed_time(e_end)
    ms_per_step = total_ms / args.steps
    search_ms = float(np.mean([e_begin[i].elapsed_time(e_mid[i]) for i in range(args.steps)]))
    # the query-folding kernel runs inside ann_search_batch ahead of the search
    # kernel; time it alone and take it off to get the search kernel's duration
    p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 20
    ann.ann_query_prep(index, 0, qd, nq, None, None, None, st)
    p0.record()
    for _ in range(reps):
        ann.ann_query_prep(index, 0, qd, nq, None, None, None, st)
    p1.record()
    torch.cuda.synchronize()
    prep_ms = p0.elapsed_time(p1) / reps
    # (when the batch was scheduled, the folding ran with the pivot scan and the call holds the search kernel alone)
    folded_outside = scheduling or entries is not None
    kernel_ms = search_ms if folded_outside else max(search_ms - prep_ms, 1e-6)
    achieved = bytes_search / (kernel_ms * 1e-3) / 1e9
    qps = nq / (ms_per_step * 1e-3)
    log(f"[bench] ef={ef} mode={mode}: {ms_per_step:.3f} ms/step (search call {search_ms:.3f}, fold {prep_ms:.3f}), "
        f"{qps:,.0f} QPS, search kernel {achieved:.0f} GB/s algorithmic, wall {wall_s:.2f}s")

    # steady state: a batch of 8x as many (distinct) queries of the same law.  One
    # 10,000-query batch fills the chip less than twice, so a launch spends a good
    # part of its time draining; the larger batch shows the rate the kernels sustain.
    rep = 8
    q_big = torch.from_numpy(inputs.queries(w, nq * rep)).to(dev)
    assert torch.equal(q_big[:nq], qd)        # the generator is counter-based: a longer batch extends the shorter
    pool_big = torch.empty((nq * rep, ef), dtype=torch.int32, device=dev)
    ids_big = torch.empty((nq * rep, k), dtype=torch.int32, device=dev)
    dist_big = torch.empty((nq * rep, k), dtype=torch.float32, device=dev)

    entries_big = None
    if entries is not None:
        entries_big = torch.empty((nq * rep, args.n_entry), dtype=torch.int32, device=dev)

    def big_step():
        search(q_big, nq * rep, ef, mode, pool_big, entries_big)
        finish(pool_big, ef, nq * rep, q_big, ids_big, dist_big)

    big_step()
    torch.cuda.synchronize()
    b0, b1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    big_reps = max(3, args.steps // 20)
    b0.record()
    for _ in range(big_reps):
        big_step()
    b1.record()
    torch.cuda.synchronize()
    big_ms = b0.elapsed_time(b1) / big_reps
    assert torch.equal(ids_big[:nq], out_ids)
    steady_qps = nq * rep / (big_ms * 1e-3)
    log(f"[bench] steady state ({nq * rep} queries per batch): {big_ms:.3f} ms/batch, {steady_qps:,.0f} QPS, "
        f"{bytes_search * rep / (big_ms * 1e-3) / 1e9:.0f} GB/s algorithmic incl. fold and rerank time")
    q_second, ids_second = q_big[nq:2 * nq].clone(), ids_big[nq:2 * nq].clone()   # another batch and its results

    # rotation: the timed step again, every step on another of the 8 distinct
    # batches (the headline repeats the workload's own query set, whose lines
    # may stay in the caches from one step to the next; this does not)
    rot_bytes = []
    rot_counts = torch.empty((nq, 4), dtype=torch.int32, device=dev)
    for b in range(rep):
        qb = q_big[b * nq:(b + 1) * nq]
        search(qb, nq, ef, mode, pool, entries, rot_counts, complete_table=True)
        torch.cuda.synchronize()
        rot_bytes.append(algorithmic_bytes(rot_counts.cpu().numpy().astype(np.int64), ef))
    n_rot = rep * max(2, args.steps // (2 * rep))
    rb = [torch.cuda.Event(enable_timing=True) for _ in range(n_rot)]
    rm = [torch.cuda.Event(enable_timing=True) for _ in range(n_rot)]
    r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def rot_step(i, timed):
        qb = q_big[(i % rep) * nq:(i % rep + 1) * nq]
        if entries is not None:
            ann.ann_entry_scan(index, qb, nq, args.n_entry, entries, st)
        order = schedule(qb, nq, entries)
        if timed:
            rb[i].record()
        ann.ann_search_batch(index, qb, nq, k=k, ef=ef, mode=mode, out_ids=pool, out_keys=keys_of(pool),
                             entry_ids=entries, n_entry=args.n_entry if entries is not None else 0, layout=args.layout,
                             expansions_per_step=args.expansions if mode == 1 else 0,
                             visited_slots=args.visited_slots, visited_kind=args.visited_kind,
                             query_order=order, reuse_folded_queries=order is not None or entries is not None,
                             stream=st)
        if timed:
            rm[i].record()
        finish(pool, ef, nq, qb, ids_rot, dist_rot)

    ids_rot = torch.empty((nq, k), dtype=torch.int32, device=dev)
    dist_rot = torch.empty((nq, k), dtype=torch.float32, device=dev)
    for i in range(rep):
        rot_step(i, False)
    torch.cuda.synchronize()
    r0.record()
    for i in range(n_rot):
        rot_step(i, True)
    r1.record()
    torch.cuda.synchronize()
    rot_ms = r0.elapsed_time(r1) / n_rot
    rot_call_ms = float(np.mean([rb[i].elapsed_time(rm[i]) for i in range(n_rot)]))
    rot_kernel_ms = rot_call_ms if (scheduling or entries is not None) else max(rot_call_ms - prep_ms, 1e-6)
    rot_gbs = float(np.mean(rot_bytes)) / (rot_kernel_ms * 1e-3) / 1e9
    rotating = {"what": f"the same step over a rotation of {rep} distinct {nq}-query batches of the same law "
                        f"(the headline repeats the workload's own {nq} queries)",
                "ms_per_step": round(rot_ms, 4), "value": round(nq / (rot_ms * 1e-3), 1),
                "kernel_ms": round(rot_kernel_ms, 4), "algorithmic_GBps": round(rot_gbs, 1),
                "frac": round(rot_gbs / HBM_PEAK_GBS, 4)}
    log(f"[bench] rotation of {rep} distinct batches: {rot_ms:.3f} ms/step {nq / rot_ms * 1e3:,.0f} QPS, "
        f"search kernel {rot_kernel_ms:.3f} ms = {rot_gbs:.0f} GB/s algorithmic")
    del q_big, pool_big, ids_big, dist_big

    # Algorithm 1 as the paper defines it (one expansion per step) at the same ef:
    # its own step time and roofline figures beside the headline's
    exact = None
    if mode == 1 and (ef, 0, 0) in sweep_counts:
        c0 = sweep_counts[(ef, 0, 0)]
        rec0 = next(r["recall"] for r in sweep if r["ef"] == ef and r["mode"] == 0)
        x_layout = max((r for r in sweep if r["ef"] == ef and r["mode"] == 0), key=lambda r: r["qps"])["layout"]
        n_x = max(10, args.steps // 4)
        xb = [torch.cuda.Event(enable_timing=True) for _ in range(n_x)]
        xm = [torch.cuda.Event(enable_timing=True) for _ in range(n_x)]
        x0, x1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

        def exact_step(i):
            if entries is not None:
                ann.ann_entry_scan(index, qd, nq, args.n_entry, entries, st)
            order = schedule(qd, nq, entries)
            if i >= 0:
                xb[i].record()
            ann.ann_search_batch(index, qd, nq, k=k, ef=ef, mode=0, out_ids=pool, out_keys=keys_of(pool),
                                 entry_ids=entries, n_entry=args.n_entry if entries is not None else 0, layout=x_layout,
                                 visited_slots=args.visited_slots, visited_kind=args.visited_kind,
                                 query_order=order, reuse_folded_queries=order is not None or entries is not None,
                                 stream=st)
            if i >= 0:
                xm[i].record()
            finish(pool, ef, nq, qd, ids_rot, dist_rot)

        for _ in range(3):
            exact_step(-1)
        torch.cuda.synchronize()
        x0.record()
        for i in range(n_x):
            exact_step(i)
        x1.record()
        torch.cuda.synchronize()
        x_ms = x0.elapsed_time(x1) / n_x
        x_call = float(np.mean([xb[i].elapsed_time(xm[i]) for i in range(n_x)]))
        x_kernel = x_call if (scheduling or entries is not None) else max(x_call - prep_ms, 1e-6)
        x_bytes = algorithmic_bytes(c0, ef)
        x_gbs = x_bytes / (x_kernel * 1e-3) / 1e9
        exact = {"what": "one expansion per step (results identical to the sequential algorithm), same ef, same step",
                 "ef": ef, "layout": x_layout, f"recall_at_{k}": rec0, "ms_per_step": round(x_ms, 4), "value": round(nq / (x_ms * 1e-3), 1),
                 "kernel_ms": round(x_kernel, 4), "algorithmic_bytes_per_launch": x_bytes,
                 "algorithmic_GBps": round(x_gbs, 1), "frac": round(x_gbs / HBM_PEAK_GBS, 4)}
        log(f"[bench] exact mode ef={ef}: {x_ms:.3f} ms/step {nq / x_ms * 1e3:,.0f} QPS, search kernel {x_kernel:.3f} ms = "
            f"{x_gbs:.0f} GB/s algorithmic ({x_gbs / HBM_PEAK_GBS:.3f} of peak)")

    # latency of one query alone on the device (batch of 1): folding, search and
    # rerank launched back to back, host-synchronised; median over 1,000 launches
    pool1 = torch.empty((1, ef), dtype=torch.int32, device=dev)
    ids1 = torch.empty((1, k), dtype=torch.int32, device=dev)
    dist1 = torch.empty((1, k), dtype=torch.float32, device=dev)

    def single_query_latency(p_):
        lat = []
        for i in range(1020):
            q1 = qd[i % nq:i % nq + 1]
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            ann.ann_search_batch(index, q1, 1, k=k, ef=ef, mode=mode, out_ids=pool1, out_keys=keys_of(pool1), layout=args.layout,
                                 expansions_per_step=p_ if mode == 1 else 0,
                                 visited_slots=args.visited_slots, visited_kind=args.visited_kind, stream=st)
            finish(pool1, ef, 1, q1, ids1, dist1)
            torch.cuda.synchronize()
            if i >= 20:
                lat.append((time.perf_counter() - t1) * 1e6)
        lat.sort()
        return lat[len(lat) // 2], lat[int(len(lat) * 0.99)]

    lat_med, lat_p99 = single_query_latency(args.expansions)
    log(f"[bench] one query alone: median {lat_med:.0f} us, p99 {lat_p99:.0f} us (launch + search + rerank, host-synchronised)")
    # a query alone is bound by its chain of dependent steps: the same with eight expansions per step
    lat8 = None
    if mode == 1 and n_expansions != 8:
        lat8 = single_query_latency(8)
        log(f"[bench] one query alone, eight expansions per step: median {lat8[0]:.0f} us, p99 {lat8[1]:.0f} us")

    # variant: pool sizes between the workload's own values.  The headline keeps to the list the workload
    # names; the smallest pool between the chosen one and the one below it that still meets the target
    # is what "queries/s at the recall target" would be on a finer curve.
    finer = None
    below = max([e for e in efs if e < ef], default=0)
    if not args.ef and not args.ef_list and rec >= 0.95 and ef - below >= 32:
        for ef_f in sorted({below + (ef - below) * j // 4 // 8 * 8 for j in (1, 2, 3)} - {below, ef}):
            if ef_f < k:
                continue
            pool_f = torch.empty((nq, ef_f), dtype=torch.int32, device=dev)
            run_step(ef_f, mode, pool_f)
            torch.cuda.synchronize()
            rec_f = recall_at_k(out_ids.cpu().numpy(), gt)
            if rec_f < 0.95:
                continue
            f0, f1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            n_f = max(10, args.steps // 4)
            f0.record()
            for _ in range(n_f):
                run_step(ef_f, mode, pool_f)
            f1.record()
            torch.cuda.synchronize()
            ms_f = f0.elapsed_time(f1) / n_f
            finer = {"what": "smallest pool size between the workload's listed values that meets the recall target; same step",
                     "ef": ef_f, "mode": mode_name, f"recall_at_{k}": round(rec_f, 4), "ms_per_step": round(ms_f, 4),
                     "value": round(nq / (ms_f * 1e-3), 1)}
            log(f"[bench] finer pool size: ef={ef_f} recall@{k}={rec_f:.4f} {ms_f:.3f} ms/step {nq / ms_f * 1e3:,.0f} QPS")
            break
        run_step(ef, mode, pool)        # leave the timed configuration's results in place
        torch.cuda.synchronize()

    # variant: per-query entry points from a scan of 1024 sampled base vectors
    # (the entry-point stage) instead of the medoid; same recall target
    variant = None
    if entries is None:
        ann.ann_build_entry_table(index, 1024, st)
        ent = torch.empty((nq, 1), dtype=torch.int32, device=dev)

        v_order = torch.empty(nq, dtype=torch.int32, device=dev)

        def variant_step(ef_v, pool_v):
            ann.ann_entry_scan(index, qd, nq, 1, ent, st)
            order_v = None
            if scheduling:          # the entry scan's result is the scheduling key: no second scan
                ann.ann_schedule_queries(ent, nq, n, v_order, st)
                order_v = v_order
            ann.ann_search_batch(index, qd, nq, k=k, ef=ef_v, mode=1, out_ids=pool_v, out_keys=keys_of(pool_v), entry_ids=ent, n_entry=1,
                                 expansions_per_step=args.expansions if mode == 1 else ann.ann_default_expansions_per_step(ef_v, adj.shape[1]),
                                 query_order=order_v, reuse_folded_queries=True, layout=args.layout if args.layout != 1 else 0, stream=st)
            finish(pool_v, ef_v)

        for ef_v in efs:
            pool_v = torch.empty((nq, ef_v), dtype=torch.int32, device=dev)
            variant_step(ef_v, pool_v)
            torch.cuda.synchronize()
            rec_v = recall_at_k(out_ids.cpu().numpy(), gt)
            if rec_v >= 0.95 or ef_v == efs[-1]:
                v0, v1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                n_v = max(10, args.steps // 4)
                v0.record()
                for _ in range(n_v):
                    variant_step(ef_v, pool_v)
                v1.record()
                torch.cuda.synchronize()
                ms_v = v0.elapsed_time(v1) / n_v
                variant = {"entry": "closest of 1024 scanned pivots", "ef": ef_v,
                           "mode": f"multi-expansion ({args.expansions if mode == 1 else ann.ann_default_expansions_per_step(ef_v, adj.shape[1])} per step)",
                           f"recall_at_{k}": round(rec_v, 4), "ms_per_step": round(ms_v, 4),
                           "value": round(nq / (ms_v * 1e-3), 1)}
                log(f"[bench] variant with entry-point stage: ef={ef_v} recall@{k}={rec_v:.4f} {ms_v:.3f} ms/step "
                    f"{nq / ms_v * 1e3:,.0f} QPS (scan + search + rerank)")
                break

    # variant: consecutive batches overlapped on two streams of the same index
    # (the index keeps one query workspace per stream): the next batch fills the
    # chip while the previous one drains
    pipelined = None
    if entries is None and len(w.bits) == 1 and args.layout != 1 and not adaptive:
        ann.ann_build_entry_table(index, args.schedule_pivots or 256, st)
        lanes = []
        for q_lane, ids_lane in ((qd, ref_ids), (q_second, ids_second)):    # two different batches
            lanes.append(dict(ix=index, stream=torch.cuda.Stream(), q=q_lane, expect=ids_lane,
                              keys=torch.empty(nq, dtype=torch.int32, device=dev),
                              order=torch.empty(nq, dtype=torch.int32, device=dev),
                              pool=torch.empty((nq, ef), dtype=torch.int32, device=dev),
                              ids=torch.empty((nq, k), dtype=torch.int32, device=dev),
                              dist=torch.empty((nq, k), dtype=torch.float32, device=dev)))
        torch.cuda.synchronize()

        def lane_step(L):
            sp = L["stream"].cuda_stream
            ann.ann_entry_scan(L["ix"], L["q"], nq, 1, L["keys"], sp)
            ann.ann_schedule_queries(L["keys"], nq, n, L["order"], sp)
            ann.ann_search_batch(L["ix"], L["q"], nq, k=k, ef=ef, mode=mode, out_ids=L["pool"], query_order=L["order"],
                                 expansions_per_step=args.expansions if mode == 1 else 0,
                                 reuse_folded_queries=True, layout=args.layout, stream=sp)
            ann.ann_rerank(L["ix"], L["q"], nq, L["pool"], min(n_rerank, ef), ef, k, L["ids"], L["dist"], sp)

        for i in range(4):
            lane_step(lanes[i % 2])
        torch.cuda.synchronize()
        n_p = max(20, args.steps // 2)
        t_p = time.perf_counter()
        for i in range(n_p):
            lane_step(lanes[i % 2])
        torch.cuda.synchronize()
        ms_p = (time.perf_counter() - t_p) * 1e3 / n_p
        assert all(torch.equal(L["ids"], L["expect"]) for L in lanes)
        pipelined = {"what": "two different batches alternate between two streams on the one index; wall clock over "
                             f"{n_p} batches", "ms_per_step": round(ms_p, 4), "value": round(nq / (ms_p * 1e-3), 1)}
        log(f"[bench] two batches in flight (two streams): {ms_p:.3f} ms/step {nq / ms_p * 1e3:,.0f} QPS")

    # variant: the same index with its nodes renumbered so that the rows of one
    # region of the space lie together (an index-layout choice a builder can
    # make; ids are mapped back before recall is taken).  Region = the closest of
    # 1024 pivots, found with the library's own pivot scan over the base vectors.
    relabel = None
    if entries is None and len(w.bits) == 1 and args.layout != 1 and args.coverage == 1.0 and not adaptive and not args.unit_norm_l2_keys and not args.query_15bit:
        ann.ann_build_entry_table(index, 1024, st)
        region = torch.empty(n, dtype=torch.int32, device=dev)
        ann.ann_entry_scan(index, xd, n, 1, region, st)
        torch.cuda.synchronize()
        perm = torch.argsort(region.to(torch.int64), stable=True)            # new id -> old id
        inv = torch.empty_like(perm)
        inv[perm] = torch.arange(n, device=dev)
        x2 = xd[perm].contiguous()
        adj_old = torch.from_numpy(adj.astype(np.int64)).to(dev)[perm]
        pad = adj_old == 0xFFFFFFFF
        adj2 = inv[torch.where(pad, torch.zeros_like(adj_old), adj_old)]
        adj2[pad] = 0xFFFFFFFF
        adj2 = (adj2 & 0xFFFFFFFF).to(torch.uint32).view(torch.int32).contiguous()
        codes2 = torch.empty((n, d if bits == 8 else d // 2), dtype=torch.uint8, device=dev)
        norm2 = torch.empty(n, dtype=torch.float32, device=dev)
        ann.ann_sq_encode(x2, n, d, bits, lo, delta, codes2, norm2, st)      # same codebook: it does not depend on the order
        index2 = ann.ann_upload_index(n=n, d=d, degree=adj.shape[1], metric=metric, vectors=x2,
                                      levels=[(bits, codes2, lo, delta, norm2)], adjacency=adj2,
                                      entry_point=int(inv[entry].item()), stream=st)
        del codes2, adj2, adj_old, region
        ann.ann_build_entry_table(index2, args.schedule_pivots or 256, st)
        if args.layout == 2:
            ann.ann_build_row_norms(index2, st)
        keys2 = torch.empty(nq, dtype=torch.int32, device=dev)
        order2 = torch.empty(nq, dtype=torch.int32, device=dev)
        pool2 = torch.empty((nq, ef), dtype=torch.int32, device=dev)
        ids2 = torch.empty((nq, k), dtype=torch.int32, device=dev)
        dist2 = torch.empty((nq, k), dtype=torch.float32, device=dev)

        def relabel_step():
            ann.ann_entry_scan(index2, qd, nq, 1, keys2, st)
            ann.ann_schedule_queries(keys2, nq, n, order2, st)
            ann.ann_search_batch(index2, qd, nq, k=k, ef=ef, mode=mode, out_ids=pool2, query_order=order2,
                                 expansions_per_step=args.expansions if mode == 1 else 0,
                                 reuse_folded_queries=True, layout=args.layout, stream=st)
            ann.ann_rerank(index2, qd, nq, pool2, min(n_rerank, ef), ef, k, ids2, dist2, st)

        for _ in range(3):
            relabel_step()
        r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n_r = max(10, args.steps // 4)
        r0.record()
        for _ in range(n_r):
            relabel_step()
        r1.record()
        torch.cuda.synchronize()
        ms_r = r0.elapsed_time(r1) / n_r
        back = perm[ids2.to(torch.int64) & 0xFFFFFFFF].cpu().numpy()            # old ids
        rec_r = recall_at_k(back, gt)
        relabel = {"what": "nodes renumbered by region (closest of 1024 pivots) before upload; same graph, same queries",
                   "ef": ef, "mode": mode_name, f"recall_at_{k}": round(rec_r, 4),
                   "ms_per_step": round(ms_r, 4), "value": round(nq / (ms_r * 1e-3), 1)}
        log(f"[bench] variant with nodes renumbered by region: ef={ef} recall@{k}={rec_r:.4f} {ms_r:.3f} ms/step "
            f"{nq / ms_r * 1e3:,.0f} QPS")
        ann.ann_free_index(index2)
        del x2

    mean_degree = float((adj != 0xFFFFFFFF).sum(1).mean())
    shape_label = {1_000_000: "1M", 10_000_000: "10M", 5_000_000: "5M"}.get(n, str(n)) + f" x {d} " + \
        "->".join(f"SQ{b}" for b in w.bits)
    mfma_scan = scheduling and bits == 8 and d <= 256 and (entries is None or args.n_entry == 1)
    default_config = (not args.query_15bit and not adaptive and not args.unit_norm_l2_keys and not args.rerank_mult and args.workload == "c2" and not args.n and not args.nq and not args.visited_slots and not args.visited_kind
                      and not args.pivots and auto_layout and args.expansions == 4 and args.coverage == 1.0
                      and args.schedule_pivots == 256
                      and ef == 128 and mode == 1)
    traffic = MEASURED_TRAFFIC.get(kernel_source_hash()) if default_config else None
    result = {
        "metric": f"queries/sec at recall@{k}>=0.95 ({shape_label}, ef sweep)",
        "value": round(qps, 1),
        "unit": "queries/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8 traversal (int32 accumulate) + f32 rerank",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: N={n} d={d} SQ{bits} R={adj.shape[1]} (mean out-degree {mean_degree:.1f}: the graph "
                               f"fixture prunes without back-fill) {w.metric} k={k} nq={nq} "
                               + (f"rescore pool with SQ{w.bits[1]}, " if len(w.bits) > 1 else "")
                               + f"rerank top {min(n_rerank, ef)}",
                   "query_order": ((f"scheduled by the closest of {args.schedule_pivots} scanned pivots (inside the timed step"
                                    + ("; folding and pivot scan are one int8 MFMA kernel" if mfma_scan else "") + ")")
                                   if scheduling and not args.pivots else
                                   "scheduled by the entry scan's result" if scheduling else "natural"),
                   "matrix_cores_in_timed_step": ("int8 MFMA in the pivot scan that orders the batch (a dense integer contraction, "
                                                  "exact); none in the search, rescore or rerank kernels") if mfma_scan else "none",
                   "codebook": "per-dimension min/max" if args.coverage >= 1.0 else f"truncated range, coverage {args.coverage}",
                   "query_bits": 15 if args.query_15bit else 8,
                   "key_form": "Euclidean form on unit-norm inner-product data" if args.unit_norm_l2_keys else "the metric's own",
                   "rerank": (f"per-query prefix from the key gap: gamma {args.rerank_gamma}, {min(n_rerank, ef)}..{min(args.rerank_max or ef, ef)} "
                              f"candidates, mean {float(n_reranked[nq].float().mean()):.1f}" if adaptive else f"fixed prefix of {min(n_rerank, ef)}"),
                   "layout": {0: "code rows and norm terms gathered",
                              1: f"PRS, redundancy ratio {args.prs_ratio}",
                              2: "code rows gathered; a neighbour's norm term is stored and read with the adjacency row"}[args.layout]
                             + (" (the faster of the two gathered layouts, both in the sweep)" if auto_layout and len(layouts) > 1 else ""),
                   "entry": "medoid" if not args.pivots else f"closest {args.n_entry} of {args.pivots} scanned pivots",
                   "ef": ef, "mode": mode_name, f"recall_at_{k}": round(rec, 4),
                   "recall_target_met": bool(rec >= 0.95), "evaluations_per_query": round(float(c[:, 1].mean()), 1),
                   "evaluations_per_query_timed": round(evals_timed, 1),
                   "steady_state_8x_batch": {"queries_per_batch": nq * rep, "ms_per_batch": round(big_ms, 4),
                                             "value": round(steady_qps, 1),
                                             "algorithmic_GBps": round(bytes_search * rep / (big_ms * 1e-3) / 1e9, 1)},
                   "single_query_latency_us": {"median": round(lat_med, 1), "p99": round(lat_p99, 1),
                                               "launches": 1000,
                                               "what": "batch of 1: fold + search (+ rescore) + rerank, host-synchronised, one launch sequence per query",
                                               "with_8_expansions_per_step": None if lat8 is None else
                                               {"median": round(lat8[0], 1), "p99": round(lat8[1], 1)}},
                   "entry_stage_variant": variant,
                   "renumbered_nodes_variant": relabel,
                   "two_batches_in_flight": pipelined,
                   "rotating_batches": rotating,
                   "exact_mode": exact,
                   "finer_pool_size_variant": finer,
                   "sweep": sweep},
        "ground_truth": {"kernel": "ann_bruteforce_topk (fp32 MFMA 128x128 tiles, shared top-k bounds, exact re-evaluation)", "bound": "mfma",
                         "seconds": round(bf_s, 4), "achieved": round(2 * n * nq * d / bf_s / 1e12, 1),
                         "peak": 157.3, "unit": "TFLOP/s", "frac": round(2 * n * nq * d / bf_s / 1e12 / 157.3, 3),
                         "note": "set-up, outside the timed region; wall time of the whole call"},
        "roofline": {"bound": "hbm", "kernel": "search_kernel (one expansion per step)" if mode == 0 else "search_kernel (multi-expansion)",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "achieved_is": "algorithmic gathered bytes (adjacency rows + code rows + norm terms needed by the algorithm, "
                                    "counted by a run with a complete visited table) / search kernel time from HIP events in this run; "
                                    "not a measurement of HBM traffic",
                     "traffic_is": "bytes at the L2-fabric boundary per launch from rocprofv3 FETCH_SIZE/WRITE_SIZE of an earlier run of "
                                   "this command (profiles/), stored in bench.py and keyed to a hash of the kernel sources; null "
                                   "when the sources or the configuration differ; part of it is served by the 256 MB Infinity "
                                   "Cache (the workload's hot set is about that size), not HBM",
                     "traffic_measured_in_run": False,
                     "algorithmic_bytes_per_launch": bytes_search, "kernel_ms": round(kernel_ms, 4),
                     "rerank_bytes_per_launch": bytes_rerank,
                     "rest_of_step_ms": round(ms_per_step - search_ms, 4),
                     "rest_of_step": "query folding + pivot scan + scheduling + fp32 rerank" if folded_outside
                                     else "fp32 rerank (the folding is inside the search call)"},
    }

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, X, Q, adj, entry, ef, k, n_rerank, metric, args.coverage,
                                              key_metric=ann.L2 if args.unit_norm_l2_keys else metric,
                                              query_bits=15 if args.query_15bit else 8)

    ann.ann_free_index(index)
    print(json.dumps(result), flush=True)


def bruteforce_only(w, metric):
    """Whole-call time of ann_bruteforce_topk (best of five, host clock) for two values of k."""
    import torch

    import inputs
    import paper_2503_17911_amd as ann
    dev = "cuda:0"
    st = torch.cuda.current_stream().cuda_stream
    xd = torch.from_numpy(inputs.base_vectors(w)).to(dev)
    qd = torch.from_numpy(inputs.queries(w)).to(dev)
    out = {"workload": f"{w.name}: N={w.n} d={w.d} {w.metric}", "peak_TFLOPs": 157.3, "runs": []}
    for k, nq in ((10, w.nq), (100, max(1, w.nq // 5))):
        ids = torch.empty((nq, k), dtype=torch.int32, device=dev)
        dist = torch.empty((nq, k), dtype=torch.float32, device=dev)
        best = float("inf")
        for _ in range(6):      # the first call is a warm-up
            t0 = time.perf_counter()
            ann.ann_bruteforce_topk(xd, w.n, w.d, qd, nq, k, metric, ids, dist, st)
            torch.cuda.synchronize()
            best = min(best, time.perf_counter() - t0) if _ else best
        tf = 2.0 * w.n * nq * w.d / best / 1e12
        log(f"[bench] brute force k={k}: {nq} x {w.n} x {w.d} in {best * 1e3:.1f} ms = {tf:.1f} TFLOP/s")
        out["runs"].append({"k": k, "nq": nq, "ms": round(best * 1e3, 2), "TFLOPs": round(tf, 1), "frac": round(tf / 157.3, 3)})
    print(json.dumps(out), flush=True)


def oracle_fit_threaded(oracle, X, bits, coverage, threads):
    """The oracle's codebook training and encoding, split over the host's cores:
    training by blocks of columns (each dimension is trained on its own),
    encoding by blocks of rows.  Same functions, same results as one call."""
    import numpy as np
    n, d = X.shape
    lo, delta = np.empty(d, np.float32), np.empty(d, np.float32)
    col_blocks = [b for b in np.array_split(np.arange(d), threads) if len(b)]

    def train(b):
        Xb = np.ascontiguousarray(X[:, b[0]:b[-1] + 1])
        lo[b[0]:b[-1] + 1], delta[b[0]:b[-1] + 1] = (oracle.sq_train(Xb, bits) if coverage >= 1.0
                                                     else oracle.sq_train_truncated(Xb, bits, coverage))
        log(f"[bench] oracle codebook: columns {b[0]}..{b[-1]} done")

    ts = [threading.Thread(target=train, args=(b,)) for b in col_blocks]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    rb = d if bits == 8 else (d + 1) // 2
    codes, norm = np.empty((n, rb), np.uint8), np.empty(n, np.float32)
    row_blocks = [b for b in np.array_split(np.arange(n), threads) if len(b)]

    def encode(b):
        L = oracle.sq_encode(X[b[0]:b[-1] + 1], bits, lo, delta)
        codes[b[0]:b[-1] + 1], norm[b[0]:b[-1] + 1] = L.codes, L.norm_term

    ts = [threading.Thread(target=encode, args=(b,)) for b in row_blocks]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    return oracle.SQLevel(bits, lo, delta, codes, norm)


def cpu_baseline(w, X, Q, adj, entry, ef, k, n_rerank, metric, coverage=1.0, key_metric=None, query_bits=8):
    """The CPU oracle as it stands (plain C++, -O2, no SIMD intrinsics), timed
    on this host: same workload, same ef, search + rerank, on a bounded sample
    of the queries split over the host's cores (queries are independent)."""
    import numpy as np

    import oracle
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    threads = max(1, min(16, cores))
    key_metric = metric if key_metric is None else key_metric
    t0 = time.time()
    level = oracle_fit_threaded(oracle, X, w.bits[0], coverage, threads)
    log(f"[bench] oracle encode {time.time() - t0:.1f}s")
    # size the sample from a short probe so that the timed part is ~15 s of CPU work
    probe = Q[:32]
    t0 = time.perf_counter()
    oracle.search_batch(level, w.d, adj, entry, probe, ef, metric=key_metric, query_bits=query_bits)
    per_q = (time.perf_counter() - t0) / len(probe)
    want = 15.0 / max(per_q, 1e-6)                      # queries worth ~15 s of CPU work
    sample = int(min(len(Q), max(threads * 8, want)))
    passes = int(max(1, min(8, round(want / sample))))  # small query sets are run several times
    Qs = Q[:sample]
    parts = np.array_split(np.arange(sample), threads)

    def work(idx):
        if len(idx) == 0:
            return
        for _ in range(passes):
            ids, _, _, _ = oracle.search_batch(level, w.d, adj, entry, Qs[idx], ef, metric=key_metric, query_bits=query_bits)
            oracle.rerank_batch(X, Qs[idx], ids[:, :min(n_rerank, ef)], k, metric=metric)

    ts = [threading.Thread(target=work, args=(p,)) for p in parts]
    t0 = time.perf_counter()
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    dt = time.perf_counter() - t0
    done = sample * passes
    log(f"[bench] oracle: {done} queries on {threads} threads in {dt:.2f}s ({done / dt:,.0f} QPS; "
        f"{per_q * 1e3:.2f} ms/query single-thread probe)")
    return {"value": round(done / dt, 1), "unit": "queries/s", "cores": threads, "kind": "oracle",
            "sample": f"first {sample} of {len(Q)} queries x {passes} passes, ef={ef}, search + rerank, "
                      f"one thread per core",
            "single_thread_qps": round(1.0 / per_q, 1)}


if __name__ == "__main__":
    main()
