#!/usr/bin/env python3
"""Benchmark of the walk + SGNS path on one MI355X.

One "step" is one batch of positive pairs taken through the whole path:
walks (the step's share of the walk launch), pair emission (same), negative
sampling and the SGNS iteration.  All inputs are synthetic, seeded and resident
in HBM before the timed region.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 0..4]
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "sgns_step_hbm_traffic.json")
CSRC = os.path.join(ROOT, "paper_2407_15452_amd", "csrc")


def sgns_bytes_per_pair(k: int, dim: int, elem_bytes: int, window: int) -> float:
    """Algorithmic bytes per positive pair of one batch-synchronous SGNS iteration
    without any reuse: K+2 rows read for the logits, K+1 context-table rows read
    again and written for the update, the centre row read and written once per
    run of 2*window equal centres ((3(K+1) + 2/(2W)) rows in all), the 8 + 4K
    index bytes of the pair and 4 bytes of gradient coefficient per term."""
    rb = dim * elem_bytes
    return (3 * (k + 1) + 2.0 / (2 * window)) * rb + (8 + 4 * k) + 4 * (k + 1)


def code_hash(*names: str) -> str:
    """sha256 over C++ sources (comments and white space removed: edits to comments do not
    change it, edits to the code do) and the compiler flags the library is built with."""
    import re
    from paper_2407_15452_amd import build as gs_build
    h = hashlib.sha256()
    for name in names:
        text = open(os.path.join(CSRC, name), encoding="utf-8").read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        text = re.sub(r"//[^\n]*", "", text)
        h.update(re.sub(r"\s+", "", text).encode())
    h.update(" ".join(gs_build.HIPCC_FLAGS).encode())
    return h.hexdigest()


def stored_record(workload_name: str, hash_field: str, *sources: str):
    """Counter record of a committed rocprofv3 run for this workload, or None when there is
    none or the kernels it was taken on have changed since."""
    try:
        rec = json.load(open(TRAFFIC_FILE))[workload_name]
        return rec if rec.get(hash_field) == code_hash(*sources) else None
    except (OSError, KeyError, ValueError):
        return None


def traffic_record(workload_name: str):
    return stored_record(workload_name, "sgns_code_sha256", "sgns.hip", "common.h")


def walk_record(workload_name: str):
    rec = stored_record(workload_name, "walk_code_sha256", "walk.hip", "common.h")
    return rec if rec and "walk_fetch_bytes_per_transition" in rec else None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=2)
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the graph (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the momentum / Adam / LINE / fused-negatives / get-put measurements")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device copy and one gather of 2^21 distinct random "
                         "rows (kernels of known traffic: references for the byte counters)")
    ap.add_argument("--walk-sample", type=int, default=4_000_000,
                    help="walks in the stand-alone walk-throughput launch")
    return ap.parse_args()


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    from paper_2407_15452_amd import binding as gs, inputs
    gs.lib()
    dev = "cuda:0"
    wl = inputs.WORKLOADS[args.workload]
    if args.scale != 1.0:
        wl = wl.scaled(args.scale)
    K, W = args.steps, args.warmup
    B, k, L, win = wl.batch_pairs, wl.num_neg, wl.walk_len, wl.window
    elem_bytes = 2 if wl.dtype == "bf16" else 4

    # ------------------------------------------------------------------ setup (untimed)
    t0 = time.time()
    src, dst, w = inputs.edge_list(wl, dev)
    flags = gs.GS_DROP_SELF_LOOPS | gs.GS_DEDUPE | (0 if wl.directed else gs.GS_SYMMETRIZE)
    g = gs.gs_csr_build(src, dst, w, wl.num_nodes, flags, wl.offset_bits)
    del src, dst, w
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    log(f"[setup] graph {wl.name}: N={wl.num_nodes} entries={g.num_entries} "
        f"({time.time() - t0:.1f}s)")
    t0 = time.time()
    row_alias = gs.gs_alias_build(g.offsets, g.weights) if wl.weighted else None
    noise_w = inputs.noise_weights(g.offsets)
    seg = torch.tensor([0, wl.num_nodes], dtype=torch.int64, device=dev)
    noise = gs.gs_alias_build(seg, noise_w)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    log(f"[setup] alias tables ({time.time() - t0:.1f}s)")
    # a lived-in context table (zero rows would make the first updates trivial)
    w_in, w_out = inputs.init_tables(wl.num_nodes, wl.dim, wl.init_seed, dev, wl.dtype,
                                     context_seed=wl.init_seed + 1)
    torch.cuda.empty_cache()

    if wl.node2vec:
        def walk_fn(st, base, out=None):
            return gs.gs_node2vec_walk(g, row_alias, st, L, wl.p, wl.q, wl.walk_seed, base, out)
    else:
        def walk_fn(st, base, out=None):
            return gs.gs_random_walk(g, row_alias, st, L, wl.walk_seed, base, out)

    # Walks needed per batch.  Undirected: a walk from a node with edges never
    # dies, so the yield is exact.  Directed: measured on a probe launch.
    P = inputs.pairs_per_full_walk(L, win)
    live = (g.offsets[1:] > g.offsets[:-1])
    live_frac = float(live.float().mean().item())
    if wl.directed:
        probe = inputs.walk_starts(wl.num_nodes, 0, 200_000, dev)
        _, _, n_probe = gs.gs_make_pairs(walk_fn(probe, 0), win)
        pairs_per_walk = max(n_probe / probe.numel(), 1e-3)
        del probe
    else:
        pairs_per_walk = P * live_frac
    total_steps = W + K

    def walks_for(pairs_needed, first_walk):
        """Starts of a walk range that yields at least `pairs_needed` pairs."""
        count = int(pairs_needed / pairs_per_walk * 1.05) + 64
        while True:
            st = inputs.walk_starts(wl.num_nodes, first_walk, count, dev)
            if wl.directed or int(live[st.long()].sum().item()) * P >= pairs_needed:
                return st
            count = int(count * 1.3) + 64

    starts_warm = walks_for(max(W, 1) * B, 0)
    starts_timed = walks_for(K * B, starts_warm.numel())
    n_max = max(starts_warm.numel(), starts_timed.numel())
    walks_buf = torch.empty((n_max, L), dtype=torch.int32, device=dev)
    cap = gs.pair_capacity(n_max, L, win)
    centers = torch.zeros(cap, dtype=torch.int32, device=dev)
    contexts = torch.zeros(cap, dtype=torch.int32, device=dev)
    n_pairs_dev = torch.zeros(1, dtype=torch.int64, device=dev)
    pairs_ws = torch.empty(max(256, gs.lib().gs_make_pairs_workspace_bytes(n_max)),
                           dtype=torch.uint8, device=dev)
    negs = torch.empty((B, k), dtype=torch.int32, device=dev)
    sgns_dtype = gs.GS_BF16 if wl.dtype == "bf16" else gs.GS_F32
    sgns_ws = torch.empty(gs.gs_sgns_step_workspace_bytes(B, wl.num_nodes, k, wl.dim, sgns_dtype),
                          dtype=torch.uint8, device=dev)
    losses = torch.zeros(total_steps, dtype=torch.float64, device=dev)
    lr = inputs.learning_rate(wl, 0, 1)
    ev = lambda: torch.cuda.Event(enable_timing=True)  # noqa: E731

    def run(starts, first_walk, steps, step0, pair_base, sgns_events=None, stage_events=None):
        """Walk + pairs for `steps` batches, then negatives + SGNS per batch."""
        nw = starts.numel()
        if stage_events is not None:
            stage_events["walk0"].record()
        wk = walk_fn(starts, first_walk, walks_buf[:nw])
        if stage_events is not None:
            stage_events["walk1"].record()
        gs.gs_make_pairs(wk, win, centers, contexts, n_pairs_dev, pairs_ws, sync=False)
        if stage_events is not None:
            stage_events["pairs1"].record()
        n_pairs = int(n_pairs_dev.item())          # the one host read of the chunk
        if n_pairs < steps * B:
            raise RuntimeError(f"walk chunk produced {n_pairs} pairs, need {steps * B}")
        for s in range(steps):
            lo = s * B
            gs.gs_sample_negatives(noise, wl.num_nodes, B, k, wl.neg_seed, pair_base + lo, negs)
            if sgns_events is not None:
                sgns_events[s][0].record()
            gs.gs_sgns_step(w_in, w_out, centers[lo:lo + B], contexts[lo:lo + B], negs, lr,
                            loss_out=losses[step0 + s:step0 + s + 1], ws=sgns_ws)
            if sgns_events is not None:
                sgns_events[s][1].record()
        return n_pairs

    if args.calibration_copy:
        a_ = torch.zeros(1 << 28, dtype=torch.float32, device=dev)   # 1 GiB
        b_ = torch.empty_like(a_)
        b_.copy_(a_)
        torch.cuda.synchronize()
        del a_, b_
        # 2^21 distinct random rows of the input table into a dense block (gs_get_rows): reads
        # 2^21 * row bytes at random, writes 2^21 * dim * 4 bytes in a stream
        n_cal = min(1 << 21, wl.num_nodes)
        ids_cal = torch.randperm(wl.num_nodes, device=dev, generator=torch.Generator(dev).manual_seed(1))
        ids_cal = ids_cal[:n_cal].to(torch.int32).contiguous()
        blk_cal = torch.empty((n_cal, wl.dim), dtype=torch.float32, device=dev)
        gs.gs_get_rows(w_in, ids_cal, out=blk_cal)
        torch.cuda.synchronize()
        del ids_cal, blk_cal

    # ------------------------------------------------------------------ warm-up + timed region
    if W > 0:
        run(starts_warm, 0, W, 0, 0)
    torch.cuda.synchronize()
    sgns_events = [(ev(), ev()) for _ in range(K)]
    stage_events = {n: ev() for n in ("walk0", "walk1", "pairs1")}
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    run(starts_timed, starts_warm.numel(), K, W, W * B, sgns_events, stage_events)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start

    ms_per_step = elapsed * 1e3 / K
    pairs_per_s = K * B / elapsed
    sgns_ms = float(np.mean([a.elapsed_time(b) for a, b in sgns_events]))
    walk_ms = stage_events["walk0"].elapsed_time(stage_events["walk1"])
    pairs_ms = stage_events["walk1"].elapsed_time(stage_events["pairs1"])
    mean_loss = float(losses[W:].sum().item()) / (K * B)
    bpp = sgns_bytes_per_pair(k, wl.dim, elem_bytes, win)
    achieved = B * bpp / (sgns_ms * 1e-3) / 1e9

    # ------------------------------------------------------------------ stand-alone walk throughput
    nws = min(args.walk_sample, wl.num_nodes * wl.walks_per_node)
    st = inputs.walk_starts(wl.num_nodes, 0, nws, dev)
    big = torch.empty((nws, L), dtype=torch.int32, device=dev)
    walk_fn(st, 0, big)
    torch.cuda.synchronize()
    e0, e1 = ev(), ev()
    e0.record()
    walk_fn(st, 0, big)
    e1.record()
    torch.cuda.synchronize()
    walk_big_ms = e0.elapsed_time(e1)
    valid_steps = int((big[:, 1:] >= 0).sum().item())
    walk_steps_per_s = valid_steps / (walk_big_ms * 1e-3)
    del big

    # ------------------------------------------------------------------ extra measurements
    # (other entry points on the same tables and batches; --no-extras leaves them out, e.g. for
    # a kernel profile of the timed path alone)
    momentum_ms = adam_ms = fused = line = storage = from_walks_ms = small = shared = None
    if not args.no_extras:
        # ------------------------------------------------------------------ momentum variant (extra)
        # the paper's optimizer (dense mult / sparse put / dense mult_add); timed on the last batch
        if 2 * wl.num_nodes * wl.dim * elem_bytes <= 32e9:
            m_in, m_out = torch.zeros_like(w_in), torch.zeros_like(w_out)
            lo = (K - 1) * B
            for _ in range(2):
                gs.gs_sgns_momentum_step(w_in, w_out, m_in, m_out, centers[lo:lo + B],
                                         contexts[lo:lo + B], negs, lr, 0.9, loss_out=losses[:1],
                                         ws=sgns_ws)
            torch.cuda.synchronize()
            e0, e1 = ev(), ev()
            e0.record()
            for _ in range(5):
                gs.gs_sgns_momentum_step(w_in, w_out, m_in, m_out, centers[lo:lo + B],
                                         contexts[lo:lo + B], negs, lr, 0.9, loss_out=losses[:1],
                                         ws=sgns_ws)
            e1.record()
            torch.cuda.synchronize()
            momentum_ms = e0.elapsed_time(e1) / 5
            del m_in, m_out
        if wl.dtype == "f32" and 6 * wl.num_nodes * wl.dim * 4 <= 48e9:
            # throw-away copies: Adam's unit-sized steps would disturb the tables the later extras read
            a_tabs = [w_in.clone(), w_out.clone()] + [torch.zeros_like(w_in) for _ in range(4)]
            lo = (K - 1) * B
            adam = lambda t: gs.gs_sgns_adam_step(*a_tabs, centers[lo:lo + B], contexts[lo:lo + B], negs,  # noqa: E731
                                                  1e-3, 0.9, 0.999, 1e-8, t, loss_out=losses[:1],
                                                  ws=sgns_ws)
            for t in (1, 2):
                adam(t)
            torch.cuda.synchronize()
            e0, e1 = ev(), ev()
            e0.record()
            for t in range(3, 8):
                adam(t)
            e1.record()
            torch.cuda.synchronize()
            adam_ms = e0.elapsed_time(e1) / 5
            del a_tabs

        # ------------------------------------------------------------------ fused negatives (extra)
        # the same batches with the negatives drawn inside the step, against the two separate calls
        fused_ws = torch.empty(gs.gs_sgns_step_fused_workspace_bytes(B, wl.num_nodes, k, wl.dim, sgns_dtype),
                               dtype=torch.uint8, device=dev)

        def two_calls(j):
            gs.gs_sample_negatives(noise, wl.num_nodes, B, k, wl.neg_seed, pair_index_base=j * B, out=negs)
            gs.gs_sgns_step(w_in, w_out, centers[j * B:(j + 1) * B], contexts[j * B:(j + 1) * B], negs, lr,
                            loss_out=losses[:1], ws=sgns_ws)

        def one_call(j):
            gs.gs_sgns_step_fused(w_in, w_out, centers[j * B:(j + 1) * B], contexts[j * B:(j + 1) * B],
                                  noise, k, wl.neg_seed, lr, pair_index_base=j * B, loss_out=losses[:1],
                                  ws=fused_ws)

        fused = {}
        for name, fn in (("negatives_then_step_ms", two_calls), ("fused_step_ms", one_call)):
            for j in range(min(2, K)):
                fn(j)
            torch.cuda.synchronize()
            e0, e1 = ev(), ev()
            e0.record()
            for j in range(K):
                fn(j)
            e1.record()
            torch.cuda.synchronize()
            fused[name] = e0.elapsed_time(e1) / K
        del fused_ws

        # ------------------------------------------------------------------ pairs made in the step (extra)
        # gs_make_pairs + gs_sample_negatives + gs_sgns_step per batch against one
        # gs_sgns_step_from_walks per batch (gs_pair_offsets once per walk chunk), same batches
        nw_t = starts_timed.numel()
        wk_t = walks_buf[:nw_t]
        fw_ws = torch.empty(gs.gs_sgns_step_from_walks_workspace_bytes(B, wl.num_nodes, k, wl.dim, sgns_dtype),
                            dtype=torch.uint8, device=dev)
        offs = gs.gs_pair_offsets(wk_t, win)

        def from_walks(j):
            gs.gs_sgns_step_from_walks(w_in, w_out, wk_t, win, offs, j * B, B, noise, k, wl.neg_seed, lr,
                                       pair_index_base=j * B, loss_out=losses[:1], ws=fw_ws)

        def three_calls(j):
            if j == 0:
                gs.gs_make_pairs(wk_t, win, centers, contexts, n_pairs_dev, pairs_ws, sync=False)
            two_calls(j)

        from_walks_ms = {}
        for name, fn in (("make_pairs_negatives_step_ms", three_calls), ("from_walks_step_ms", from_walks)):
            for j in range(min(2, K)):
                fn(j)
            torch.cuda.synchronize()
            e0, e1 = ev(), ev()
            e0.record()
            if name == "from_walks_step_ms":
                gs.gs_pair_offsets(wk_t, win, out=offs)
            for j in range(K):
                fn(j)
            e1.record()
            torch.cuda.synchronize()
            from_walks_ms[name] = e0.elapsed_time(e1) / K
        del fw_ws, offs

        # ------------------------------------------------------------------ LINE batches (extra)
        # B sampled edges (uniform over the CSR entries) + negatives + the same step
        if True:
            lc = torch.empty(B, dtype=torch.int32, device=dev)
            lo_ = torch.empty(B, dtype=torch.int32, device=dev)

            lc_raw = torch.empty(B, dtype=torch.int32, device=dev)
            lo_raw = torch.empty(B, dtype=torch.int32, device=dev)
            sort_ws = torch.empty(gs.gs_sort_pairs_workspace_bytes(B), dtype=torch.uint8, device=dev)

            def sample_sorted(it):
                """B sampled edges, reordered by source id so that equal sources form runs."""
                gs.gs_sample_edges(g, None, B, wl.walk_seed ^ 0x4c494e45, sample_index_base=it * B,
                                   centers_out=lc_raw, contexts_out=lo_raw)
                gs.gs_sort_pairs(lc_raw, lo_raw, wl.num_nodes, centers_out=lc, contexts_out=lo_,
                                 ws=sort_ws)

            def line_batch(it):
                sample_sorted(it)
                gs.gs_sample_negatives(noise, wl.num_nodes, B, k, wl.neg_seed ^ 0x4c494e45,
                                       pair_index_base=it * B, out=negs)
                gs.gs_sgns_step(w_in, w_out, lc, lo_, negs, lr, loss_out=losses[:1], ws=sgns_ws)

            for it in range(2):
                line_batch(it)
            torch.cuda.synchronize()
            e0, e1 = ev(), ev()
            e0.record()
            for it in range(2, 7):
                line_batch(it)
            e1.record()
            torch.cuda.synchronize()
            line_ms = e0.elapsed_time(e1) / 5
            line = {"ms_per_batch": line_ms, "edges_per_s": B / (line_ms * 1e-3),
                    "what": "gs_sample_edges + gs_sort_pairs + gs_sample_negatives + gs_sgns_step per batch of "
                            "B edges"}
            # first order: the same batches on one table (a throw-away copy)
            if wl.num_nodes * wl.dim * elem_bytes <= 16e9:
                w_one = w_in.clone()
                l1_ws = torch.empty(gs.gs_line1_step_workspace_bytes(B, wl.num_nodes, k, wl.dim,
                                                                     sgns_dtype),
                                    dtype=torch.uint8, device=dev)

                def line1_batch(it):
                    sample_sorted(it)
                    gs.gs_sample_negatives(noise, wl.num_nodes, B, k, wl.neg_seed ^ 0x4c494e45,
                                           pair_index_base=it * B, out=negs)
                    gs.gs_line1_step(w_one, lc, lo_, negs, lr, loss_out=losses[:1], ws=l1_ws)

                for it in range(2):
                    line1_batch(it)
                torch.cuda.synchronize()
                e0, e1 = ev(), ev()
                e0.record()
                for it in range(2, 7):
                    line1_batch(it)
                e1.record()
                torch.cuda.synchronize()
                line["first_order_ms_per_batch"] = e0.elapsed_time(e1) / 5
                del w_one, l1_ws
            del lc, lo_, lc_raw, lo_raw, sort_ws

        # ------------------------------------------------------------------ get / put of a batch (extra)
        # the ids of the last batch: merge, fetch the block of distinct rows, add a block back
        lo = (K - 1) * B
        batch_ids = torch.cat([centers[lo:lo + B], contexts[lo:lo + B], negs.reshape(-1)])
        uniq_ws = torch.empty(gs.gs_unique_ids_workspace_bytes(batch_ids.numel(), wl.num_nodes), dtype=torch.uint8,
                              device=dev)
        uniq, ucount, _ = gs.gs_unique_ids(batch_ids, wl.num_nodes, ws=uniq_ws)
        n_uniq = int(ucount.item())
        block = torch.empty((n_uniq, wl.dim), dtype=torch.float32, device=dev)

        def timed(fn, reps=5):
            fn()
            torch.cuda.synchronize()
            a, b = ev(), ev()
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps

        unique_ms = timed(lambda: gs.gs_unique_ids(batch_ids, wl.num_nodes, ws=uniq_ws))
        get_ms = timed(lambda: gs.gs_get_rows(w_out, uniq[:n_uniq], out=block))
        put_ms = timed(lambda: gs.gs_put_rows(w_out, uniq[:n_uniq], block, 0.0))
        rb_blk = wl.dim * 4
        row_bytes = wl.dim * elem_bytes
        storage = {"batch_ids": int(batch_ids.numel()), "distinct": n_uniq, "unique_ms": unique_ms,
                   "get_ms": get_ms, "get_GBps": n_uniq * (row_bytes + rb_blk) / get_ms / 1e6,
                   "put_ms": put_ms, "put_GBps": n_uniq * (2 * row_bytes + rb_blk) / put_ms / 1e6}
        del block, uniq_ws, batch_ids

        # ------------------------------------------------------------------ shared negatives (extra)
        # A variant of the method, not the timed configuration: every pair of a run of equal
        # centres (one centre position of a walk) uses the negatives drawn for the run's first
        # pair.  Same call, same kernels; the rows of a run's negatives are then gathered once
        # from HBM and found in the L2 for the other pairs of the run.
        cb = centers[lo:lo + B]
        starts_run = torch.ones(B, dtype=torch.bool, device=dev)
        starts_run[1:] = cb[1:] != cb[:-1]
        first_of_run = torch.nonzero(starts_run).flatten()
        shared_negs = negs[first_of_run[torch.cumsum(starts_run, 0) - 1]].contiguous()
        shared = {"runs": int(first_of_run.numel()),
                  "step_ms": timed(lambda: gs.gs_sgns_step(w_in, w_out, cb, contexts[lo:lo + B], shared_negs, lr,
                                                           loss_out=losses[:1], ws=sgns_ws))}
        del shared_negs, starts_run, first_of_run

        # ------------------------------------------------------------------ small batches (extra)
        # 2048 pairs on the same graph: the regime where a step is a chain of short dependent
        # kernels; with a caller workspace and on the library's static scratch array
        small = None
        if wl.dim <= 256:
            sb = min(2048, B)
            sc, so_, sn = centers[lo:lo + sb], contexts[lo:lo + sb], negs[:sb]
            small_ws = torch.empty(gs.gs_sgns_step_workspace_bytes(sb, wl.num_nodes, k, wl.dim), dtype=torch.uint8,
                                   device=dev)
            small = {"pairs": sb,
                     "step_ms": timed(lambda: gs.gs_sgns_step(w_in, w_out, sc, so_, sn, lr, loss_out=losses[:1],
                                                              ws=small_ws), reps=50),
                     "static_step_ms": timed(lambda: gs.gs_sgns_step_static(w_in, w_out, sc, so_, sn, lr,
                                                                            loss_out=losses[:1]), reps=50)}
            del small_ws

    walk_kind = ("node2vec p=%g q=%g" % (wl.p, wl.q)) if wl.node2vec else "first-order"
    walk_kind += ", alias-weighted" if wl.weighted else ", uniform"
    result = {
        "metric": "SGNS positive pairs/sec + walk steps/sec; % of MI355X HBM peak",
        "value": pairs_per_s,
        "unit": "positive pairs/s (whole path: walks, pairs, negatives, SGNS step)",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if wl.dtype == "f32" else "bf16 storage, f32 arithmetic",
        "data": "synthetic",
        "config": {"workload": wl.name, "num_nodes": wl.num_nodes, "csr_entries": g.num_entries,
                   "offset_bits": wl.offset_bits, "batch_pairs": B, "negatives": k, "dim": wl.dim,
                   "walk_len": L, "window": win, "walk": walk_kind, "lr": lr,
                   "live_start_fraction": live_frac},
        "walk_steps_per_s": walk_steps_per_s,
        "walk_launch": {"walks": nws, "valid_steps": valid_steps, "ms": walk_big_ms},
        "stages_ms": {"walk_chunk": walk_ms, "pairs_chunk": pairs_ms, "sgns_step_mean": sgns_ms,
                      "chunk_walks": int(starts_timed.numel())},
        "mean_loss_per_pair": mean_loss,
        "momentum_step_ms": momentum_ms,
        "adam_step_ms": adam_ms,
        "fused_negatives": fused,
        "pairs_made_in_step": from_walks_ms,
        "line": line,
        "storage_ops": storage,
        "small_batch": small,
        "shared_negatives_per_run": shared,
        "roofline": {"bound": "hbm", "kernel": "gs_sgns_step (all kernels of one call)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "algorithmic_frac": achieved / HBM_PEAK_GBS,
                     "bytes_per_pair": bpp,
                     "what": "algorithmic (no-reuse) bytes of the batch-synchronous iteration over the "
                             "measured time of one call",
                     "traffic": None},
    }
    wrec = walk_record(wl.name)
    if wrec:
        # counter-measured bytes fetched per transition times the transition rate measured here
        rate = wrec["walk_fetch_bytes_per_transition"] * walk_steps_per_s / 1e9
        result["walk_roofline"] = {"bound": "hbm", "kernel": "node2vec / walk kernel, stand-alone launch",
                                   "achieved": rate, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                   "frac": rate / HBM_PEAK_GBS,
                                   "fetch_bytes_per_transition": wrec["walk_fetch_bytes_per_transition"],
                                   "fetch_source": wrec.get("source", "profiles/") + " (stored; code hash matched)",
                                   "fetch_measured_in_this_run": False,
                                   "algorithmic_bytes_per_transition": 132,
                                   "algorithmic_frac": 132 * walk_steps_per_s / 1e9 / HBM_PEAK_GBS,
                                   "l2_hit_rate": wrec.get("walk_l2_hit_rate")}
    rec = traffic_record(wl.name)
    if rec:
        # Bytes per call that crossed the L2 -> fabric boundary (FETCH_SIZE + WRITE_SIZE of a
        # committed rocprofv3 counter run on the same kernels: stored, not measured in this run),
        # over the step time measured here.  Reads served by the Infinity Cache count in it: it
        # bounds the HBM traffic from above.
        rate = rec["hbm_bytes_per_call"] / (sgns_ms * 1e-3) / 1e9
        result["roofline"].update({
            "traffic": rec["hbm_bytes_per_call"], "traffic_GBps": rate, "traffic_frac": rate / HBM_PEAK_GBS,
            "traffic_what": "L2-miss traffic (L2 <-> fabric bytes; Infinity Cache hits included)",
            "traffic_source": rec.get("source", "profiles/") + " (stored; code hash matched)",
            "traffic_measured_in_this_run": False,
            "l2_hit_rate": rec.get("l2_hit_rate")})

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, g, row_alias, noise, w_in, w_out, lr)
    print(json.dumps(result), flush=True)


def cpu_baseline(wl, g, row_alias, noise, w_in, w_out, lr, target_pairs=2_000_000):
    """The CPU reference, as it stands, on a bounded sample of the same workload
    (single thread): walks for the sample, pairs, negatives, one SGNS iteration.
    The SGNS iteration runs on a compacted copy of the rows the sample names
    (an iteration touches no other row), so the tables need not fit on the host."""
    import oracle
    oracle.build()
    from paper_2407_15452_amd import inputs
    off = g.offsets.cpu().numpy()
    nb = g.nbrs.cpu().numpy()
    table = None if row_alias is None else (row_alias.prob.cpu().numpy(),
                                            row_alias.alias.cpu().numpy())
    noise_t = (noise.prob.cpu().numpy(), noise.alias.cpu().numpy())
    P = inputs.pairs_per_full_walk(wl.walk_len, wl.window)
    live_frac = float((np.diff(off) > 0).mean())
    nw = int(target_pairs / P / max(live_frac, 1e-3)) + 8
    starts = inputs.walk_starts(wl.num_nodes, 0, nw).numpy()
    t0 = time.perf_counter()
    if wl.node2vec:
        walks = oracle.node2vec_walk(off, nb, starts, wl.walk_len, wl.p, wl.q, wl.walk_seed,
                                     alias=table)
    else:
        walks = oracle.random_walk(off, nb, starts, wl.walk_len, wl.walk_seed, alias=table)
    t1 = time.perf_counter()
    c, o = oracle.make_pairs(walks, wl.window)
    neg = oracle.sample_negatives(noise_t, wl.num_nodes, c.size, wl.num_neg, wl.neg_seed)
    t2 = time.perf_counter()
    # compact the named rows (untimed: it stands for tables that are already resident)
    ids, inv = np.unique(np.concatenate([c, o, neg.ravel()]), return_inverse=True)
    inv = inv.astype(np.int32)
    cc, oo, nn = inv[:c.size], inv[c.size:2 * c.size], inv[2 * c.size:].reshape(neg.shape)
    sel = torch.as_tensor(ids, dtype=torch.long, device=w_in.device)
    if wl.dtype == "bf16":
        h_in = w_in[sel].view(torch.int16).cpu().numpy().view(np.uint16).copy()
        h_out = w_out[sel].view(torch.int16).cpu().numpy().view(np.uint16).copy()
        dt = oracle.BF16
    else:
        h_in, h_out, dt = w_in[sel].cpu().numpy(), w_out[sel].cpu().numpy(), oracle.F32
    t3 = time.perf_counter()
    oracle.sgns_step(h_in, h_out, cc, oo, nn, lr, dtype=dt)
    t4 = time.perf_counter()
    steps = int((walks[:, 1:] >= 0).sum())
    secs = (t2 - t0) + (t4 - t3)
    return {"value": c.size / secs, "unit": "positive pairs/s (whole path)", "cores": 1,
            "kind": "oracle",
            "sample": f"{nw} walks -> {c.size} pairs of {wl.name}, one SGNS iteration over them",
            "walk_steps_per_s": steps / max(t1 - t0, 1e-9),
            "sgns_pairs_per_s": c.size / max(t4 - t3, 1e-9),
            "seconds": secs, "host_cpus": os.cpu_count()}


if __name__ == "__main__":
    main()
