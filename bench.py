#!/usr/bin/env python3
"""Benchmark of the MI355X training step: edges/sec on one GPU, roofline of the dominant
kernel, and the CPU oracle timed beside it.

A step is one pass of the whole hot path over one batch: negative sampling, unique-row
index, row gather, score block + softmax + both gradient contractions on the matrix cores,
chain rule, per-row reduce and the sparse Adagrad scatter.  All inputs (edge list, tables)
are resident in device memory before the timed region.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3       # MI355X dense fp32 matrix peak
PEAK_HBM_GBS = 8000.0
# HBM bytes of the two contraction passes of one full kg_small step, from the rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE runs summarised in profiles/traffic_k_flash_kg_small.md (counters scaled by a 1 GiB copy).
MEASURED_FLASH_TRAFFIC = {"kg_small": 238.0e6}


def oracle_baseline(w, es, er, ed, budget_s=15.0):
    """Times the oracle (numpy fp64, as it stands) on whole steps of the same workload.  The cost of a step
    depends on the batch geometry and the row width, not on the table size: tables too large to build on
    the host are replaced by a 2 M-row table and the ids are folded into it (said in `sample`)."""
    import numpy as np
    from oracle import sampling, step as ostep
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    V = w.num_nodes
    note = ""
    if V * w.dim > 400_000_000:
        V = 2_000_000
        note = ", node table reduced to 2 M rows (ids folded)"
        es, ed = es % V, ed % V
    rng = np.random.default_rng(w.seed)
    ne = (rng.standard_normal((V, w.dim), dtype=np.float32) * np.float32(w.init_std))
    re_ = (rng.standard_normal((w.num_rels, w.dim), dtype=np.float32) * np.float32(w.init_std))
    ns, rs = np.zeros_like(ne), np.zeros_like(re_)
    edges = 0
    steps = 0
    t_total = 0.0
    i = 0
    last_note = time.perf_counter()
    while True:
        lo, hi = i * w.batch_size, min((i + 1) * w.batch_size, es.shape[0])
        t0 = time.perf_counter()
        nsrc, ndst = sampling.sample_negatives(w.seed, i, V, es, ed, w.num_chunks, w.negs_per_chunk,
                                               w.deg_negs_per_chunk)
        ostep.train_batch(w.model, np.float32(w.lr), np.float32(w.eps), w.chunk_size, ne, ns, re_, rs,
                          es[lo:hi], er[lo:hi], ed[lo:hi], nsrc, ndst)
        dt = time.perf_counter() - t0
        if time.perf_counter() - last_note > 20.0:          # a sign of life during long CPU work
            sys.stderr.write("cpu baseline: oracle step %d took %.2f s\n" % (i, dt)); sys.stderr.flush()
            last_note = time.perf_counter()
        if i > 0:                       # first step is warm-up (BLAS thread start, page faults)
            t_total += dt; edges += hi - lo; steps += 1
        i += 1
        if (steps >= 3 and t_total >= budget_s) or steps >= 40 or (i + 1) * w.batch_size > es.shape[0]:
            break
    return dict(value=edges / t_total, unit="edges/s", cores=int(threads), kind="oracle",
                sample="%d whole steps of workload %s (batch %d) after 1 warm-up step, numpy fp64%s" % (steps, w.name, w.batch_size, note))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="kg_small")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--edges", type=int, default=0, help="shorten the synthetic edge list (the per-step work is unchanged)")
    ap.add_argument("--nodes", type=int, default=0, help="shrink the node table (row width and batch geometry are unchanged)")
    ap.add_argument("--no-phase-events", action="store_true", help="time the steps without the per-phase HIP events")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import numpy as np
    import torch
    import synth
    import paper_2101_08358_amd as mar

    if not os.path.exists(mar.library_path()):
        from paper_2101_08358_amd import build
        build.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    w = synth.get_workload(args.workload)
    if args.edges:
        w = w.scaled(num_edges=args.edges)
    if args.nodes:
        w = w.scaled(num_nodes=args.nodes)
    src, rel, dst = synth.make_graph(w.num_nodes, w.num_rels, w.num_edges, w.node_zipf, w.rel_zipf, seed=w.seed,
                                     device=dev if w.num_edges > 10_000_000 else "cpu")
    d_src, d_rel, d_dst = src.to(dev), rel.to(dev), dst.to(dev)
    tr = mar.Trainer(w.num_nodes, w.num_rels, w.dim, w.model, w.batch_size, w.num_chunks, w.negs_per_chunk,
                     w.deg_negs_per_chunk, w.lr, w.eps, w.init_std, w.seed, device=dev)
    nb = (w.num_edges + w.batch_size - 1) // w.batch_size
    bounds = [(b * w.batch_size, min((b + 1) * w.batch_size, w.num_edges)) for b in range(nb)]
    batches = [(d_src[lo:hi], d_rel[lo:hi], d_dst[lo:hi], hi - lo) for lo, hi in bounds]

    def step(i):
        s, r, d, n = batches[i % nb]
        mar.mar_sample_negatives(tr.ctx, i, d_src, d_dst, w.num_edges, tr.neg_src, tr.neg_dst)
        mar.mar_train_batch(tr.ctx, s, r, d, n, tr.neg_src, tr.neg_dst, tr.loss, None)
        return n

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # Timed region: K steps; only the dominant kernel (the two contraction passes) carries HIP events
    # (two per launch, on the stream it is launched on) so that the events cost the step little.
    FLASH = (1 << 2) | (1 << 3)
    if not args.no_phase_events:
        mar.mar_profile_enable(tr.ctx, min(args.steps, 4096), FLASH)
    edges = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.warmup, args.warmup + args.steps):
        edges += step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    elapsed = t1 - t0
    if args.no_phase_events:
        flash_phase, prof_steps = [0.0] * mar.NUM_PHASES, 0
    else:
        flash_phase, prof_steps = mar.mar_profile_read(tr.ctx)
    loss = float(tr.loss.item())
    last_batch_edges = batches[(args.warmup + args.steps - 1) % nb][3]

    # edges covered by the profiled steps (the first prof_steps of the timed region)
    prof_edges = sum(batches[i % nb][3] for i in range(args.warmup, args.warmup + prof_steps))
    flash_ms = flash_phase[2] + flash_phase[3]
    algo_flops = 12.0 * prof_edges * w.negs_per_chunk * w.dim          # 3 contractions x 2 sides x 2 n N d
    achieved = algo_flops / (flash_ms * 1e-3) / 1e12 if flash_ms > 0 else 0.0
    flash_us = flash_ms / max(prof_steps, 1) * 1e3

    # A second, untimed pass with events on every phase for the per-phase report.
    all_steps = min(args.steps, 200)
    mar.mar_profile_enable(tr.ctx, all_steps, (1 << mar.NUM_PHASES) - 1)
    for i in range(args.warmup + args.steps, args.warmup + args.steps + all_steps):
        step(i)
    torch.cuda.synchronize()
    phase_ms, phase_steps = mar.mar_profile_read(tr.ctx)
    mar.mar_profile_enable(tr.ctx, 0, 0)

    # one extra step with debug outputs for the unique-row count behind the bandwidth figures
    s, r, d, n = batches[0]
    dbg, t = tr.make_debug(n)
    mar.mar_train_batch(tr.ctx, s, r, d, n, tr.neg_src, tr.neg_dst, tr.loss, dbg)
    torch.cuda.synchronize()
    nu = t["num_uniq"].cpu().numpy()
    U = int(nu[0] + nu[1])
    cn = w.num_chunks * w.negs_per_chunk
    n_occ = 3 * n + 2 * cn
    dk = (w.dim + 3) // 4 * 4
    per_step = lambda ms: ms / max(phase_steps, 1)
    gather_bytes = (3 * n + 2 * cn) * w.dim * 4 + (2 * n + 2 * cn) * dk * 4        # rows read + operands written
    scatter_bytes = n_occ * dk * 4 + U * w.dim * 16                                 # gradient rows read + theta/state r+w
    phases = {name: round(per_step(ms) * 1e3, 2) for name, ms in zip(mar.binding.PHASE_NAMES, phase_ms)}
    out = {
        "metric": "training edges/sec per MI355X; achieved HBM GB/s + MFMA util vs peak",
        "value": edges / elapsed,
        "unit": "edges/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "num_nodes": w.num_nodes, "num_rels": w.num_rels, "num_edges": w.num_edges,
                   "score": ["DistMult", "ComplEx", "TransE", "Dot"][w.model], "dim": w.dim, "batch": w.batch_size,
                   "chunks": w.num_chunks, "negs_per_chunk": w.negs_per_chunk, "deg_negs_per_chunk": w.deg_negs_per_chunk},
        "roofline": {"bound": "mfma", "kernel": "k_flash (pass 1 + pass 2 of every step)", "achieved": achieved,
                     "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_FP32_MFMA_TFLOPS,
                     "traffic": MEASURED_FLASH_TRAFFIC.get(w.name) if not (args.edges or args.nodes) else None,
                     "us_per_step": round(flash_us, 2),
                     "algorithmic_flops_per_step": 12.0 * w.batch_size * w.negs_per_chunk * w.dim},
        "phases_us_per_step": phases,
        "hbm_phases": {
            "gather": {"bytes": gather_bytes, "GB/s": gather_bytes / (per_step(phase_ms[1]) * 1e-3) / 1e9 if phase_ms[1] > 0 else None,
                       "peak": PEAK_HBM_GBS},
            "reduce_adagrad": {"bytes": scatter_bytes, "unique_rows": U,
                               "GB/s": scatter_bytes / (per_step(phase_ms[5]) * 1e-3) / 1e9 if phase_ms[5] > 0 else None,
                               "peak": PEAK_HBM_GBS}},
        "final_loss_per_edge": loss / last_batch_edges,
    }
    if not args.no_cpu_baseline:
        m = min(w.num_edges, 64 * w.batch_size)          # the oracle only walks the first batches
        out["cpu_baseline"] = oracle_baseline(w, src[:m].cpu().numpy(), rel[:m].cpu().numpy(), dst[:m].cpu().numpy())
    tr.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
