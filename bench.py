#!/usr/bin/env python3
"""Benchmark of the MI355X training step: edges/sec on one GPU, roofline of the dominant
kernel, and the CPU oracle timed beside it.

A step is one pass of the whole hot path over one batch: negative sampling, unique-row
index, row gather, score block + softmax + both gradient contractions on the matrix cores,
chain rule, per-row reduce and the sparse Adagrad scatter.  All inputs (edge list, tables)
are resident in device memory before the timed region.

With no arguments the headline is the largest workload that fits one GPU (`wide`: 50 M x 400
tables and accumulators, 160 GB, the full 500 M-edge list); the same record for the two
d = 100 workloads (`social`, `kg_large`; full-size tables, edge lists shortened as stated in
each record) rides along under "other_workloads".  `--workload NAME` measures one workload alone.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3       # MI355X dense fp32 matrix peak
PEAK_BF16_MFMA_TFLOPS = 2500.0      # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0
DEFAULT_STEPS = {"tiny": (300, 30), "kg_small": (500, 50), "social": (150, 15), "social_dot": (150, 15),
                 "kg_large": (150, 15), "wide": (100, 10)}


SPLIT_DTYPE = "bf16x3 (fp32 operands as bf16 hi + lo, three bf16 matrix products per product, fp32 accumulation)"


def note(msg):
    sys.stderr.write("bench: %s\n" % msg)
    sys.stderr.flush()


def measured_traffic(workload):
    """HBM bytes per launch of each kernel from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary committed as
    profiles/traffic_<workload>.md (`<workload>_split`: the same workload with the split-precision contraction) (table rows `| `kernel` | fetch MB | write MB | total MB |`).  Returns
    {kernel name without template arguments: bytes} or {} if there is no summary for this workload."""
    path = os.path.join(ROOT, "profiles", "traffic_%s.md" % workload)
    out = {}
    if not os.path.exists(path):
        return out
    for line in open(path):
        m = re.match(r"\|\s*`(k_[a-z_0-9]+)[^`]*`\s*\|.*\|\s*([0-9.]+)\s*\|\s*$", line)
        if m:
            out[m.group(1)] = out.get(m.group(1), 0.0) + float(m.group(2)) * 1e6
    return out


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
    extra = ""
    if V * w.dim > 400_000_000:
        V = 2_000_000
        extra = ", node table reduced to 2 M rows (ids folded)"
        es, ed = es % V, ed % V
    rng = np.random.default_rng(w.seed)
    ne = (rng.standard_normal((V, w.dim), dtype=np.float32) * np.float32(w.init_std))
    re_ = (rng.standard_normal((w.num_rels, w.dim), dtype=np.float32) * np.float32(w.init_std))
    ns, rs = np.zeros_like(ne), np.zeros_like(re_)
    edges = 0
    steps = 0
    t_total = 0.0
    i = 0
    while True:
        lo, hi = i * w.batch_size, min((i + 1) * w.batch_size, es.shape[0])
        t0 = time.perf_counter()
        nsrc, ndst = sampling.sample_negatives(w.seed, i, V, es, ed, w.num_chunks, w.negs_per_chunk,
                                               w.deg_negs_per_chunk)
        ostep.train_batch(w.model, np.float32(w.lr), np.float32(w.eps), w.chunk_size, ne, ns, re_, rs,
                          es[lo:hi], er[lo:hi], ed[lo:hi], nsrc, ndst)
        dt = time.perf_counter() - t0
        note("cpu baseline: oracle step %d took %.2f s" % (i, dt))
        if i > 0:                       # first step is warm-up (BLAS thread start, page faults)
            t_total += dt; edges += hi - lo; steps += 1
        i += 1
        if (steps >= 3 and t_total >= budget_s) or steps >= 40 or (i + 1) * w.batch_size > es.shape[0]:
            break
    return dict(value=edges / t_total, unit="edges/s", cores=int(threads), kind="oracle",
                sample="%d whole steps of workload %s (batch %d) after 1 warm-up step, numpy fp64%s" % (steps, w.name, w.batch_size, extra))


def run_workload(name, steps, warmup, edges=0, nodes=0, phase_events=True, cpu_baseline=False, precision=0, with_split=False):
    """Builds the workload's inputs on the device, times `steps` training steps and returns the record.
    precision 1: the split-precision contraction (config `precision`); with_split: after the fp32 measurement the
    same steps are timed again in split precision on the same tables and reported under "split_bf16"."""
    import torch
    import synth
    import paper_2101_08358_amd as mar

    dev = torch.device("cuda:0")
    w = synth.get_workload(name)
    full_edges = w.num_edges
    if edges and edges < w.num_edges:
        w = w.scaled(num_edges=edges)
    if nodes:
        w = w.scaled(num_nodes=nodes)
    t_build = time.perf_counter()
    src, rel, dst = synth.make_graph(w.num_nodes, w.num_rels, w.num_edges, w.node_zipf, w.rel_zipf, seed=w.seed,
                                     device=dev if w.num_edges > 10_000_000 else "cpu")
    d_src, d_rel, d_dst = src.to(dev), rel.to(dev), dst.to(dev)
    tr = mar.Trainer(w.num_nodes, w.num_rels, w.dim, w.model, w.batch_size, w.num_chunks, w.negs_per_chunk,
                     w.deg_negs_per_chunk, w.lr, w.eps, w.init_std, w.seed, device=dev, precision=precision)
    torch.cuda.synchronize()
    note("%s: %d edges, %.1f GB of tables built in %.1f s" % (w.name, w.num_edges, 2 * 4e-9 * w.dim * (w.num_nodes + w.num_rels),
                                                           time.perf_counter() - t_build))
    nb = (w.num_edges + w.batch_size - 1) // w.batch_size
    bounds = lambda b: (b * w.batch_size, min((b + 1) * w.batch_size, w.num_edges))

    def step(i, tr=tr):
        lo, hi = bounds(i % nb)
        mar.mar_sample_negatives(tr.ctx, i, d_src, d_dst, w.num_edges, tr.neg_src, tr.neg_dst)
        mar.mar_train_batch(tr.ctx, d_src[lo:hi], d_rel[lo:hi], d_dst[lo:hi], hi - lo, tr.neg_src, tr.neg_dst, tr.loss, None)
        return hi - lo

    def contraction_roofline(flash_phase, prof_steps, prof_edges, split):
        """Roofline record of the two contraction launches from their HIP-event times.  fp32: the algorithmic flops
        (3 contractions x 2 sides x 2 n N d) against the fp32 matrix peak.  Split precision: the bf16 flops executed
        (each pass computes the scores and one more product, every product as three bf16 products: 2 x 3 x 8 n N d)
        against the bf16 matrix peak; `fp32_equivalent` is the algorithmic rate."""
        per_launch = lambda ms: ms / max(prof_steps, 1) * 1e3                     # us per launch
        flops = lambda k: k * prof_edges * w.negs_per_chunk * w.dim / max(prof_steps, 1)
        tflops = lambda fl, us: fl / (us * 1e-6) / 1e12 if us > 0 else 0.0
        us1, us2 = per_launch(flash_phase[2]), per_launch(flash_phase[3])
        if not split:
            peak, k1, k2, names = PEAK_FP32_MFMA_TFLOPS, 8.0, 4.0, ("k_flash", "k_flash_bwd")
            kernel = "k_flash + k_flash_bwd (the two contraction launches of every step)"
        else:
            peak, k1, k2, names = PEAK_BF16_MFMA_TFLOPS, 24.0, 24.0, ("k_split_pass1", "k_split_pass2")
            kernel = "k_split<.., 1> + k_split<.., 2> (the two contraction launches of every step, split precision)"
        achieved = tflops(flops(k1 + k2), us1 + us2)
        r = {"bound": "mfma", "kernel": kernel, "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
             "traffic": None, "us_per_step": round(us1 + us2, 2),
             "algorithmic_flops_per_step": 12.0 * w.batch_size * w.negs_per_chunk * w.dim,
             names[0]: {"us": round(us1, 2), "flops": flops(k1), "frac": tflops(flops(k1), us1) / peak},
             names[1]: {"us": round(us2, 2), "flops": flops(k2), "frac": tflops(flops(k2), us2) / peak}}
        if split:
            r["executed_flops_per_step"] = 48.0 * w.batch_size * w.negs_per_chunk * w.dim
            r["fp32_equivalent_TFLOP/s"] = tflops(flops(12.0), us1 + us2)
        return r

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    # Timed region: K steps; only the dominant kernel (the two contraction passes) carries HIP events
    # (two per launch, on the stream it is launched on) so that the events cost the step little.
    FLASH = (1 << 2) | (1 << 3)
    if phase_events:
        mar.mar_profile_enable(tr.ctx, min(steps, 4096), FLASH)
    edges_done = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(warmup, warmup + steps):
        edges_done += step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    if phase_events:
        flash_phase, prof_steps = mar.mar_profile_read(tr.ctx)
    else:
        flash_phase, prof_steps = [0.0] * mar.NUM_PHASES, 0
    loss = float(tr.loss.item())
    last_batch_edges = bounds((warmup + steps - 1) % nb)[1] - bounds((warmup + steps - 1) % nb)[0]

    # edges covered by the profiled steps (the first prof_steps of the timed region)
    prof_edges = sum(bounds(i % nb)[1] - bounds(i % nb)[0] for i in range(warmup, warmup + prof_steps))
    roof = contraction_roofline(flash_phase, prof_steps, prof_edges, bool(precision))

    # A second, untimed pass with events on every phase for the per-phase report.
    all_steps = min(steps, 100)
    mar.mar_profile_enable(tr.ctx, all_steps, (1 << mar.NUM_PHASES) - 1)
    for i in range(warmup + steps, warmup + steps + all_steps):
        step(i)
    torch.cuda.synchronize()
    phase_ms, phase_steps = mar.mar_profile_read(tr.ctx)
    mar.mar_profile_enable(tr.ctx, 0, 0)

    # one extra step with debug outputs for the unique-row count behind the bandwidth figures
    lo, hi = bounds(0)
    n = hi - lo
    dbg, t = tr.make_debug(n)
    mar.mar_train_batch(tr.ctx, d_src[lo:hi], d_rel[lo:hi], d_dst[lo:hi], n, tr.neg_src, tr.neg_dst, tr.loss, dbg)
    torch.cuda.synchronize()
    nu = t["num_uniq"].cpu().numpy()
    U = int(nu[0] + nu[1])
    roles = 2 if w.model == 3 else 3
    cn = w.num_chunks * w.negs_per_chunk
    dk = (w.dim + 3) // 4 * 4
    per_step = lambda ms: ms / max(phase_steps, 1)
    gather_bytes = (roles * n + 2 * cn) * w.dim * 4 + (2 * n + 2 * cn) * dk * 4     # rows read + operands written
    scatter_bytes = (roles * n + 2 * cn) * dk * 4 + U * w.dim * 16                   # gradient rows read + theta/state r+w
    chain_bytes = n * (2 * dk + 2 * roles * w.dim) * 4                               # operand gradients + s/r/d read, gradient rows written
    phases = {nm: round(per_step(ms) * 1e3, 2) for nm, ms in zip(mar.binding.PHASE_NAMES, phase_ms)}
    traffic = measured_traffic(w.name + ("_split" if precision else "")) if not nodes else {}   # per-launch bytes do not depend on the edge list
    if not precision:
        roof["traffic"] = (traffic.get("k_flash", 0.0) + traffic.get("k_flash_bwd", 0.0)) or None
    else:
        roof["traffic"] = traffic.get("k_split", 0.0) or None
    # Bandwidth of the row phases two ways: algorithmic bytes (what the phase has to move) and the bytes the
    # rocprofv3 FETCH_SIZE / WRITE_SIZE counters saw per launch (profiles/traffic_<workload>.md), both over the
    # phase's time between HIP events on its stream.
    def phase(kernels, algo_bytes, ms, **extra):
        cb = sum(traffic.get(k, 0.0) for k in kernels) or None
        t = per_step(ms) * 1e-3
        d = {"kernel": " + ".join(kernels), "us": round(t * 1e6, 2), "bytes": algo_bytes,
             "GB/s": algo_bytes / t / 1e9 if t > 0 else None, "frac": algo_bytes / t / 1e9 / PEAK_HBM_GBS if t > 0 else None,
             "counter_bytes": cb, "counter_GB/s": cb / t / 1e9 if cb and t > 0 else None,
             "counter_frac": cb / t / 1e9 / PEAK_HBM_GBS if cb and t > 0 else None}
        d.update(extra)
        return d
    hbm_phases = {"gather": phase(("k_prep",), gather_bytes, phase_ms[1]),
                  "chain_rule": phase(("k_chain",), chain_bytes, phase_ms[4], note="runs on the second stream beside the second contraction pass"),
                  "reduce_adagrad": phase(("k_reduce_apply", "k_span_apply"), scatter_bytes, phase_ms[5], unique_rows=U),
                  "peak_GB/s": PEAK_HBM_GBS}
    cfg = {"workload": w.name, "num_nodes": w.num_nodes, "num_rels": w.num_rels, "num_edges": w.num_edges,
           "score": ["DistMult", "ComplEx", "TransE", "Dot"][w.model], "dim": w.dim, "batch": w.batch_size,
           "chunks": w.num_chunks, "negs_per_chunk": w.negs_per_chunk, "deg_negs_per_chunk": w.deg_negs_per_chunk,
           "table_bytes": 2 * 4 * w.dim * (w.num_nodes + w.num_rels)}
    if w.num_edges != full_edges:
        cfg["edge_list"] = "shortened from %d edges (the per-step work does not depend on the list's length)" % full_edges
    rec = {
        "value": edges_done / elapsed,
        "unit": "edges/s",
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": elapsed / steps * 1e3,
        "dtype": SPLIT_DTYPE if precision else "f32",
        "config": cfg,
        "roofline": roof,
        "phases_us_per_step": phases,
        "hbm_phases": hbm_phases,
        "final_loss_per_edge": loss / last_batch_edges,
    }
    if with_split and not precision and w.model != 2:
        # the same steps in split precision, on the same tables (a second context over them)
        tr2 = mar.Trainer(w.num_nodes, w.num_rels, w.dim, w.model, w.batch_size, w.num_chunks, w.negs_per_chunk,
                          w.deg_negs_per_chunk, w.lr, w.eps, w.init_std, w.seed, device=dev, node_emb=tr.node_emb,
                          rel_emb=tr.rel_emb, node_state=tr.node_state, rel_state=tr.rel_state, precision=1)
        for i in range(warmup):
            step(i, tr2)
        torch.cuda.synchronize()
        mar.mar_profile_enable(tr2.ctx, min(steps, 4096), FLASH)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        done2 = 0
        for i in range(warmup, warmup + steps):
            done2 += step(i, tr2)
        torch.cuda.synchronize()
        el2 = time.perf_counter() - t0
        fp2, ps2 = mar.mar_profile_read(tr2.ctx)
        pe2 = sum(bounds(i % nb)[1] - bounds(i % nb)[0] for i in range(warmup, warmup + ps2))
        mar.mar_profile_enable(tr2.ctx, all_steps, (1 << mar.NUM_PHASES) - 1)
        for i in range(warmup + steps, warmup + steps + all_steps):
            step(i, tr2)
        torch.cuda.synchronize()
        pm2, pst2 = mar.mar_profile_read(tr2.ctx)
        mar.mar_profile_enable(tr2.ctx, 0, 0)
        roof2 = contraction_roofline(fp2, ps2, pe2, True)
        if not nodes:
            roof2["traffic"] = measured_traffic(w.name + "_split").get("k_split") or None
        rec["split_bf16"] = {"value": done2 / el2, "unit": "edges/s", "steps": steps, "ms_per_step": el2 / steps * 1e3,
                             "dtype": SPLIT_DTYPE, "roofline": roof2,
                             "phases_us_per_step": {nm: round(ms / max(pst2, 1) * 1e3, 2) for nm, ms in zip(mar.binding.PHASE_NAMES, pm2)},
                             "final_loss_per_edge": float(tr2.loss.item()) / last_batch_edges,
                             "speedup_over_f32": (done2 / el2) / (edges_done / elapsed)}
        tr2.close()
        del tr2
    if cpu_baseline:
        m = min(w.num_edges, 64 * w.batch_size)          # the oracle only walks the first batches
        rec["cpu_baseline"] = oracle_baseline(w, src[:m].cpu().numpy(), rel[:m].cpu().numpy(), dst[:m].cpu().numpy())
    tr.close()
    del tr, d_src, d_rel, d_dst, src, rel, dst, dbg, t
    torch.cuda.empty_cache()
    return rec


def run_host_tables(name, depth, steps, warmup, nodes, edges):
    """Out-of-memory training (Sec. 3): node table and accumulators in pinned host memory, `depth` batches in
    flight.  Returns the record; the host link is what bounds it."""
    import torch
    import synth
    import paper_2101_08358_amd as mar

    dev = torch.device("cuda:0")
    w = synth.get_workload(name)
    w = w.scaled(num_nodes=nodes or min(w.num_nodes, 10_000_000), num_edges=edges or min(w.num_edges, 20_000_000))
    src, rel, dst = synth.make_graph(w.num_nodes, w.num_rels, w.num_edges, w.node_zipf, w.rel_zipf, seed=w.seed, device=dev)
    t0 = time.perf_counter()
    h_ne = torch.empty((w.num_nodes, w.dim), dtype=torch.float32, pin_memory=True)
    h_ns = torch.zeros((w.num_nodes, w.dim), dtype=torch.float32, pin_memory=True)
    step_rows = 1 << 20                                          # filled on the device, copied out in slices
    g = torch.Generator(device=dev); g.manual_seed(w.seed)
    for lo in range(0, w.num_nodes, step_rows):
        hi = min(lo + step_rows, w.num_nodes)
        h_ne[lo:hi].copy_(torch.randn((hi - lo, w.dim), device=dev, generator=g) * w.init_std)
    d_re = torch.randn((w.num_rels, w.dim), device=dev, generator=g) * w.init_std
    d_rs = torch.zeros((w.num_rels, w.dim), device=dev)
    cfg = mar.MarConfig(w.num_nodes, w.num_rels, w.dim, w.model, w.batch_size, w.num_chunks, w.negs_per_chunk,
                        w.deg_negs_per_chunk, w.lr, w.eps, w.init_std, w.seed)
    nbytes = mar.mar_pipe_workspace_bytes(cfg, depth)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    pipe = mar.mar_pipe_create(cfg, h_ne, h_ns, d_re, d_rs, ws, nbytes, depth)
    cn = w.num_chunks * w.negs_per_chunk
    negs = [[torch.empty(cn, dtype=torch.int32, device=dev) for _ in range(2)] for _ in range(depth + 1)]
    loss = torch.zeros(1, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    note("%s, host tables: %.1f GB pinned in %.1f s, workspace %.2f GB, depth %d" % (w.name, 8e-9 * w.dim * w.num_nodes,
                                                                                   time.perf_counter() - t0, nbytes / 1e9, depth))
    nb = w.num_edges // w.batch_size

    def step(i):
        lo = (i % nb) * w.batch_size
        ns_, nd_ = negs[i % (depth + 1)]                         # fresh uniform negatives; the buffers of the batches in flight stay untouched
        ns_.random_(0, w.num_nodes, generator=g); nd_.random_(0, w.num_nodes, generator=g)
        mar.mar_pipe_submit(pipe, src[lo:lo + w.batch_size], rel[lo:lo + w.batch_size], dst[lo:lo + w.batch_size], w.batch_size,
                            ns_, nd_, loss)

    for i in range(warmup):
        step(i)
    mar.mar_pipe_drain(pipe)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(warmup, warmup + steps):
        step(i)
    mar.mar_pipe_drain(pipe)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    final = float(loss.item()) / w.batch_size
    mar.mar_pipe_destroy(pipe)
    return {"value": steps * w.batch_size / dt, "unit": "edges/s", "ms_per_step": dt / steps * 1e3,
            "config": {"workload": "%s, node table and accumulators in pinned host memory, %d batches in flight" % (w.name, depth),
                       "num_nodes": w.num_nodes, "dim": w.dim, "batch": w.batch_size, "chunks": w.num_chunks,
                       "negs_per_chunk": w.negs_per_chunk, "negatives": "uniform ids (torch) drawn per step",
                       "host_table_bytes": 8 * w.dim * w.num_nodes},
            "final_loss_per_edge": final}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (default: per workload, about a second of GPU time)")
    ap.add_argument("--warmup", type=int, default=0)
    ap.add_argument("--workload", default="", help="measure this workload alone (default: wide, with social and kg_large beside it)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the records of the other workloads")
    ap.add_argument("--edges", type=int, default=0, help="shorten the synthetic edge list (the per-step work is unchanged)")
    ap.add_argument("--other-edges", type=int, default=100_000_000, help="edge-list length of the other workloads' records")
    ap.add_argument("--nodes", type=int, default=0, help="shrink the node table (row width and batch geometry are unchanged)")
    ap.add_argument("--no-phase-events", action="store_true", help="time the steps without the per-phase HIP events")
    ap.add_argument("--precision", choices=("f32", "split"), default="f32",
                    help="arithmetic of the two contraction passes of the measured record (default f32, the paper's)")
    ap.add_argument("--no-split", action="store_true", help="skip the split-precision record that rides along with every f32 record")
    ap.add_argument("--host-tables", type=int, default=0, metavar="DEPTH",
                    help="measure out-of-memory training instead: node table in pinned host memory, DEPTH batches in flight")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import torch
    import paper_2101_08358_amd as mar

    if not os.path.exists(mar.library_path()):
        from paper_2101_08358_amd import build
        build.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.host_tables:
        name = args.workload or "social"
        steps, warmup = args.steps or 60, args.warmup or 8
        rec = run_host_tables(name, args.host_tables, steps, warmup, args.nodes, args.edges)
        out = {"metric": "training edges/sec per MI355X, node table in host memory", "n_gpus": 1, "steps": steps, "warmup": warmup,
               "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic"}
        out.update(rec)
        print(json.dumps(out))
        return
    name = args.workload or "wide"
    steps, warmup = DEFAULT_STEPS.get(name, (100, 10))
    steps, warmup = args.steps or steps, args.warmup or warmup
    prec = 1 if args.precision == "split" else 0
    rec = run_workload(name, steps, warmup, args.edges, args.nodes, not args.no_phase_events, not args.no_cpu_baseline,
                       precision=prec, with_split=not args.no_split)
    out = {"metric": "training edges/sec per MI355X; achieved HBM GB/s + MFMA util vs peak",
           "value": rec["value"], "unit": "edges/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
           "ms_per_step": rec["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": rec["dtype"], "data": "synthetic"}
    for k in ("config", "roofline", "cpu_baseline", "phases_us_per_step", "hbm_phases", "final_loss_per_edge", "split_bf16"):
        if k in rec:
            out[k] = rec[k]
    if not args.workload and not args.no_others:
        out["other_workloads"] = {}
        for other in ("social", "kg_large"):
            s, wu = DEFAULT_STEPS[other]
            out["other_workloads"][other] = run_workload(other, s, wu, args.other_edges, precision=prec, with_split=not args.no_split)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
