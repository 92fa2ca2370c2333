#!/usr/bin/env python3
"""Benchmark of the COMM-RAND hot path on one MI355X.

A step is one mini-batch through the whole path: (root partitioning once per epoch,) grouped
sub-graph sampling, feature gather + mean aggregation, SAGE projections on the matrix cores, loss,
backward and SGD.  Inputs (graph, feature table, labels, weights) are resident in HBM before the
timed region.  Prints ONE JSON line.

The default workload is the largest single-GPU configuration: the papers100M-shaped graph (111 M nodes,
3.2 G adjacency entries, 28 GB bf16 feature table), generated on the GPU before the timed region.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload papers|products|reddit|arxiv|tiny]
                    [--scale S] [--group G] [--no-sweep] [--grid] [--no-cpu-baseline] [--no-input-stats]
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

HBM_PEAK_GBPS = 8000.0
METRIC = "epoch time + gathered-feature GB/s (% HBM peak) vs randomness knob, 1 MI355X"


def gather0_bytes(hdr0, n_feat, elem_bytes, f_pad):
    """Algorithmic bytes of one mini-batch's share of a layer-0 gather/aggregate launch: every gathered row
    (neighbours and the destination's own row) once, 4 bytes of index per edge (its global id), 4 bytes per
    destination for its own id, the row pointers, and the two bf16 outputs (self rows, aggregated rows)."""
    n_dst, n_src, nnz = int(hdr0[0]), int(hdr0[1]), int(hdr0[2])
    reads = (nnz + n_dst) * n_feat * elem_bytes + 4 * nnz + 4 * n_dst + 4 * (n_dst + 1)
    writes = 2 * n_dst * f_pad * 2
    return reads + writes, (nnz + n_dst) * n_feat * elem_bytes


def run_setting(tr, policy, mix, p, steps, warmup, epoch0, serial="none", input_stats=True):
    """Times `steps` steps (after `warmup` untimed ones) of one knob setting."""
    import torch
    from paper_2504_18082_amd import binding as B
    stats = dict(gather_bytes=0, feat_bytes=0, rows0=0, launches=0)

    def run(n_steps, epoch, timed):
        # whole epochs (root partitioning, then the batches group by group) until n_steps steps are done
        done = 0
        collect = (lambda n, slot: hdrs.append((n, tr.block_slots[slot][0].hdr.clone()))) if timed else None
        while done < n_steps:
            if serial == "none":
                nb = tr.build_batches(policy, mix, epoch)
                first = 0
                while first < min(nb, n_steps - done):
                    n = min(tr.G, min(nb, n_steps - done) - first)
                    tr.sample_group(first, n, p, epoch, slot=0)
                    for g in range(n):
                        tr.train_batch(g, slot=0)
                    if collect:
                        collect(n, 0)
                    first += n
                done += first
            else:
                done += tr.run_epoch(policy, mix, p, epoch, max_batches=n_steps - done, on_group=collect,
                                     gather_on_side_stream=(serial == "all"), weights_on_side_stream=(serial in ("sample+weights", "all")))
            epoch += 1
        return epoch

    hdrs = []
    tr.time_gather0 = False
    run(warmup, epoch0, False)
    torch.cuda.synchronize()
    tr.time_gather0 = True
    tr.gather0_events = []
    t0 = time.perf_counter()
    run(steps, epoch0 + 1000, True)
    t_enq = time.perf_counter()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    tr.time_gather0 = False
    stats["enqueue_s"] = t_enq - t0
    gather_ms = sum(a.elapsed_time(b) for a, b in tr.gather0_events)
    elem = 2 if tr.feat_dtype == B.CR_BF16 else 4
    for n, h in hdrs:
        h = h.cpu().numpy()
        for g in range(n):
            tot, feat = gather0_bytes(h[g], tr.cfg.n_feat, elem, tr.layers[0].F_pad)
            stats["gather_bytes"] += tot
            stats["feat_bytes"] += feat
            stats["rows0"] += int(h[g][2]) + int(h[g][0])
            stats["launches"] += 1
    # distinct input nodes per batch: counted outside the timed region (a training step does not need them)
    mean_input_nodes, unique_row_ratio = tr.input_node_stats(policy, mix, p, epoch0 + 1000) if input_stats else (float("nan"), float("nan"))
    # one launch of the layer-0 gather serves one mini-batch, or (grouped gather) every mini-batch of a sampled group
    n_launch = max(1, len(tr.gather0_events))
    n_batches = max(1, stats["launches"])
    return dict(ms_per_step=dt * 1e3 / steps, total_s=dt, host_enqueue_ms_per_step=stats["enqueue_s"] * 1e3 / steps,
                gather_ms_per_launch=gather_ms / n_launch, gather_bytes_per_launch=stats["gather_bytes"] / n_launch,
                gather_ms_per_batch=gather_ms / n_batches, batches_per_launch=n_batches / n_launch,
                feat_bytes_per_step=stats["feat_bytes"] / n_batches,
                unique_row_ratio=unique_row_ratio, mean_input_nodes=mean_input_nodes)


def cpu_baseline(w, n_batches_sample, seed, all_cores=False):
    """The oracle as it stands on the first batches of a fully random epoch: one thread (the oracle proper), or the
    same source built with OpenMP (row loops over all host cores).  Returns the record with per-stage seconds."""
    import oracle
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from oracle_step import StageTimers, oracle_train_step
    from paper_2504_18082_amd import synth
    cfg = w.cfg
    threads = oracle.use_all_cores(all_cores)
    try:
        params = [(W.astype(np.float64), b.astype(np.float64)) for W, b in synth.init_weights(cfg, seed)]
        pos = np.full(cfg.n_nodes, -1, dtype=np.int32)
        elem = 2 if w.features.dtype == np.uint16 else 4
        tm = StageTimers()
        t0 = time.perf_counter()
        perm = oracle.build_batches(oracle.RAND, 1, seed, 0, w.train_ids, w.comm, cfg.n_comm)
        tm.add("build_batches (per epoch)", t0)
        t_batches = time.perf_counter() - t0
        feat_bytes = 0
        t0 = time.perf_counter()
        for b in range(n_batches_sample):
            roots = perm[b * cfg.batch_size:(b + 1) * cfg.batch_size]
            ref = oracle_train_step(w.graph, w.features, cfg.n_feat, w.labels, roots, cfg.fanouts, 0.5, seed, 0, b, params, 0.01, 5e-4, pos,
                                    timers=tm)
            params = ref["params"]
            feat_bytes += (ref["blocks"][0].nnz + ref["blocks"][0].n_dst) * cfg.n_feat * elem
        dt = time.perf_counter() - t0
    finally:
        oracle.use_all_cores(False)
    n_epoch_batches = -(-len(w.train_ids) // cfg.batch_size)
    step_ms = dt * 1e3 / n_batches_sample
    return dict(value=round(feat_bytes / dt / 1e9, 5), unit="GB/s", cores=threads,
                kind="oracle" if not all_cores else "oracle source built with OpenMP (row loops over all cores)",
                sample=f"{n_batches_sample} mini-batch(es) of the same workload through the whole path (RAND roots, p=0.5): "
                       f"{dt:.1f} s; root partitioning of the epoch {t_batches:.2f} s on top",
                ms_per_step=round(step_ms, 1),
                epoch_s_extrapolated=round(t_batches + step_ms * 1e-3 * n_epoch_batches, 1),
                stage_s={k: round(v, 3) for k, v in tm.items()})


GRID_POLICIES = (("RAND-ROOTS", "rand", None), ("COMM-RAND-MIX-50%", "mix", 50.0), ("COMM-RAND-MIX-25%", "mix", 25.0),
                 ("COMM-RAND-MIX-12.5%", "mix", 12.5), ("COMM-RAND-MIX-0%", "mix", 0.0), ("NORAND-ROOTS", "norand", None))
GRID_P = (0.5, 0.9, 1.0)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="papers", help="papers (default: the largest single-GPU configuration) | products | reddit | arxiv | tiny")
    ap.add_argument("--generator", default="auto", choices=["auto", "gpu", "host"],
                    help="where the synthetic workload is generated (auto: on the GPU from 5 M edges on)")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload's node / edge / community counts by this factor")
    ap.add_argument("--group", type=int, default=32)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--grid", action="store_true",
                    help="also time the paper's whole grid of settings: six root policies x p in {0.5, 0.9, 1.0} (Section 5, evaluated schemes)")
    ap.add_argument("--grid-steps", type=int, default=256)
    ap.add_argument("--no-input-stats", action="store_true",
                    help="skip the untimed extra sampling pass that counts the distinct input nodes per batch (keeps a "
                         "kernel trace down to the timed path)")
    ap.add_argument("--row-order", default="auto", choices=["auto", "on", "off"],
                    help="process the input-side block's rows in community order (auto: when a batch holds >= 32 rows per community)")
    ap.add_argument("--overlap", default="none", choices=["none", "sample", "sample+weights", "all"],
                    help="side streams: 'sample' = sampling of the next group overlaps training; '+weights' = weight "
                         "gradients and SGD leave the backward pass's critical path; 'all' = also the layer-0 gather "
                         "(default none: every call on one stream, which keeps the per-kernel timing clean)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-batches", type=int, default=1)
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (the whole graph and feature table are resident in one "
              "MI355X's HBM; no collectives are part of it). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2504_18082_amd import binding as B
    from paper_2504_18082_amd import synth
    from paper_2504_18082_amd.trainer import Trainer
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.lib()                                   # fail loudly if the HIP library was not built

    wl_cfg = synth.CONFIGS[args.workload]
    if args.scale != 1.0:
        wl_cfg = synth.scaled(wl_cfg, args.scale)
    # the large shapes are generated on the GPU (set-up, untimed); the two small ones on the host, as the tests do
    on_gpu = args.generator == "gpu" or (args.generator == "auto" and wl_cfg.n_edges_undirected > 5_000_000)
    t_gen = time.perf_counter()
    if on_gpu:
        from paper_2504_18082_amd import synth_gpu
        w = synth_gpu.make_workload_gpu(wl_cfg, seed=args.seed, verbose=True)
        torch.cuda.synchronize()
    else:
        w = synth.make_workload(wl_cfg, seed=args.seed)
    t_gen = time.perf_counter() - t_gen
    cfg = w.cfg
    n_entries = int(w.indices.numel()) if on_gpu else len(w.indices)
    tr = Trainer(w, group_size=args.group, lr=0.01, weight_decay=5e-4, seed=args.seed,
                 order_rows={"auto": "auto", "on": True, "off": False}[args.row_order])
    steps = args.steps if args.steps is not None else tr.n_batches          # default: one epoch
    c_train = w.n_comm_in_train if on_gpu else int(len(np.unique(w.comm[w.train_ids])))
    mix_of = lambda percent: B.cr_mix_count_from_percent(percent, c_train)

    if args.calibration_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")       # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # headline: the fully random setting (RAND-ROOTS, p = 0.5), the paper's baseline
    main_res = run_setting(tr, B.CR_ROOTS_RAND, 1, 0.5, steps, args.warmup, 0, args.overlap, not args.no_input_stats)
    sweep = []

    def sweep_row(name, r):
        return dict(setting=name, ms_per_step=round(r["ms_per_step"], 4), epoch_ms=round(r["ms_per_step"] * tr.n_batches, 3),
                    speedup_vs_random=round(main_res["ms_per_step"] / r["ms_per_step"], 3),
                    gather_GBps=round(r["gather_bytes_per_launch"] / r["gather_ms_per_launch"] / 1e6, 1),
                    gather_us=round(r["gather_ms_per_batch"] * 1e3, 2),
                    mean_input_nodes=None if r["mean_input_nodes"] != r["mean_input_nodes"] else round(r["mean_input_nodes"], 1),
                    unique_row_ratio=None if r["unique_row_ratio"] != r["unique_row_ratio"] else round(r["unique_row_ratio"], 4))

    if not args.no_sweep:
        for name, policy, mix, p in (("mid: COMM-RAND-MIX-12.5% p=1.0", B.CR_ROOTS_COMM_RAND, mix_of(12.5), 1.0),
                                     ("fully community: NORAND-ROOTS p=1.0", B.CR_ROOTS_NORAND, 1, 1.0)):
            sweep.append(sweep_row(name, run_setting(tr, policy, mix, p, steps, min(args.warmup, 4), 50, args.overlap, not args.no_input_stats)))
    grid = []
    if args.grid:
        gsteps = min(args.grid_steps, tr.n_batches)
        for pname, kind, percent in GRID_POLICIES:
            policy = {"rand": B.CR_ROOTS_RAND, "mix": B.CR_ROOTS_COMM_RAND, "norand": B.CR_ROOTS_NORAND}[kind]
            mix = mix_of(percent) if kind == "mix" else 1
            for p in GRID_P:
                r = run_setting(tr, policy, mix, p, gsteps, 4, 100, args.overlap, not args.no_input_stats)
                row = sweep_row(f"{pname} p={p}", r)
                row["steps"] = gsteps
                grid.append(row)
                print(f"# grid {row['setting']}: {row['ms_per_step']} ms/step, gather {row['gather_us']} us", file=sys.stderr, flush=True)

    algorithmic = main_res["gather_bytes_per_launch"] / main_res["gather_ms_per_launch"] / 1e6      # GB/s
    value = main_res["feat_bytes_per_step"] / main_res["ms_per_step"] / 1e6                           # GB/s over the whole step
    # HBM bytes per launch as rocprofv3's counters saw them: taken per mini-batch from the committed counter summary of
    # this workload (profiles/, its own run) and scaled to this run's launch size
    traffic, traffic_src = None, None
    tpath = os.path.join(ROOT, "profiles", f"gather_fwd_{args.workload}_hbm_traffic.txt")
    if os.path.exists(tpath) and args.scale == 1.0:
        per_batch = None
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_batch"):
                per_batch = float(line.split("=")[1])
        if per_batch is not None:
            traffic = round(per_batch * main_res["batches_per_launch"])
            traffic_src = f"profiles/{os.path.basename(tpath)}: counted bytes per mini-batch x this run's batches_per_launch"
    achieved, basis = algorithmic, "algorithmic bytes / HIP-event time"
    if algorithmic > HBM_PEAK_GBPS and traffic is not None:
        # a table that sits in the caches: requests are served on chip and algorithmic bytes per second say nothing
        # about the memory; price the launch by the bytes that were counted at the memory instead
        achieved = traffic / main_res["gather_ms_per_launch"] / 1e6
        basis = "counted HBM bytes / HIP-event time (algorithmic bytes exceed the HBM peak: the table is cache resident)"
    elem_name = "bf16" if cfg.feat_dtype == "bf16" else "f32"
    out = {
        "metric": METRIC,
        "value": round(value, 3),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": args.warmup,
        "ms_per_step": round(main_res["ms_per_step"], 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": f"{elem_name} feature rows summed in f32; bf16 MFMA operands, hidden activations and inter-kernel gradients; "
                 f"f32 accumulation, logits, loss and master weights",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.n_nodes} nodes, {n_entries} CSR entries, {cfg.n_feat}-d {cfg.feat_dtype} "
                               f"features, {len(cfg.fanouts)}-layer GraphSAGE-mean hidden {cfg.hidden}, fanout {cfg.fanouts}, "
                               f"batch {cfg.batch_size}, {tr.n_batches} batches/epoch",
                   "generated": f"{'on the GPU (torch)' if on_gpu else 'on the host (numpy)'} in {t_gen:.1f} s, "
                                f"{n_entries / (2.0 * cfg.n_edges_undirected):.4f} of the edge count asked for, "
                                f"{w.achieved_intra_fraction:.3f} intra-community",
                   "setting": "fully random: RAND-ROOTS p=0.5", "group_size": args.group,
                   "schedule": "one stream" if args.overlap == "none" else "side streams: " + args.overlap,
                   "row_order": ("layer-0 gather once per sampled group, rows of all its batches in community order" if tr.group_gather
                                 else "input-side rows processed in community order" if tr.order_rows
                                 else "input-side rows processed in block order"),
                   "value_definition": "layer-0 gathered feature bytes per second of whole-step time"},
        "epoch_ms": round(main_res["ms_per_step"] * tr.n_batches, 3),
        "host_enqueue_ms_per_step": round(main_res["host_enqueue_ms_per_step"], 4),
        "mean_input_nodes": None if main_res["mean_input_nodes"] != main_res["mean_input_nodes"] else round(main_res["mean_input_nodes"], 1),
        "unique_row_ratio": None if main_res["unique_row_ratio"] != main_res["unique_row_ratio"] else round(main_res["unique_row_ratio"], 4),
        "roofline": {"bound": "hbm", "kernel": "gather_mean_fwd_kernel (layer 0)", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "basis": basis,
                     "traffic": traffic, "traffic_source": traffic_src,
                     "algorithmic_GBps": round(algorithmic, 1),
                     "cache_amplification": None if not traffic else round(main_res["gather_bytes_per_launch"] / traffic, 3),
                     "bytes_per_launch": round(main_res["gather_bytes_per_launch"]),
                     "us_per_launch": round(main_res["gather_ms_per_launch"] * 1e3, 2),
                     "us_per_batch": round(main_res["gather_ms_per_batch"] * 1e3, 2),
                     "batches_per_launch": round(main_res["batches_per_launch"], 2)},
        "sweep": sweep,
    }
    if grid:
        out["grid"] = grid
    if not args.no_cpu_baseline:
        t0 = time.perf_counter()
        hw = w.host() if on_gpu else w
        t_copy = time.perf_counter() - t0
        out["cpu_baseline"] = cpu_baseline(hw, args.cpu_batches, args.seed)
        if on_gpu:
            out["cpu_baseline"]["sample"] += f"; inputs copied from the GPU in {t_copy:.1f} s (untimed)"
        out["cpu_baseline"]["host"] = _host_name()
        out["cpu_baseline_all_cores"] = cpu_baseline(hw, args.cpu_batches, args.seed, all_cores=True)
    print(json.dumps(out))


def _host_name():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return f"{line.split(':', 1)[1].strip()}, {os.cpu_count()} logical CPUs visible"
    except OSError:
        pass
    return f"{os.cpu_count()} logical CPUs visible"


if __name__ == "__main__":
    main()
