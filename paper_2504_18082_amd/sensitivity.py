"""Sensitivity of COMM-RAND's per-step speed-up to the ratio of the feature table to the on-chip caches
(Section 6.5, sensitivity to on-chip cache capacity; Section 6.1's relation between per-epoch time and the
size of the input features a batch touches).  The paper shrinks the
cache with GPU partitions; here the cache stays (4 MB of L2 per XCD, 256 MB of memory-side cache) and the table
grows or shrinks: the same graph recipe at several node counts and feature widths.

    python -m paper_2504_18082_amd.sensitivity --workload arxiv --scales 0.25 1 4 16 --widths 128

Prints one JSON line per (scale, width): table size, ms per step and layer-0 gather time per mini-batch for the fully random
baseline and for two COMM-RAND settings, and the speed-ups over the baseline."""
from __future__ import annotations

import argparse
import copy
import json
import sys
import time

DEFAULT_SETTINGS = ["rand:0.5", "mix12.5:0.9", "mix0:1.0"]      # <root policy>:<p>, as in fit.py; the first is the baseline


def time_setting(tr, policy, mix, p, steps, warmup, epoch0):
    import torch

    def run(n_steps, epoch):
        done = 0
        while done < n_steps:
            done += tr.run_epoch_serial(policy, mix, p, epoch, max_batches=n_steps - done)
            epoch += 1

    tr.time_gather0 = False
    run(warmup, epoch0)
    torch.cuda.synchronize()
    tr.time_gather0, tr.gather0_events = True, []
    t0 = time.perf_counter()
    run(steps, epoch0 + 1000)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    tr.time_gather0 = False
    # per mini-batch: a launch covers one batch or, for the grouped layer-0 gather, a whole sampled group
    gather_ms = sum(a.elapsed_time(b) for a, b in tr.gather0_events) / max(1, steps)
    # input nodes per batch (the rows of X a batch touches), over the first groups of one more epoch
    n_in, _ = tr.input_node_stats(policy, mix, p, epoch0 + 2000)
    return dt * 1e3 / steps, gather_ms, n_in


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="arxiv")
    ap.add_argument("--scales", type=float, nargs="+", default=[0.25, 1.0, 4.0, 16.0])
    ap.add_argument("--widths", type=int, nargs="+", default=[0], help="feature widths (0 = the workload's own)")
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--group", type=int, default=32)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--model", default="sage", choices=["sage", "gcn", "gat"])
    ap.add_argument("--settings", nargs="+", default=DEFAULT_SETTINGS)
    ap.add_argument("--row-order", default="auto", choices=["auto", "on", "off"],
                    help="process the input-side block's rows in community order (the sorted-frontier ablation: off)")
    args = ap.parse_args(argv)

    import numpy as np
    import torch
    from . import synth, synth_gpu
    from .fit import parse_setting
    from .trainer import Trainer
    if not torch.cuda.is_available():
        sys.exit("sensitivity needs a GPU: the path has no CPU fallback")
    for scale in args.scales:
        for width in args.widths:
            cfg = synth.scaled(synth.CONFIGS[args.workload], scale) if scale != 1.0 else copy.deepcopy(synth.CONFIGS[args.workload])
            if width:
                cfg.n_feat = width
            if cfg.n_edges_undirected > 5_000_000:        # large graphs are drawn on the GPU and stay there
                w = synth_gpu.make_workload_gpu(cfg, args.seed)
                n_comm_train = w.n_comm_in_train
                table_bytes = w.features.numel() * w.features.element_size()
            else:
                w = synth.make_workload(cfg, args.seed)
                n_comm_train = int(np.unique(w.comm[w.train_ids]).size)
                table_bytes = w.features.nbytes
            tr = Trainer(w, group_size=args.group, seed=args.seed, model=args.model,
                         order_rows={"auto": "auto", "on": True, "off": False}[args.row_order])
            out = dict(workload=cfg.name, model=args.model, n_nodes=cfg.n_nodes, n_feat=cfg.n_feat, scale=scale,
                       row_order=args.row_order, table_MB=round(table_bytes / 1e6, 1), steps=args.steps, settings={})
            for i, name in enumerate(args.settings):
                policy, mix, p = parse_setting(name, n_comm_train)
                ms, gather_ms, n_in = time_setting(tr, policy, mix, p, args.steps, args.warmup, 10 * i)
                row_bytes = cfg.n_feat * (2 if cfg.feat_dtype == "bf16" else 4)
                out["settings"][name] = dict(ms_per_step=round(ms, 4), gather0_ms=round(gather_ms, 4),
                                             input_nodes=round(n_in), input_MB=round(n_in * row_bytes / 1e6, 2))
            base = out["settings"][args.settings[0]]
            for name in args.settings[1:]:
                s = out["settings"][name]
                s["speedup_step"] = round(base["ms_per_step"] / s["ms_per_step"], 3)
                s["speedup_gather0"] = round(base["gather0_ms"] / s["gather0_ms"], 3)
            print(json.dumps(out), flush=True)
            del tr, w
            torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
