"""Train to convergence with the paper's protocol (Section 5, training methodology) on a synthetic workload
and report what its end-to-end comparison reports per knob setting (Section 6.1): number of epochs, time
per epoch, total training time and validation accuracy.

    python -m paper_2504_18082_amd.fit --workload arxiv --settings rand:0.5 mix12.5:0.9 norand:1.0

A setting is <root policy>:<p>, the policy being rand, norand or mix<k> (k percent of the communities per
super-block).  Prints one JSON line per setting and training seed; with --seeds N (the paper trains every setting
with five seeds) also one line per setting with the mean and standard deviation over the seeds.  The graph, its features
and labels stay the same for all training seeds (--graph-seed)."""
from __future__ import annotations

import argparse
import json
import sys


def parse_setting(text: str, n_comm_train: int):
    from . import binding as B, synth
    pol, p = text.split(":")
    p = float(p)
    if pol == "rand":
        return B.CR_ROOTS_RAND, 1, p
    if pol == "norand":
        return B.CR_ROOTS_NORAND, 1, p
    if pol.startswith("mix"):
        return B.CR_ROOTS_COMM_RAND, B.cr_mix_count_from_percent(float(pol[3:]), n_comm_train), p
    raise ValueError(f"unknown root policy '{pol}'")


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="arxiv")
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--settings", nargs="+", default=["rand:0.5", "mix12.5:0.9", "norand:1.0"])
    ap.add_argument("--max-epochs", type=int, default=100)
    ap.add_argument("--patience", type=int, default=6)
    ap.add_argument("--lr-patience", type=int, default=3)
    ap.add_argument("--lr", type=float, default=0.1)
    ap.add_argument("--weight-decay", type=float, default=5e-4)
    ap.add_argument("--group", type=int, default=32)
    ap.add_argument("--seed", type=int, default=0, help="first training seed (weights, root order, neighbour sampling)")
    ap.add_argument("--seeds", type=int, default=1, help="number of training seeds: seed, seed+1, ...")
    ap.add_argument("--graph-seed", type=int, default=0)
    ap.add_argument("--model", default="sage", choices=["sage", "gcn", "gat"])
    args = ap.parse_args(argv)

    import numpy as np
    import torch
    from . import synth, synth_gpu
    from .trainer import Trainer
    if not torch.cuda.is_available():
        sys.exit("fit needs a GPU: the path has no CPU fallback")
    cfg = synth.CONFIGS[args.workload]
    if args.scale != 1.0:
        cfg = synth.scaled(cfg, args.scale)
    if cfg.n_edges_undirected > 5_000_000:          # large graphs are drawn on the GPU and stay there
        w = synth_gpu.make_workload_gpu(cfg, args.graph_seed)
        n_comm_train, val = w.n_comm_in_train, w.val_ids
    else:
        w = synth.make_workload(cfg, args.graph_seed)
        n_comm_train = int(np.unique(w.comm[w.train_ids]).size)
        val = torch.from_numpy(w.val_ids).cuda()
    for text in args.settings:
        policy, mix, p = parse_setting(text, n_comm_train)
        runs = []
        for seed in range(args.seed, args.seed + args.seeds):
            tr = Trainer(w, group_size=args.group, lr=args.lr, weight_decay=args.weight_decay, seed=seed, model=args.model)
            hist = tr.fit(policy, mix, p, val, args.max_epochs, args.patience, args.lr_patience)
            out = dict(workload=cfg.name, model=args.model, setting=text, mix_count=mix, seed=seed, **hist.summary())
            out["val_acc_by_epoch"] = [round(v, 4) for v in hist.val_acc]
            print(json.dumps(out), flush=True)
            runs.append(out)
            del tr
            torch.cuda.empty_cache()
        if args.seeds > 1:
            agg = dict(workload=cfg.name, model=args.model, setting=text, mix_count=mix, seeds=args.seeds)
            for key in ("epochs", "best_val_acc", "final_val_acc", "mean_epoch_ms", "total_train_ms"):
                vals = np.array([r[key] for r in runs], dtype=np.float64)
                agg[key + "_mean"], agg[key + "_std"] = round(float(vals.mean()), 4), round(float(vals.std(ddof=1)), 4)
            print(json.dumps(agg), flush=True)


if __name__ == "__main__":
    main()
