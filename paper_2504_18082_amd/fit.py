"""Train to convergence with the paper's protocol (Section 5, training methodology) on a synthetic workload
and report what its end-to-end comparison reports per knob setting (Section 6.1): number of epochs, time
per epoch, total training time and validation accuracy.

    python -m paper_2504_18082_amd.fit --workload arxiv --settings rand:0.5 mix12.5:0.9 norand:1.0

A setting is <root policy>:<p>, the policy being rand, norand or mix<k> (k percent of the communities per
super-block).  Prints one JSON line per setting."""
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
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--model", default="sage", choices=["sage", "gcn", "gat"])
    args = ap.parse_args(argv)

    import numpy as np
    import torch
    from . import synth
    from .trainer import Trainer
    if not torch.cuda.is_available():
        sys.exit("fit needs a GPU: the path has no CPU fallback")
    cfg = synth.CONFIGS[args.workload]
    if args.scale != 1.0:
        cfg = synth.scaled(cfg, args.scale)
    w = synth.make_workload(cfg, args.seed)
    n_comm_train = int(np.unique(w.comm[w.train_ids]).size)
    val = torch.from_numpy(w.val_ids).cuda()
    for text in args.settings:
        policy, mix, p = parse_setting(text, n_comm_train)
        tr = Trainer(w, group_size=args.group, lr=args.lr, weight_decay=args.weight_decay, seed=args.seed, model=args.model)
        hist = tr.fit(policy, mix, p, val, args.max_epochs, args.patience, args.lr_patience)
        out = dict(workload=cfg.name, model=args.model, setting=text, mix_count=mix, **hist.summary())
        out["val_acc_by_epoch"] = [round(v, 4) for v in hist.val_acc]
        print(json.dumps(out), flush=True)
        del tr
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
