"""Software-managed feature cache study (Section 6.5, impact of software-managed caches): the feature table stays
in pinned host memory, as in the paper's set-up for its largest graph; every batch brings the rows of its distinct
input nodes over the host link, either all of them (no cache) or only the ones that miss in a set-associative LRU
cache of `--cache-rows` rows in GPU memory.  Reports, per knob setting: the cache's miss rate, ms per step and the
per-step speed-up over the fully random setting in the same mode.

    python -m paper_2504_18082_amd.cache_study --workload papers --scale 0.05 --cache-rows 2000000

Prints one JSON line per mode."""
from __future__ import annotations

import argparse
import json
import sys
import time

DEFAULT_SETTINGS = ["rand:0.5", "mix50:1.0", "mix25:1.0", "mix12.5:1.0", "mix0:1.0"]


def run(tr, policy, mix, p, steps, warmup, epoch0):
    import torch

    def go(n_steps, epoch):
        done = 0
        while done < n_steps:
            done += tr.run_epoch_serial(policy, mix, p, epoch, max_batches=n_steps - done)
            epoch += 1

    go(warmup, epoch0)
    torch.cuda.synchronize()
    before = tr.cache.stats() if tr.cache is not None else None
    t0 = time.perf_counter()
    go(steps, epoch0 + 100)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    out = dict(ms_per_step=round(ms, 4))
    if before is not None:
        q, m, u, status = tr.cache.stats()
        out.update(miss_rate=round((m - before[1]) / max(1, q - before[0]), 4), lookups_per_step=round((q - before[0]) / steps),
                   uncached_misses=u - before[2])
    return out


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="papers")
    ap.add_argument("--scale", type=float, default=0.05)
    ap.add_argument("--cache-rows", type=int, default=2_000_000)
    ap.add_argument("--ways", type=int, default=16)
    ap.add_argument("--settings", nargs="+", default=DEFAULT_SETTINGS)
    ap.add_argument("--modes", nargs="+", default=["host", "host+cache"], choices=["hbm", "host", "host+cache"])
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=60, help="untimed steps that also warm the cache")
    ap.add_argument("--group", type=int, default=32)
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args(argv)

    import numpy as np
    import torch
    from . import synth
    from .fit import parse_setting
    from .trainer import Trainer
    if not torch.cuda.is_available():
        sys.exit("cache_study needs a GPU: the path has no CPU fallback")
    cfg = synth.CONFIGS[args.workload]
    if args.scale != 1.0:
        cfg = synth.scaled(cfg, args.scale)
    w = synth.make_workload(cfg, args.seed, verbose=True)
    n_comm_train = int(np.unique(w.comm[w.train_ids]).size)
    print(f"# {cfg.name}: {cfg.n_nodes} nodes, table {w.features.nbytes / 1e6:.0f} MB, {len(w.train_ids)} training nodes", file=sys.stderr, flush=True)
    for mode in args.modes:
        out = dict(workload=cfg.name, mode=mode, n_nodes=cfg.n_nodes, table_MB=round(w.features.nbytes / 1e6, 1),
                   cache_rows=args.cache_rows if mode == "host+cache" else 0, ways=args.ways, steps=args.steps, settings={})
        for i, name in enumerate(args.settings):
            policy, mix, p = parse_setting(name, n_comm_train)
            tr = Trainer(w, group_size=args.group, seed=args.seed, host_features=mode != "hbm",
                         cache_rows=args.cache_rows if mode == "host+cache" else 0, cache_ways=args.ways,
                         relabel_input=True)
            out["settings"][name] = run(tr, policy, mix, p, args.steps, args.warmup, 10 * i)
            print(f"# {mode} {name}: {out['settings'][name]}", file=sys.stderr, flush=True)
            if tr.host_store is not None:
                torch.cuda.synchronize()
                tr.host_store.free()
            del tr
            torch.cuda.empty_cache()
        base = out["settings"][args.settings[0]]["ms_per_step"]
        for name in args.settings[1:]:
            out["settings"][name]["speedup_step"] = round(base / out["settings"][name]["ms_per_step"], 3)
        print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
