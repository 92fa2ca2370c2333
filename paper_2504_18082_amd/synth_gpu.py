"""Seeded synthetic inputs generated on the GPU, for the workloads too large to build on the host in
reasonable time (the reddit-, products- and papers100M-shaped graphs of Table 2).

Same recipe as synth.py -- degree-corrected planted partition, node ids contiguous by community,
features, labels, training / validation sets -- written with torch device operations only: edge-list
draw, sort, de-duplicate, CSR.  Set-up code that runs before any timed region.  Like synth.py this
module holds input generation only; none of the method's arithmetic lives here, and neither the HIP
library nor the oracle is used.  The random numbers are torch's (Philox generator of the device, seeded),
so a graph is a pure function of (config, seed) on a given torch build; they are not the numbers numpy
draws in synth.py, so the two modules give different graphs of the same shape.

The adjacency of the largest shape has more than 2^31 entries, so the sort runs over row ranges
("buckets") of roughly equal mass rather than over one array.
"""
from __future__ import annotations

import sys
import time
from dataclasses import dataclass
from typing import Optional

import numpy as np

from . import synth

# How many undirected edges are drawn per edge asked for: drawing with replacement loses the repeated pairs
# when the adjacency is de-duplicated.  Measured once per shape (the loss is a property of the recipe); a
# top-up round below closes whatever gap is left, so these only save that round.
DRAW_FACTOR = {"reddit": 1.21, "products": 1.145, "papers": 1.02}


@dataclass
class DeviceWorkload:
    """A workload whose arrays live in device memory (torch tensors); host() gives the numpy form."""
    cfg: synth.WorkloadConfig
    indptr: "torch.Tensor"        # int64 [N+1]
    indices: "torch.Tensor"       # int32 [nnz], rows ascending, no self loops, no duplicates
    comm: "torch.Tensor"          # int32 [N]
    comm_ptr: np.ndarray          # int64 [n_comm+1] (host)
    features: "torch.Tensor"      # float32 [N, ld], or int16 [N, ld] holding raw bf16
    labels: "torch.Tensor"        # int32 [N]
    train_ids: "torch.Tensor"     # int32, ascending
    val_ids: "torch.Tensor"       # int32, ascending, disjoint from train_ids
    achieved_intra_fraction: float = 0.0
    n_comm_in_train: int = 0
    _host: Optional[synth.Workload] = None

    @property
    def n_entries(self) -> int:
        return int(self.indices.numel())

    def host(self, with_features: bool = True) -> synth.Workload:
        """The same arrays as numpy (copied once, then kept)."""
        if self._host is None or (with_features and self._host.features.shape[0] == 0):
            ld = int(self.features.shape[1])
            if with_features:
                f = self.features.cpu().numpy()
                feats = f.view(np.uint16) if f.dtype == np.int16 else f
            else:
                feats = np.zeros((0, ld), dtype=np.float32)
            self._host = synth.Workload(self.cfg, self.indptr.cpu().numpy(), self.indices.cpu().numpy(), self.comm.cpu().numpy(),
                                        self.comm_ptr, feats, self.labels.cpu().numpy(), self.train_ids.cpu().numpy(),
                                        self.val_ids.cpu().numpy(), self.achieved_intra_fraction)
        return self._host


def make_workload_gpu(cfg, seed: int = 0, device: str = "cuda", verbose: bool = False, with_features: bool = True,
                      n_buckets: Optional[int] = None) -> DeviceWorkload:
    """n_buckets: number of row ranges the sort is split into (default: about 150 M entries per range)."""
    import torch
    if isinstance(cfg, str):
        cfg = synth.CONFIGS[cfg]
    t_start = time.perf_counter()
    say = (lambda msg: print(f"# synth_gpu [{time.perf_counter() - t_start:6.1f} s]: {msg}", file=sys.stderr, flush=True)) if verbose else (lambda msg: None)
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed((int(seed) << 20) ^ 0xC0DE1)
    N, E = cfg.n_nodes, cfg.n_edges_undirected
    shift = max(1, (N - 1).bit_length())
    assert 2 * shift <= 62, "node ids too wide for a 64-bit (row, column) key"

    # communities (sizes on the host: n_comm numbers), ids contiguous by community
    sizes = synth._community_sizes(N, cfg.n_comm, cfg.comm_size_exponent)
    comm_ptr = np.zeros(cfg.n_comm + 1, dtype=np.int64)
    np.cumsum(sizes, out=comm_ptr[1:])
    comm = torch.repeat_interleave(torch.arange(cfg.n_comm, dtype=torch.int32, device=dev), torch.from_numpy(sizes).to(dev))
    comm_ptr_d = torch.from_numpy(comm_ptr).to(dev)

    # degree propensities and their cumulative mass
    u = torch.rand(N, dtype=torch.float64, device=dev, generator=gen)
    if cfg.degree_law == "powerlaw":
        theta = (1.0 - u).pow_(-1.0 / (cfg.degree_param - 1.0))
        theta.clamp_(max=float(np.sqrt(2.0 * E) / max(1.0, 2.0 * E / N)))
    else:
        theta = torch.exp(cfg.degree_param * torch.randn(N, dtype=torch.float64, device=dev, generator=gen))
    del u
    cum = torch.cumsum(theta, 0)
    del theta
    total = float(cum[-1])
    cum_hi = cum[comm_ptr_d[1:] - 1]
    cum_lo = torch.cat([torch.zeros(1, dtype=torch.float64, device=dev), cum_hi[:-1]])

    # row ranges of roughly equal mass; every range's entries are sorted on their own
    if n_buckets is None:
        n_buckets = int(min(64, max(1, -(-(2 * E) // 150_000_000))))
    qs = torch.arange(1, n_buckets, dtype=torch.float64, device=dev) * (total / n_buckets)
    bounds = torch.searchsorted(cum, qs).to(torch.int64)                 # first row of buckets 1..n_buckets-1
    bound_keys = bounds << shift
    row_first = [0] + [int(x) for x in bounds.cpu().tolist()] + [N]
    pending = [[] for _ in range(n_buckets)]

    def draw(n_edges: int):
        """Draws n_edges undirected edges and files both directions, as (row << shift | column) keys, by row range."""
        chunk = 32_000_000
        for start in range(0, n_edges, chunk):
            m = min(chunk, n_edges - start)
            a = torch.searchsorted(cum, torch.rand(m, dtype=torch.float64, device=dev, generator=gen) * total, right=True).clamp_(max=N - 1)
            want_intra = torch.rand(m, device=dev, generator=gen) < cfg.intra_fraction
            ca = comm[a].to(torch.int64)
            lo, hi = cum_lo[ca], cum_hi[ca]
            r = torch.rand(m, dtype=torch.float64, device=dev, generator=gen)
            # second endpoint by propensity: inside a's community, or among all nodes outside it (the community's
            # stretch of the cumulative mass is skipped, so no draw is wasted)
            t_out = r * (total - (hi - lo))
            target = torch.where(want_intra, lo + r * (hi - lo), torch.where(t_out < lo, t_out, t_out + (hi - lo)))
            del r, t_out, lo, hi
            b = torch.searchsorted(cum, target, right=True).clamp_(max=N - 1)
            del target
            keep = (a != b) & ((comm[b].to(torch.int64) == ca) == want_intra)     # self loops; rounding at a community's edge
            a, b = a[keep], b[keep]
            del keep, ca, want_intra
            keys = torch.cat([(a << shift) | b, (b << shift) | a])
            del a, b
            if n_buckets == 1:
                pending[0].append(keys)
            else:               # sorted, a row range is one contiguous slice of the chunk
                keys = torch.sort(keys).values
                cuts = [0] + torch.searchsorted(keys, bound_keys).cpu().tolist() + [int(keys.numel())]
                for k in range(n_buckets):
                    if cuts[k + 1] > cuts[k]:
                        pending[k].append(keys[cuts[k]:cuts[k + 1]])
            del keys
        say(f"{n_edges} edges drawn")

    uniq = [None] * n_buckets

    def settle():
        """Sorts and de-duplicates what is pending, bucket by bucket; returns the number of distinct entries."""
        count = 0
        for k in range(n_buckets):
            if pending[k]:
                parts = ([uniq[k]] if uniq[k] is not None else []) + pending[k]
                pending[k] = []
                keys = torch.cat(parts)
                del parts
                keys = torch.sort(keys).values
                uniq[k] = torch.unique_consecutive(keys)
                del keys
            count += 0 if uniq[k] is None else int(uniq[k].numel())
        return count

    draw(int(E * DRAW_FACTOR.get(cfg.name.split("_x")[0], 1.0)))
    n_entries = settle()
    say(f"{n_entries} distinct directed entries ({n_entries / (2 * E):.4f} of the target)")
    for _ in range(3):                      # top up what the repeated pairs took away
        if n_entries >= 0.995 * 2 * E:
            break
        drawn_yield = max(0.2, n_entries / (2.0 * E * DRAW_FACTOR.get(cfg.name.split("_x")[0], 1.0)))
        draw(int((2 * E - n_entries) / 2 / drawn_yield * 1.02) + 1)
        n_entries = settle()
        say(f"{n_entries} distinct directed entries after a top-up ({n_entries / (2 * E):.4f} of the target)")

    # CSR
    deg = torch.zeros(N, dtype=torch.int64, device=dev)
    indices = torch.empty(n_entries, dtype=torch.int32, device=dev)
    mask = (1 << shift) - 1
    at = 0
    n_intra = 0
    for k in range(n_buckets):
        keys = uniq[k]
        uniq[k] = None
        if keys is None or keys.numel() == 0:
            continue
        rows = keys >> shift
        cols = keys & mask
        del keys
        r0, r1 = row_first[k], row_first[k + 1]
        deg[r0:r1] = torch.bincount(rows - r0, minlength=r1 - r0)[: r1 - r0]
        n_intra += int((comm[rows] == comm[cols]).sum())
        indices[at:at + cols.numel()] = cols.to(torch.int32)
        at += int(cols.numel())
        del rows, cols
    assert at == n_entries
    indptr = torch.zeros(N + 1, dtype=torch.int64, device=dev)
    torch.cumsum(deg, 0, out=indptr[1:])
    del deg, cum, cum_lo, cum_hi
    intra = n_intra / max(1, n_entries)
    say(f"CSR built: {n_entries} entries, {intra:.4f} intra-community")

    # features: N(0,1) plus a per-community offset, float32 (row stride padded to 4) or bf16 (round to nearest even)
    gen.manual_seed((int(seed) << 20) ^ 0xFEA72)
    ld = (cfg.n_feat + 3) // 4 * 4
    bf16 = cfg.feat_dtype == "bf16"
    if with_features:
        feats = torch.zeros((N, ld), dtype=torch.int16 if bf16 else torch.float32, device=dev)
        off = None
        if cfg.feat_comm_offset:
            off = cfg.feat_comm_offset * torch.randn((cfg.n_comm, cfg.n_feat), device=dev, generator=gen)
        step = 1 << 21
        for s in range(0, N, step):
            n = min(step, N - s)
            x = torch.randn((n, cfg.n_feat), device=dev, generator=gen)
            if off is not None:
                x += off[comm[s:s + n].to(torch.int64)]
            if bf16:
                feats[s:s + n, :cfg.n_feat] = x.to(torch.bfloat16).view(torch.int16)
            else:
                feats[s:s + n, :cfg.n_feat] = x
            del x
        del off
    else:
        feats = torch.zeros((0, ld), dtype=torch.int16 if bf16 else torch.float32, device=dev)
    say("features built")

    # labels: the class of the community, with label noise
    gen.manual_seed((int(seed) << 20) ^ 0x1ABE3)
    if cfg.label_noise == 0.0:
        labels = (comm % cfg.n_classes).to(torch.int32)
    else:
        cls_of_comm = torch.randint(0, cfg.n_classes, (cfg.n_comm,), device=dev, generator=gen, dtype=torch.int32)
        labels = cls_of_comm[comm.to(torch.int64)]
        noisy = torch.rand(N, device=dev, generator=gen) < cfg.label_noise
        labels = torch.where(noisy, torch.randint(0, cfg.n_classes, (N,), device=dev, generator=gen, dtype=torch.int32), labels)
    # training set, and a validation set among the other nodes
    gen.manual_seed((int(seed) << 20) ^ 0x7EA14)
    is_train = torch.rand(N, device=dev, generator=gen) < cfg.train_fraction
    train_ids = torch.nonzero(is_train).flatten().to(torch.int32)
    p_val = min(1.0, cfg.val_fraction / max(1e-9, 1.0 - cfg.train_fraction))
    val_ids = torch.nonzero(~is_train & (torch.rand(N, device=dev, generator=gen) < p_val)).flatten().to(torch.int32)
    n_comm_in_train = int(torch.unique(comm[train_ids.to(torch.int64)]).numel())
    say(f"done: {int(train_ids.numel())} training nodes in {n_comm_in_train} communities")
    return DeviceWorkload(cfg, indptr, indices, comm, comm_ptr, feats, labels, train_ids, val_ids, intra, n_comm_in_train)
