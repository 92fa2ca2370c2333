"""Seeded synthetic inputs shaped like the paper's workloads (Table 2).

This module is the only code shared by the CPU oracle's tests and the GPU
path's tests/benchmark.  It holds input generation only: planted-community
graphs, features, labels, training sets and initial weights.  None of the
method's arithmetic (random stream of the method, shuffles, sampling,
aggregation) lives here; randomness comes from numpy's PCG64.

The real datasets (reddit, igb-small, ogbn-products, ogbn-papers100M) and their
RABBIT community labels are not available offline; degree-corrected planted
partition graphs with the same node counts, edge counts, feature widths, class
counts and training fractions stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np


@dataclass
class WorkloadConfig:
    name: str
    n_nodes: int
    n_edges_undirected: int
    n_comm: int
    comm_size_exponent: float      # size_c ~ rank^-exponent (0 = equal sizes)
    degree_law: str                # "powerlaw" | "lognormal"
    degree_param: float            # exponent gamma, or lognormal sigma
    intra_fraction: float
    n_feat: int
    feat_dtype: str                # "f32" | "bf16"
    n_classes: int
    train_fraction: float
    fanouts: List[int] = field(default_factory=list)   # by GNN layer, 0 = input side
    hidden: int = 256
    batch_size: int = 1024
    feat_comm_offset: float = 0.0
    label_noise: float = 0.1
    val_fraction: float = 0.1      # of all nodes, drawn among the nodes outside the training set


CONFIGS = {
    # tiny planted-community graph
    "tiny": WorkloadConfig("tiny", 10_000, 50_000, 50, 0.0, "lognormal", 0.5, 0.80, 64, "f32", 10,
                           0.50, [10, 5], 64, 256, 0.5, 0.0),
    # sparse citation-like graph
    "arxiv": WorkloadConfig("arxiv", 170_000, 1_200_000, 500, 1.0, "powerlaw", 2.5, 0.75, 128,
                            "f32", 40, 0.55, [15, 10, 5], 256, 1024, 0.3),
    # dense social-like graph (reddit's shape)
    "reddit": WorkloadConfig("reddit", 233_000, 57_000_000, 50, 0.5, "lognormal", 1.0, 0.85, 602,
                             "f32", 41, 0.66, [25, 10], 256, 1024, 0.3),
    # co-purchase-like graph (ogbn-products' shape)
    "products": WorkloadConfig("products", 2_450_000, 62_000_000, 5000, 1.0, "powerlaw", 2.5, 0.80,
                               100, "f32", 47, 0.08, [15, 10, 5], 256, 1024, 0.3),
    # large citation-like graph (ogbn-papers100M's shape); see scaled()
    "papers": WorkloadConfig("papers", 111_000_000, 1_600_000_000, 100_000, 1.0, "powerlaw", 2.5,
                             0.70, 128, "bf16", 172, 0.011, [15, 10, 5], 256, 1024, 0.3),
}
CONFIG_ORDER = ["tiny", "arxiv", "reddit", "products", "papers"]


def scaled(cfg: WorkloadConfig, factor: float, name: str | None = None) -> WorkloadConfig:
    """Same recipe at `factor` times the node / edge / community counts."""
    import copy
    c = copy.deepcopy(cfg)
    c.name = name or f"{cfg.name}_x{factor:g}"
    c.n_nodes = max(64, int(cfg.n_nodes * factor))
    c.n_edges_undirected = max(64, int(cfg.n_edges_undirected * factor))
    c.n_comm = max(2, int(cfg.n_comm * factor))
    return c


@dataclass
class Workload:
    cfg: WorkloadConfig
    indptr: np.ndarray        # int64 [N+1]
    indices: np.ndarray       # int32 [nnz], rows ascending, no self loops, no duplicates
    comm: np.ndarray          # int32 [N], ids contiguous by community
    comm_ptr: np.ndarray      # int64 [n_comm+1]
    features: np.ndarray      # float32 [N, ld]  (ld = n_feat rounded up to 4) or uint16 (bf16)
    labels: np.ndarray        # int32 [N]
    train_ids: np.ndarray     # int32, ascending
    val_ids: np.ndarray = None  # int32, ascending, disjoint from train_ids
    achieved_intra_fraction: float = 0.0

    @property
    def graph(self):
        return (self.indptr, self.indices, self.comm)


def _community_sizes(n_nodes, n_comm, exponent, floor=16):
    if exponent == 0.0:
        base = np.full(n_comm, n_nodes // n_comm, dtype=np.int64)
        base[: n_nodes - base.sum()] += 1
        return base
    w = np.arange(1, n_comm + 1, dtype=np.float64) ** (-exponent)
    floor = min(floor, max(1, n_nodes // (2 * n_comm)))
    sizes = np.maximum(floor, np.floor(w / w.sum() * (n_nodes - floor * n_comm)).astype(np.int64) + floor)
    # fix the total on the largest community
    sizes[0] += n_nodes - sizes.sum()
    assert sizes[0] > 0 and sizes.sum() == n_nodes
    return sizes


def float_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> raw bfloat16 bit patterns (storage only)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


def bf16_bits_to_float(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def make_graph(cfg: WorkloadConfig, seed: int = 0, verbose: bool = False):
    """Degree-corrected planted-partition graph.  Returns (indptr, indices, comm, comm_ptr, intra)."""
    import sys
    say = (lambda msg: print(f"# synth: {msg}", file=sys.stderr, flush=True)) if verbose else (lambda msg: None)
    rng = np.random.default_rng([seed, 0xC0DE, 1])
    N, E = cfg.n_nodes, cfg.n_edges_undirected
    sizes = _community_sizes(N, cfg.n_comm, cfg.comm_size_exponent)
    comm_ptr = np.zeros(cfg.n_comm + 1, dtype=np.int64)
    np.cumsum(sizes, out=comm_ptr[1:])
    comm = np.repeat(np.arange(cfg.n_comm, dtype=np.int32), sizes)

    u = rng.random(N)
    if cfg.degree_law == "powerlaw":
        theta = (1.0 - u) ** (-1.0 / (cfg.degree_param - 1.0))
        theta = np.minimum(theta, np.sqrt(2.0 * E) / max(1.0, 2.0 * E / N))
    else:
        theta = np.exp(cfg.degree_param * rng.standard_normal(N))
    cum = np.cumsum(theta)
    cum_lo = np.concatenate(([0.0], cum))[comm_ptr[:-1]]     # mass before each community
    cum_hi = cum[comm_ptr[1:] - 1]
    total = cum[-1]

    def draw(m):
        """m undirected edges as directed (row * N + column) keys, both directions."""
        a = np.minimum(np.searchsorted(cum, rng.random(m) * total, side="right"), N - 1)
        want_intra = rng.random(m) < cfg.intra_fraction
        ca = comm[a]
        lo, width = cum_lo[ca], cum_hi[ca] - cum_lo[ca]
        r = rng.random(m)
        # second endpoint by propensity: inside a's community, or among all nodes outside it (the community's
        # stretch of the cumulative mass is skipped, so no draw is wasted)
        t_out = r * (total - width)
        target = np.where(want_intra, lo + r * width, np.where(t_out < lo, t_out, t_out + width))
        b = np.minimum(np.searchsorted(cum, target, side="right"), N - 1)
        keep = (a != b) & ((comm[b] == ca) == want_intra)      # self loops; rounding at a community's edge
        a, b = a[keep].astype(np.int64), b[keep].astype(np.int64)
        return [a * N + b, b * N + a]

    # Drawing with replacement loses the repeated pairs when the adjacency is de-duplicated: draw, de-duplicate, and
    # top up what is missing until the graph has (within half a percent) the number of edges asked for.
    key = np.zeros(0, dtype=np.int64)
    want = E
    for _ in range(8):
        keys = [key]
        chunk = 8_000_000
        for start in range(0, want, chunk):
            keys += draw(min(chunk, want - start))
            say(f"edges drawn {min(want, start + chunk)} / {want}")
        before = key.size
        key = np.unique(np.concatenate(keys))
        del keys
        if key.size >= 0.995 * 2 * E:
            break
        yield_ = max(0.2, (key.size - before) / (2.0 * want))
        want = int((2 * E - key.size) / 2 / yield_ * 1.02) + 1
    say(f"{key.size} directed entries after symmetrising and de-duplicating")
    rows = key // N
    indices = (key - rows * N).astype(np.int32)
    indptr = np.zeros(N + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows, minlength=N), out=indptr[1:])
    intra = float((comm[rows] == comm[indices]).mean()) if key.size else 0.0
    return indptr, indices, comm, comm_ptr, intra


def make_workload(cfg: WorkloadConfig | str, seed: int = 0, with_features: bool = True, verbose: bool = False) -> Workload:
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    indptr, indices, comm, comm_ptr, intra = make_graph(cfg, seed, verbose)
    N = cfg.n_nodes
    rng = np.random.default_rng([seed, 0xFEA7, 2])
    ld = (cfg.n_feat + 3) // 4 * 4
    if with_features:
        feats = np.zeros((N, ld), dtype=np.float32)
        step = 1 << 20
        for s in range(0, N, step):
            feats[s:s + step, :cfg.n_feat] = rng.standard_normal((min(step, N - s), cfg.n_feat), dtype=np.float32)
        if cfg.feat_comm_offset:
            off = (cfg.feat_comm_offset * rng.standard_normal((cfg.n_comm, cfg.n_feat))).astype(np.float32)
            feats[:, :cfg.n_feat] += off[comm]
        if cfg.feat_dtype == "bf16":
            feats = float_to_bf16_bits(feats)
    else:
        feats = np.zeros((0, ld), dtype=np.float32)
    rng = np.random.default_rng([seed, 0x1ABE, 3])
    if cfg.label_noise == 0.0:
        labels = (comm % cfg.n_classes).astype(np.int32)
    else:
        cls_of_comm = rng.integers(0, cfg.n_classes, size=cfg.n_comm, dtype=np.int32)
        labels = cls_of_comm[comm]
        noisy = rng.random(N) < cfg.label_noise
        labels = np.where(noisy, rng.integers(0, cfg.n_classes, size=N, dtype=np.int32), labels).astype(np.int32)
    rng = np.random.default_rng([seed, 0x7EA1, 4])
    is_train = rng.random(N) < cfg.train_fraction
    train_ids = np.nonzero(is_train)[0].astype(np.int32)
    rng = np.random.default_rng([seed, 0x7A1D, 6])
    p_val = min(1.0, cfg.val_fraction / max(1e-9, 1.0 - cfg.train_fraction))
    val_ids = np.nonzero(~is_train & (rng.random(N) < p_val))[0].astype(np.int32)
    return Workload(cfg, indptr, indices, comm, comm_ptr, feats, labels, train_ids, val_ids, intra)


def layer_dims(cfg: WorkloadConfig):
    """(F_in, F_out) of every GNN layer."""
    L = len(cfg.fanouts)
    dims = []
    for l in range(L):
        fin = cfg.n_feat if l == 0 else cfg.hidden
        fout = cfg.n_classes if l == L - 1 else cfg.hidden
        dims.append((fin, fout))
    return dims


def init_weights(cfg: WorkloadConfig, seed: int = 0, n_operands: int = 2):
    """Glorot-uniform [n_operands*F_in, F_out] (two operands: rows of W_self then W_neigh) and zero biases, float32."""
    rng = np.random.default_rng([seed, 0x3E16, 5])
    out = []
    for fin, fout in layer_dims(cfg):
        a = np.sqrt(6.0 / (fin + fout))
        W = rng.uniform(-a, a, size=(n_operands * fin, fout)).astype(np.float32)
        b = np.zeros(fout, dtype=np.float32)
        out.append((W, b))
    return out


def init_gat_weights(cfg: WorkloadConfig, seed: int = 0, heads: int = 4):
    """Per layer (W [F_in, heads*D], a_l [heads*D], a_r [heads*D], bias [heads*D]) in float32: `heads` heads of width
    hidden/heads on hidden layers (concatenated), one head of width n_classes on the last.  Glorot-uniform W and
    attention vectors, zero bias."""
    rng = np.random.default_rng([seed, 0x6A7, 5])
    out = []
    dims = layer_dims(cfg)
    for l, (fin, fout) in enumerate(dims):
        h = heads if l < len(dims) - 1 else 1
        assert fout % h == 0
        D = fout // h
        a = np.sqrt(6.0 / (fin + fout))
        W = rng.uniform(-a, a, size=(fin, fout)).astype(np.float32)
        c = np.sqrt(6.0 / (D + 1))
        a_l = rng.uniform(-c, c, size=fout).astype(np.float32)
        a_r = rng.uniform(-c, c, size=fout).astype(np.float32)
        out.append((W, a_l, a_r, np.zeros(fout, dtype=np.float32)))
    return out


def star_graph(n_leaves_intra: int, n_leaves_inter: int):
    """Node 0 joined to n_leaves_intra leaves of its own community and
    n_leaves_inter leaves of another one (tiny closed-form test graph)."""
    n = 1 + n_leaves_intra + n_leaves_inter
    rows = [list(range(1, n))] + [[0] for _ in range(n - 1)]
    indptr = np.zeros(n + 1, dtype=np.int64)
    indptr[1:] = np.cumsum([len(r) for r in rows])
    indices = np.array([x for r in rows for x in r], dtype=np.int32)
    comm = np.array([0] + [0] * n_leaves_intra + [1] * n_leaves_inter, dtype=np.int32)
    return indptr, indices, comm
