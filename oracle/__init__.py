"""ctypes access to the CPU oracle (oracle/oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  Nothing in the product package imports this.
The functions of the GraphSAGE path only marshal numpy arrays, their arithmetic is in oracle.c; the GCN and GAT
layers at the end of this file are written out in numpy, in float64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_LIB_OMP = os.path.join(_HERE, "liboracle_omp.so")
_lib = None
_libs = {}


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc (no fused multiply-add contraction): the single-threaded library that everything
    uses, and the same source with OpenMP enabled for the benchmark's all-cores CPU baseline."""
    for out, extra in ((_LIB, ["-Wno-unknown-pragmas"]), (_LIB_OMP, ["-fopenmp"])):
        if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
            subprocess.check_call(
                ["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fPIC", "-shared", "-Wall"] + extra +
                ["-o", out, _SRC, "-lm"])
    return _LIB


def use_all_cores(on: bool) -> int:
    """Switches every later call between the single-threaded library (the oracle proper; the default) and the OpenMP
    build of the same source (row loops spread over the host's cores).  Returns the number of threads in use."""
    global _lib
    _lib = None
    lib(_LIB_OMP if on else _LIB)
    if on:
        omp = C.CDLL("libgomp.so.1")
        omp.omp_get_max_threads.restype = C.c_int
        return int(omp.omp_get_max_threads())
    return 1


def lib(path: str = None):
    global _lib
    if _lib is None or path is not None:
        build()
        path = path or _LIB
        if path in _libs:
            _lib = _libs[path]
            return _lib
        L = C.CDLL(path)
        L.orc_shuffle_key.restype = C.c_uint64
        L.orc_shuffle_key.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32]
        L.orc_slot_word.restype = C.c_uint32
        L.orc_slot_word.argtypes = [C.c_uint64] + [C.c_uint32] * 5
        L.orc_exp_clock_q24.restype = C.c_uint32
        L.orc_exp_clock_q24.argtypes = [C.c_uint32]
        L.orc_slot_key.restype = C.c_uint64
        L.orc_slot_key.argtypes = [C.c_uint32, C.c_int, C.c_uint32]
        L.orc_build_batches.restype = C.c_int
        L.orc_build_batches.argtypes = [C.c_int, C.c_int32, C.c_uint64, C.c_uint32, C.c_void_p,
                                        C.c_int64, C.c_void_p, C.c_int32, C.c_void_p]
        L.orc_sample_hop.restype = C.c_int64
        L.orc_sample_hop.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                     C.c_int32, C.c_uint32, C.c_int, C.c_uint64, C.c_uint32,
                                     C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_transpose_block.restype = None
        L.orc_transpose_block.argtypes = [C.c_int32, C.c_int32] + [C.c_void_p] * 4
        L.orc_round_bf16.restype = None
        L.orc_round_bf16.argtypes = [C.c_void_p, C.c_int64, C.c_void_p]
        L.orc_gather_mean.restype = None
        L.orc_gather_mean.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_int, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p]
        L.orc_gather_mean_bwd.restype = None
        L.orc_gather_mean_bwd.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        L.orc_sage_linear_fwd.restype = None
        L.orc_sage_linear_fwd.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        L.orc_sage_linear_bwd.restype = None
        L.orc_sage_linear_bwd.argtypes = [C.c_int32, C.c_int32, C.c_int32] + [C.c_void_p] * 5 + \
                                         [C.c_int, C.c_int] + [C.c_void_p] * 4
        L.orc_sgd_step.restype = None
        L.orc_sgd_step.argtypes = [C.c_int64, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                   C.c_void_p, C.c_double, C.c_double]
        L.orc_softmax_xent.restype = C.c_double
        L.orc_softmax_xent.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p,
                                       C.c_void_p]
        L.orc_count_correct.restype = C.c_int32
        L.orc_cache_fetch.restype = C.c_int32
        L.orc_cache_fetch.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        L.orc_count_correct.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p]
        _libs[path] = L
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


# ---------------------------------------------------------------- random stream
def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (C.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    o = (C.c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def shuffle_key(seed, epoch, domain, ident):
    return int(lib().orc_shuffle_key(seed, epoch, domain, ident))


def slot_word(seed, epoch, batch, layer, node, slot):
    return int(lib().orc_slot_word(seed, epoch, batch, layer, node, slot))


def exp_clock_q24(r):
    return int(lib().orc_exp_clock_q24(int(r)))


def slot_key(r, intra, q_in):
    return int(lib().orc_slot_key(int(r), int(bool(intra)), int(q_in)))


def q_intra(p: float) -> int:
    """Fixed-point intra-community weight handed to both implementations."""
    return int(round(p * 65536.0))


# ---------------------------------------------------------------- step 1
NORAND, COMM_RAND, RAND = 0, 1, 2


def build_batches(policy, mix, seed, epoch, train_ids, comm, n_comm):
    train_ids = _arr(train_ids, np.int32)
    comm = _arr(comm, np.int32)
    perm = np.empty(train_ids.shape[0], dtype=np.int32)
    rc = lib().orc_build_batches(policy, mix, seed, epoch, _p(train_ids), train_ids.shape[0],
                                 _p(comm), n_comm, _p(perm))
    if rc != 0:
        raise ValueError("orc_build_batches rejected its arguments")
    return perm


# ---------------------------------------------------------------- step 2
class Block:
    """One sampled bipartite block (numpy, host)."""

    def __init__(self, n_dst, src_ids, indptr, indices, slots):
        self.n_dst = int(n_dst)
        self.src_ids = src_ids
        self.n_src = int(src_ids.shape[0])
        self.indptr = indptr
        self.indices = indices
        self.nnz = int(indices.shape[0])
        self.slots = slots
        self.t_indptr = None
        self.t_indices = None


def sample_hop(graph, dst_ids, fanout, p, strict, seed, epoch, batch, layer, pos_map=None):
    indptr, indices, comm = graph
    dst_ids = _arr(dst_ids, np.int32)
    n_dst = dst_ids.shape[0]
    if pos_map is None:
        pos_map = np.full(indptr.shape[0] - 1, -1, dtype=np.int32)
    o_indptr = np.empty(n_dst + 1, dtype=np.int32)
    o_indices = np.empty(max(1, n_dst * fanout), dtype=np.int32)
    o_slots = np.empty(max(1, n_dst * fanout), dtype=np.int32)
    o_src = np.empty(max(1, n_dst * (1 + fanout)), dtype=np.int32)
    n_src = C.c_int32(0)
    nnz = lib().orc_sample_hop(_p(indptr), _p(indices), _p(comm), _p(dst_ids), n_dst, fanout,
                               q_intra(p), int(strict), seed, epoch, batch, layer, _p(pos_map),
                               _p(o_indptr), _p(o_indices), _p(o_src), C.byref(n_src), _p(o_slots))
    if nnz < 0:
        raise ValueError("orc_sample_hop rejected its arguments")
    return Block(n_dst, o_src[:n_src.value].copy(), o_indptr, o_indices[:nnz].copy(),
                 o_slots[:nnz].copy())


def transpose_block(blk: Block):
    t_indptr = np.empty(blk.n_src + 1, dtype=np.int32)
    t_indices = np.empty(max(1, blk.nnz), dtype=np.int32)
    lib().orc_transpose_block(blk.n_dst, blk.n_src, _p(blk.indptr), _p(blk.indices),
                              _p(t_indptr), _p(t_indices))
    blk.t_indptr, blk.t_indices = t_indptr, t_indices[:blk.nnz]
    return blk


def sample_blocks(graph, roots, fanouts, p, strict, seed, epoch, batch, pos_map=None,
                  transpose=True):
    """Blocks indexed by GNN layer (0 = input side).  Roots are expanded first,
    with fanouts[L-1]; the frontier of layer l is the destination list of l-1."""
    L = len(fanouts)
    blocks = [None] * L
    dst = _arr(roots, np.int32)
    if pos_map is None:
        pos_map = np.full(graph[0].shape[0] - 1, -1, dtype=np.int32)
    for l in range(L - 1, -1, -1):
        blk = sample_hop(graph, dst, fanouts[l], p, strict, seed, epoch, batch, l, pos_map)
        if transpose and l >= 1:
            transpose_block(blk)
        blocks[l] = blk
        dst = blk.src_ids
    return blocks


# ---------------------------------------------------------------- dense math
def round_bf16(x):
    x = _arr(x, np.float64)
    out = np.empty_like(x)
    lib().orc_round_bf16(_p(x), x.size, _p(out))
    return out


def gather_mean(blk: Block, table, indirect: bool, F=None, want_self=False):
    """table: float32 [rows, ld], uint16 (raw bf16) [rows, ld] or float64 [rows, ld]."""
    assert table.dtype in (np.float32, np.uint16, np.float64) and table.flags.c_contiguous
    F = table.shape[1] if F is None else F
    agg = np.empty((blk.n_dst, F), dtype=np.float64)
    self_rows = np.empty((blk.n_dst, F), dtype=np.float64) if want_self else None
    lib().orc_gather_mean(blk.n_dst, _p(blk.indptr), _p(blk.indices),
                          _p(blk.src_ids) if indirect else None, _p(table),
                          {np.dtype(np.float32): 0, np.dtype(np.uint16): 1, np.dtype(np.float64): 2}[table.dtype], table.shape[1], F,
                          _p(agg), _p(self_rows))
    return (agg, self_rows) if want_self else agg


def gather_mean_bwd(blk: Block, d_agg, d_self=None):
    d_agg = _arr(d_agg, np.float64)
    F = d_agg.shape[1]
    if d_self is not None:
        d_self = _arr(d_self, np.float64)
    d_src = np.empty((blk.n_src, F), dtype=np.float64)
    lib().orc_gather_mean_bwd(blk.n_dst, blk.n_src, _p(blk.indptr), _p(blk.indices), _p(d_agg),
                              _p(d_self), F, _p(d_src))
    return d_src


def sage_linear_fwd(h_self, agg, W, bias, relu, round_operands):
    h_self, agg, W, bias = (_arr(a, np.float64) for a in (h_self, agg, W, bias))
    M, F_in = h_self.shape
    F_out = W.shape[1]
    assert W.shape[0] == 2 * F_in and agg.shape == h_self.shape
    out = np.empty((M, F_out), dtype=np.float64)
    lib().orc_sage_linear_fwd(M, F_in, F_out, _p(h_self), _p(agg), _p(W), _p(bias), int(relu),
                              int(round_operands), _p(out))
    return out


def sage_linear_bwd(h_self, agg, W, out, d_out, relu, round_operands, need_dx=True):
    h_self, agg, W, out, d_out = (_arr(a, np.float64) for a in (h_self, agg, W, out, d_out))
    M, F_in = h_self.shape
    F_out = W.shape[1]
    dW = np.empty((2 * F_in, F_out), dtype=np.float64)
    db = np.empty(F_out, dtype=np.float64)
    d_self = np.empty((M, F_in), dtype=np.float64) if need_dx else None
    d_agg = np.empty((M, F_in), dtype=np.float64) if need_dx else None
    lib().orc_sage_linear_bwd(M, F_in, F_out, _p(h_self), _p(agg), _p(W), _p(out), _p(d_out),
                              int(relu), int(round_operands), _p(dW), _p(db), _p(d_self),
                              _p(d_agg))
    return dW, db, d_self, d_agg


def sgd_step(W, dW, b, db, lr, wd):
    W = _arr(W, np.float64).copy()
    b = _arr(b, np.float64).copy()
    dW = _arr(dW, np.float64)
    db = _arr(db, np.float64)
    lib().orc_sgd_step(W.size, _p(W), _p(dW), b.size, _p(b), _p(db), lr, wd)
    return W, b


def softmax_xent(logits, labels, n_classes=None):
    logits = _arr(logits, np.float64)
    labels = _arr(labels, np.int32)
    n, ld = logits.shape
    Cn = ld if n_classes is None else n_classes
    d = np.zeros_like(logits)
    loss = lib().orc_softmax_xent(n, Cn, _p(logits), ld, _p(labels), _p(d))
    return float(loss), d


def count_correct(logits, labels, n_classes=None):
    logits = _arr(logits, np.float64)
    labels = _arr(labels, np.int32)
    n, ld = logits.shape
    return int(lib().orc_count_correct(n, ld if n_classes is None else n_classes, _p(logits), ld, _p(labels)))


class FeatureCacheModel:
    """State of the set-associative, batch-synchronous LRU cache model (orc_cache_fetch)."""

    def __init__(self, n_sets, ways):
        self.n_sets, self.ways = int(n_sets), int(ways)
        self.keys = np.full(self.n_sets * self.ways, -1, dtype=np.int32)
        self.stamps = np.full(self.n_sets * self.ways, -1, dtype=np.int32)
        self.queries = 0
        self.misses = 0

    def fetch(self, ids, stamp):
        """Looks up / inserts the distinct node ids of one batch; returns (slots, n_miss); slot -1 = not cached."""
        ids = _arr(ids, np.int32)
        assert len(np.unique(ids)) == len(ids), "the ids of a batch must be distinct"
        slots = np.empty(len(ids), dtype=np.int32)
        n_miss = int(lib().orc_cache_fetch(self.n_sets, self.ways, _p(self.keys), _p(self.stamps), _p(ids), len(ids), int(stamp), _p(slots)))
        self.queries += len(ids)
        self.misses += n_miss
        return slots, n_miss


def _as_float_table(table):
    """float64 view of a float32 / raw-bf16 (uint16) table."""
    if table.dtype == np.uint16:
        return (table.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return np.asarray(table, dtype=np.float64)


def gcn_aggregate(blk: Block, table, graph_deg, indirect: bool, F=None):
    """GCN propagation on a sampled block (Section 6.4: the method applied to GCN; Kipf & Welling's rule with
    the renormalisation trick, A~ = A + I, d~ = deg + 1 taken on the full graph):

        exact :  out[v] = sum_{u in N(v) + {v}} H[u] / sqrt(d~_v d~_u)
        block :  out[v] = H[v] / d~_v + (deg_v / |N_s(v)|) / sqrt(d~_v) * sum_{u in N_s(v)} H[u] / sqrt(d~_u)

    i.e. the neighbour sum is estimated from the sampled neighbours (exact when all of them were taken; unbiased
    under uniform sampling), the self term is exact.  graph_deg: degrees of the full graph by global id.
    indirect: table rows are addressed by global id (input layer), else by local source position."""
    H = _as_float_table(table)
    F = H.shape[1] if F is None else F
    deg = np.asarray(graph_deg, dtype=np.float64)
    isd = 1.0 / np.sqrt(deg + 1.0)
    nodes = blk.src_ids.astype(np.int64)
    dst = nodes[:blk.n_dst]
    n_s = np.diff(blk.indptr).astype(np.float64)
    rows_e = np.repeat(np.arange(blk.n_dst), np.diff(blk.indptr))
    u_local = blk.indices[:blk.nnz].astype(np.int64)
    u_node = nodes[u_local]
    H_e = H[u_node, :F] if indirect else H[u_local, :F]
    acc = np.zeros((blk.n_dst, F), dtype=np.float64)
    np.add.at(acc, rows_e, H_e * isd[u_node][:, None])
    scale = np.where(n_s > 0, deg[dst] / np.maximum(n_s, 1.0) * isd[dst], 0.0)
    H_self = H[dst, :F] if indirect else H[:blk.n_dst, :F]
    return H_self / (deg[dst] + 1.0)[:, None] + scale[:, None] * acc


def gcn_aggregate_bwd(blk: Block, d_out, graph_deg):
    """Gradient of gcn_aggregate (dense addressing) with respect to the source rows: its transpose."""
    d_out = np.asarray(d_out, dtype=np.float64)
    F = d_out.shape[1]
    deg = np.asarray(graph_deg, dtype=np.float64)
    isd = 1.0 / np.sqrt(deg + 1.0)
    nodes = blk.src_ids.astype(np.int64)
    dst = nodes[:blk.n_dst]
    n_s = np.diff(blk.indptr).astype(np.float64)
    rows_e = np.repeat(np.arange(blk.n_dst), np.diff(blk.indptr))
    u_local = blk.indices[:blk.nnz].astype(np.int64)
    scale = np.where(n_s > 0, deg[dst] / np.maximum(n_s, 1.0) * isd[dst], 0.0)
    d_src = np.zeros((blk.n_src, F), dtype=np.float64)
    np.add.at(d_src, u_local, (scale[rows_e] * isd[nodes[u_local]])[:, None] * d_out[rows_e])
    d_src[:blk.n_dst] += d_out / (deg[dst] + 1.0)[:, None]
    return d_src


# ---------------------------------------------------------------------------------------------------------------
# Graph attention layer on a sampled block (Section 6.4 names GAT as the second model the method is applied to and
# gives no architecture; the layer is the one of Velickovic et al., "Graph Attention Networks", their equations
# for the attention coefficients, the neighbourhood softmax and the multi-head output with concatenated heads):
#     z[u]        = x[u] W                                    (shared linear map, split into `heads` groups of D columns)
#     e[v,u,h]    = LeakyReLU_slope( a_l[h] . z[u,h] + a_r[h] . z[v,h] )      for u in N_s(v)
#     alpha[v,.,h]= softmax of e[v,.,h] over N_s(v)
#     out[v,h]    = sum_u alpha[v,u,h] z[u,h] + bias[h]       (a row without sampled neighbours gets the bias alone)
# The attention vector of the original paper acts on the concatenation [z_v || z_u]; a_r and a_l are its two halves.
# The neighbourhood is the block's sampled in-neighbours, without an added self loop.
# ---------------------------------------------------------------------------------------------------------------
def gat_attention_fwd(blk: Block, z, a_l, a_r, bias, heads, slope=0.2):
    """z: [n_src, heads*D] projected source rows (destination v is source row v).  Returns (out [n_dst, heads*D],
    alpha: list over destinations of [deg, heads] arrays)."""
    z = np.asarray(z, dtype=np.float64)
    HD = z.shape[1]
    D = HD // heads
    a_l = np.asarray(a_l, dtype=np.float64).reshape(heads, D)
    a_r = np.asarray(a_r, dtype=np.float64).reshape(heads, D)
    bias = np.asarray(bias, dtype=np.float64).reshape(HD)
    z3 = z.reshape(-1, heads, D)
    out = np.zeros((blk.n_dst, HD))
    alphas = []
    for v in range(blk.n_dst):
        nb = blk.indices[blk.indptr[v]:blk.indptr[v + 1]].astype(np.int64)
        if len(nb) == 0:
            out[v] = bias
            alphas.append(np.zeros((0, heads)))
            continue
        s = np.einsum("uhd,hd->uh", z3[nb], a_l) + np.einsum("hd,hd->h", z3[v], a_r)[None, :]
        e = np.where(s > 0, s, slope * s)
        w = np.exp(e - e.max(axis=0, keepdims=True))
        alpha = w / w.sum(axis=0, keepdims=True)
        out[v] = np.einsum("uh,uhd->hd", alpha, z3[nb]).reshape(HD) + bias
        alphas.append(alpha)
    return out, alphas


def gat_attention_bwd(blk: Block, z, a_l, a_r, heads, d_out, slope=0.2):
    """Gradients of gat_attention_fwd for a given d_out = dL/d out: returns (d_z [n_src, heads*D], d_a_l, d_a_r,
    d_bias).  Chain rule written out per destination: value path (alpha z), softmax, LeakyReLU, the two dot products."""
    z = np.asarray(z, dtype=np.float64)
    d_out = np.asarray(d_out, dtype=np.float64)
    HD = z.shape[1]
    D = HD // heads
    a_l = np.asarray(a_l, dtype=np.float64).reshape(heads, D)
    a_r = np.asarray(a_r, dtype=np.float64).reshape(heads, D)
    z3 = z.reshape(-1, heads, D)
    g3 = d_out.reshape(-1, heads, D)
    d_z = np.zeros_like(z3)
    d_al = np.zeros_like(a_l)
    d_ar = np.zeros_like(a_r)
    d_bias = d_out.sum(axis=0)
    for v in range(blk.n_dst):
        nb = blk.indices[blk.indptr[v]:blk.indptr[v + 1]].astype(np.int64)
        if len(nb) == 0:
            continue
        s = np.einsum("uhd,hd->uh", z3[nb], a_l) + np.einsum("hd,hd->h", z3[v], a_r)[None, :]
        e = np.where(s > 0, s, slope * s)
        w = np.exp(e - e.max(axis=0, keepdims=True))
        alpha = w / w.sum(axis=0, keepdims=True)
        d_alpha = np.einsum("hd,uhd->uh", g3[v], z3[nb])                 # out = sum alpha z
        d_e = alpha * (d_alpha - (alpha * d_alpha).sum(axis=0, keepdims=True))   # softmax Jacobian
        d_s = d_e * np.where(s > 0, 1.0, slope)
        np.add.at(d_z, nb, alpha[:, :, None] * g3[v][None, :, :] + d_s[:, :, None] * a_l[None, :, :])
        d_z[v] += d_s.sum(axis=0)[:, None] * a_r
        d_al += np.einsum("uh,uhd->hd", d_s, z3[nb])
        d_ar += d_s.sum(axis=0)[:, None] * z3[v]
    return d_z.reshape(-1, HD), d_al.reshape(-1), d_ar.reshape(-1), d_bias
