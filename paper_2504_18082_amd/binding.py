"""ctypes binding of libcommrand.so: same names as the C ABI, argument marshalling only.

torch is used for device memory and streams (plumbing); no arithmetic of the method happens here.
The library must have been built (``python -m paper_2504_18082_amd.build``); loading fails loudly
otherwise -- there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libcommrand.so")

CR_MAX_LAYERS = 8
CR_MAX_FANOUT = 64
CR_HDR_WORDS = 8
CR_HDR_N_DST, CR_HDR_N_SRC, CR_HDR_NNZ, CR_HDR_STATUS = 0, 1, 2, 3
CR_OK, CR_ERR_INVALID_ARG, CR_ERR_CAPACITY, CR_ERR_UNSUPPORTED, CR_ERR_HIP, CR_ERR_ASYNC_OVERFLOW = range(6)
CR_CTX_DRY_RUN = 1
CR_CTX_STATUS_WORDS = 2
CR_ASYNC_TABLE_FULL, CR_ASYNC_FRONTIER_OVERFLOW = 1, 2
CR_ROOTS_NORAND, CR_ROOTS_COMM_RAND, CR_ROOTS_RAND = 0, 1, 2
CR_F32, CR_BF16 = 0, 1
CR_SAMPLE_STRICT_INTRA = 1
CR_SAMPLE_HASH_DEDUP = 2
CR_SAMPLE_INPUT_GLOBAL_IDS = 4
CR_SAMPLE_TRANSPOSE_INPUT = 8
CR_SAMPLE_ROW_ORDER = 16
CR_SAMPLE_SMALL_FRONTIER = 32
CR_SAMPLE_EXACT_RANKING = 64

EXPORTS = [
    "cr_last_error", "cr_version", "cr_mix_count_from_percent",
    "cr_ctx_create", "cr_ctx_destroy", "cr_ctx_make_current", "cr_ctx_poll_error",
    "cr_build_batches_workspace_bytes", "cr_build_batches", "cr_build_batches_static",
    "cr_graph_edge_classes", "cr_block_capacities", "cr_sample_blocks_workspace_bytes", "cr_sample_blocks_dedup_table", "cr_sample_blocks", "cr_selftest_clock_approximation",
    "cr_gather_aggregate_fwd", "cr_gather_aggregate_fwd_group", "cr_gather_aggregate_bwd",
    "cr_graph_gcn_norm", "cr_gcn_block_norm", "cr_gcn_aggregate_fwd", "cr_gcn_aggregate_fwd_group", "cr_gcn_aggregate_bwd",
    "cr_sage_padded_dims", "cr_sage_refresh_shadows", "cr_sage_linear_fwd", "cr_sage_linear_fwd_xent",
    "cr_sage_linear_bwd_workspace_bytes", "cr_sage_linear_bwd", "cr_sage_linear_bwd_input", "cr_sage_layer_bwd", "cr_softmax_xent",
    "cr_count_correct", "cr_mean_accumulate",
    "cr_gather_rows_bf16", "cr_gat_attention_fwd", "cr_gat_attention_bwd_workspace_bytes", "cr_gat_attention_bwd",
    "cr_cache_reset", "cr_cache_fetch", "cr_stage_rows", "cr_host_alloc", "cr_host_free",
]


class CrError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"cr_status {status}: {text}")
        self.status = status


class cr_batch_cfg(C.Structure):
    _fields_ = [("policy", C.c_int32), ("mix_count", C.c_int32), ("batch_size", C.c_int32),
                ("epoch", C.c_uint32), ("seed", C.c_uint64)]


class cr_graph(C.Structure):
    _fields_ = [("n_nodes", C.c_int64), ("n_entries", C.c_int64), ("indptr", C.c_void_p),
                ("indices", C.c_void_p), ("comm", C.c_void_p), ("n_comm", C.c_int32), ("reserved", C.c_int32),
                ("edge_intra", C.c_void_p)]


class cr_feature_cache(C.Structure):
    _fields_ = [("n_sets", C.c_int32), ("ways", C.c_int32), ("row_bytes", C.c_int32), ("n_overflow", C.c_int32),
                ("keys", C.c_void_p), ("stamps", C.c_void_p), ("rows", C.c_void_p), ("set_count", C.c_void_p),
                ("set_list", C.c_void_p), ("counters", C.c_void_p)]


CR_CACHE_LIST_CAP = 64


class cr_block_set(C.Structure):
    _fields_ = [("n_batches", C.c_int32), ("fanout", C.c_int32), ("cap_dst", C.c_int32),
                ("cap_src", C.c_int32), ("cap_nnz", C.c_int32), ("reserved", C.c_int32),
                ("hdr", C.c_void_p), ("src_ids", C.c_void_p), ("indptr", C.c_void_p),
                ("indices", C.c_void_p), ("t_indptr", C.c_void_p), ("t_indices", C.c_void_p),
                ("gather_ids", C.c_void_p), ("row_order", C.c_void_p), ("group_order", C.c_void_p)]


class cr_sample_cfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("fanout", C.c_int32 * CR_MAX_LAYERS),
                ("p_intra", C.c_double), ("seed", C.c_uint64), ("epoch", C.c_uint32),
                ("first_batch", C.c_uint32), ("flags", C.c_uint32), ("reserved", C.c_uint32)]


class cr_sage_layer(C.Structure):
    _fields_ = [("F_in", C.c_int32), ("F_out", C.c_int32), ("n_operands", C.c_int32), ("reserved", C.c_int32),
                ("W", C.c_void_p), ("bias", C.c_void_p), ("W_bf16", C.c_void_p), ("Wt_bf16", C.c_void_p)]


class cr_gat_params(C.Structure):
    _fields_ = [("heads", C.c_int32), ("D", C.c_int32), ("slope", C.c_float), ("reserved", C.c_int32), ("attn", C.c_void_p)]


_lib = None


def lib():
    """The loaded library; raises if it was not built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2504_18082_amd.build`")
        # torch first: the library must bind to the HIP runtime that torch brings into the process (a second copy of the
        # runtime, loaded from the system before torch's, sees no device)
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64
        L.cr_last_error.restype = C.c_char_p
        L.cr_version.restype = C.c_char_p
        L.cr_ctx_create.argtypes = [C.POINTER(vp), i32, C.c_uint32, vp]
        L.cr_ctx_destroy.argtypes = [vp]
        L.cr_ctx_make_current.argtypes = [vp]
        L.cr_ctx_poll_error.argtypes = [vp, C.POINTER(i64), i32, vp]
        L.cr_mix_count_from_percent.argtypes = [C.c_double, i32]
        L.cr_mix_count_from_percent.restype = i32
        L.cr_build_batches_workspace_bytes.argtypes = [i64, i32, C.POINTER(C.c_size_t)]
        L.cr_build_batches.argtypes = [C.POINTER(cr_batch_cfg), vp, i64, vp, i32, vp, C.c_size_t, vp,
                                       C.POINTER(i64), vp]
        L.cr_build_batches_static.argtypes = [C.POINTER(cr_batch_cfg), vp, i64, vp, i32, vp, C.POINTER(i64), vp]
        L.cr_block_capacities.argtypes = [C.POINTER(cr_sample_cfg), i64, i32, C.POINTER(i32),
                                          C.POINTER(i32), C.POINTER(i32)]
        L.cr_sample_blocks_workspace_bytes.argtypes = [C.POINTER(cr_sample_cfg), i64, i32, i32,
                                                       C.POINTER(C.c_size_t)]
        L.cr_sample_blocks_dedup_table.argtypes = [C.POINTER(cr_sample_cfg), i64, i32, C.POINTER(i32)]
        L.cr_selftest_clock_approximation.argtypes = [vp, vp]
        L.cr_graph_edge_classes.argtypes = [C.POINTER(cr_graph), vp, vp]
        L.cr_sample_blocks.argtypes = [C.POINTER(cr_graph), C.POINTER(cr_sample_cfg), vp, i64, i32, i32,
                                       vp, C.c_size_t, C.POINTER(cr_block_set), vp]
        L.cr_gather_aggregate_fwd.argtypes = [C.POINTER(cr_block_set), i32, vp, i32, i64, i32, i32, vp, vp,
                                              vp, i64, vp]
        L.cr_gather_aggregate_fwd_group.argtypes = [C.POINTER(cr_block_set), vp, i32, i64, i32, vp, vp, i64, i64, vp]
        L.cr_gather_aggregate_bwd.argtypes = [C.POINTER(cr_block_set), i32, vp, vp, i32, i64, i32, vp, i32, i64, vp,
                                              vp, i64, vp]
        L.cr_graph_gcn_norm.argtypes = [C.POINTER(cr_graph), vp, vp]
        L.cr_gcn_block_norm.argtypes = [C.POINTER(cr_block_set), i32, vp, vp, vp]
        L.cr_gcn_aggregate_fwd.argtypes = [C.POINTER(cr_block_set), i32, vp, vp, vp, i32, i64, i32, i32, vp, vp, i64, vp]
        L.cr_gcn_aggregate_bwd.argtypes = [C.POINTER(cr_block_set), i32, vp, vp, i32, i64, i32, vp, i32, i64, vp, vp, i64, vp]
        L.cr_gcn_aggregate_fwd_group.argtypes = [C.POINTER(cr_block_set), vp, vp, i32, i64, i32, vp, i64, i64, vp]
        L.cr_sage_padded_dims.argtypes = [i32, i32, C.POINTER(i32), C.POINTER(i32)]
        L.cr_sage_refresh_shadows.argtypes = [C.POINTER(cr_sage_layer), vp]
        L.cr_sage_linear_fwd.argtypes = [C.POINTER(cr_sage_layer), vp, i32, vp, vp, i64, C.c_int, vp, vp, vp]
        L.cr_sage_linear_fwd_xent.argtypes = [C.POINTER(cr_sage_layer), vp, i32, vp, vp, i64, vp, i32, vp, vp, vp, vp, vp, vp, vp]
        L.cr_sage_linear_bwd_workspace_bytes.argtypes = [i32, i32, i32, C.POINTER(C.c_size_t)]
        L.cr_sage_linear_bwd.argtypes = [C.POINTER(cr_sage_layer), vp, i32, vp, vp, i64, vp, C.c_float,
                                         C.c_float, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.cr_sage_linear_bwd_input.argtypes = [C.POINTER(cr_sage_layer), vp, i32, vp, vp, vp, vp, vp]
        L.cr_sage_layer_bwd.argtypes = [C.POINTER(cr_sage_layer), C.POINTER(cr_block_set), i32, vp, vp, i64, vp, C.c_float, C.c_float,
                                        vp, vp, i64, vp, i64, vp, vp, vp, C.c_size_t, vp]
        L.cr_softmax_xent.argtypes = [vp, i32, vp, i64, i32, vp, vp, vp, vp, vp, vp, vp]
        L.cr_count_correct.argtypes = [vp, i32, vp, i64, i32, vp, vp, vp, vp]
        L.cr_mean_accumulate.argtypes = [vp, i32, vp, vp, vp]
        L.cr_gather_rows_bf16.argtypes = [vp, i32, i64, i32, vp, vp, i32, i32, vp, i64, vp]
        L.cr_gat_attention_fwd.argtypes = [C.POINTER(cr_block_set), i32, C.POINTER(cr_gat_params), vp, i64, i32, vp, vp, vp, vp, vp, vp]
        L.cr_gat_attention_bwd_workspace_bytes.argtypes = [i32, i64, i32, C.POINTER(C.c_size_t)]
        L.cr_gat_attention_bwd.argtypes = [C.POINTER(cr_block_set), i32, C.POINTER(cr_gat_params), vp, i64, vp, vp, vp, i64, vp,
                                           C.c_float, C.c_float, vp, vp, vp, C.c_size_t, vp]
        L.cr_cache_reset.argtypes = [C.POINTER(cr_feature_cache), vp]
        L.cr_cache_fetch.argtypes = [C.POINTER(cr_feature_cache), vp, i64, vp, vp, i32, i32, i32, vp, vp]
        L.cr_stage_rows.argtypes = [vp, i64, vp, vp, i32, i32, vp, i32, vp]
        L.cr_host_alloc.argtypes = [C.c_size_t, C.POINTER(vp), C.POINTER(vp)]
        L.cr_host_free.argtypes = [vp]
        for name in EXPORTS:
            fn = getattr(L, name)
            if name not in ("cr_last_error", "cr_version", "cr_mix_count_from_percent"):
                fn.restype = i32
        _lib = L
    return _lib


def _check(status):
    if status != CR_OK:
        raise CrError(status, lib().cr_last_error().decode())


def _ptr(t):
    """Device (or host) address of a torch tensor / None."""
    return None if t is None else C.c_void_p(t.data_ptr())


_raw_stream = None


def _stream(stream=None):
    """The HIP stream to launch on: the given torch stream, else torch's current one (looked up through the raw
    accessor when this torch has it: a fraction of the cost of building a Stream object per call)."""
    global _raw_stream
    if stream is not None:
        return C.c_void_p(stream.cuda_stream)
    import torch
    if _raw_stream is None:
        get = getattr(torch._C, "_cuda_getCurrentRawStream", None)
        _raw_stream = (lambda: get(torch.cuda.current_device())) if get is not None else (lambda: torch.cuda.current_stream().cuda_stream)
    return C.c_void_p(_raw_stream())


# --------------------------------------------------------------------------- small host helpers
def cr_version() -> str:
    return lib().cr_version().decode()


class Context:
    """A cr_ctx: the dry-run flag and (optionally) the device status words that kernels record overflows in.
    The entry points follow the context that is current on the calling thread."""

    def __init__(self, device: int = 0, dry_run: bool = False, status=None):
        """status: a zeroed device int64[CR_CTX_STATUS_WORDS] tensor (kept alive here), or None."""
        self.status = status
        h = C.c_void_p()
        _check(lib().cr_ctx_create(C.byref(h), device, CR_CTX_DRY_RUN if dry_run else 0, _ptr(status)))
        self.handle = h

    def make_current(self):
        _check(lib().cr_ctx_make_current(self.handle))

    @staticmethod
    def make_none_current():
        _check(lib().cr_ctx_make_current(None))

    def poll_error(self, clear: bool = True, stream=None):
        """(status code, required): (CR_OK, 0) or (CR_ERR_ASYNC_OVERFLOW, the frontier length that was needed)."""
        req = C.c_int64(0)
        st = lib().cr_ctx_poll_error(self.handle, C.byref(req), int(clear), _stream(stream))
        if st not in (CR_OK, CR_ERR_ASYNC_OVERFLOW):
            _check(st)
        return st, req.value

    def destroy(self):
        if self.handle is not None and self.handle.value:
            lib().cr_ctx_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


_dry_ctx = None


def cr_set_dry_run(on: bool):
    """Puts the calling thread under a dry-run context (calls validate, then return without touching the GPU), or
    back under no context."""
    global _dry_ctx
    if on:
        if _dry_ctx is None:
            _dry_ctx = Context(dry_run=True)
        _dry_ctx.make_current()
    else:
        Context.make_none_current()


def cr_mix_count_from_percent(k_percent: float, n_comm_in_train: int) -> int:
    return int(lib().cr_mix_count_from_percent(k_percent, n_comm_in_train))


def make_sample_cfg(fanouts: Sequence[int], p_intra: float, seed: int, epoch: int, first_batch: int = 0,
                    flags: int = 0) -> cr_sample_cfg:
    cfg = cr_sample_cfg()
    cfg.n_layers = len(fanouts)
    for i, f in enumerate(fanouts[:CR_MAX_LAYERS]):
        cfg.fanout[i] = int(f)
    cfg.p_intra, cfg.seed, cfg.epoch, cfg.first_batch, cfg.flags = p_intra, seed, epoch, first_batch, flags
    return cfg


def cr_block_capacities(cfg: cr_sample_cfg, n_nodes: int, batch_size: int):
    L = max(1, min(cfg.n_layers, CR_MAX_LAYERS))
    a, b, c = (C.c_int32 * L)(), (C.c_int32 * L)(), (C.c_int32 * L)()
    _check(lib().cr_block_capacities(C.byref(cfg), n_nodes, batch_size, a, b, c))
    return list(a), list(b), list(c)


class BlockSet:
    """Device storage of one layer's blocks for a group of batches (torch int32 tensors)."""

    def __init__(self, n_batches, fanout, cap_dst, cap_src, cap_nnz, transposed, device="cuda", gather_ids=False, row_order=False,
                 group_order=False):
        import torch
        z = lambda *shape: torch.zeros(shape, dtype=torch.int32, device=device)
        self.n_batches, self.fanout = n_batches, fanout
        self.cap_dst, self.cap_src, self.cap_nnz = cap_dst, cap_src, cap_nnz
        self.hdr = z(n_batches, CR_HDR_WORDS)
        self.src_ids = z(n_batches, cap_src)
        self.indptr = z(n_batches, cap_dst + 1)
        self.indices = z(n_batches, cap_nnz)
        self.t_indptr = z(n_batches, cap_src + 1) if transposed else None
        self.t_indices = z(n_batches, cap_nnz) if transposed else None
        self.gather_ids = z(n_batches, cap_nnz) if gather_ids else None
        self.row_order = z(n_batches, cap_dst) if row_order else None       # processing order of the destination rows
        self.group_order = z(n_batches * cap_dst + 1) if group_order else None   # the same over the whole group (+ count)
        self.c = cr_block_set(n_batches, fanout, cap_dst, cap_src, cap_nnz, 0, _ptr(self.hdr),
                              _ptr(self.src_ids), _ptr(self.indptr), _ptr(self.indices),
                              _ptr(self.t_indptr), _ptr(self.t_indices), _ptr(self.gather_ids), _ptr(self.row_order),
                              _ptr(self.group_order))

    def hdr_ptr(self, g):
        return C.c_void_p(self.hdr.data_ptr() + g * CR_HDR_WORDS * 4)

    def src_ids_ptr(self, g):
        return C.c_void_p(self.src_ids.data_ptr() + g * self.cap_src * 4)

    @classmethod
    def from_host(cls, blk, fanout, device="cuda", gather_ids=False):
        """Upload one oracle/numpy block (n_dst, src_ids, indptr, indices[, t_indptr, t_indices]);
        gather_ids=True also uploads the per-edge global ids src_ids[indices]."""
        import numpy as np
        import torch
        tr = getattr(blk, "t_indptr", None) is not None
        cap_dst, cap_src, cap_nnz = max(1, blk.n_dst), max(1, blk.n_src, blk.n_dst), max(1, blk.nnz)
        order = getattr(blk, "row_order", None)
        bs = cls(1, fanout, cap_dst, cap_src, cap_nnz, tr, device, gather_ids, row_order=order is not None)
        if order is not None:
            bs.row_order[0, :blk.n_dst] = torch.from_numpy(np.ascontiguousarray(order, dtype=np.int32)).to(device)
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(device)
        bs.hdr[0, :3] = up([blk.n_dst, blk.n_src, blk.nnz])
        bs.src_ids[0, :blk.n_src] = up(blk.src_ids)
        bs.indptr[0, :blk.n_dst + 1] = up(blk.indptr[:blk.n_dst + 1])
        bs.indices[0, :blk.nnz] = up(blk.indices)
        if gather_ids:
            bs.gather_ids[0, :blk.nnz] = up(blk.src_ids[blk.indices])
        if tr:
            bs.t_indptr[0, :blk.n_src + 1] = up(blk.t_indptr)
            bs.t_indices[0, :blk.nnz] = up(blk.t_indices)
        return bs


def alloc_block_sets(cfg: cr_sample_cfg, n_nodes: int, batch_size: int, n_batches: int,
                     device="cuda", transpose_input: bool = False, order_input: bool = False,
                     group_order_input: bool = False) -> List[BlockSet]:
    """transpose_input: layer 0 gets a transposed block too (sampling then needs CR_SAMPLE_TRANSPOSE_INPUT);
    order_input / group_order_input: layer 0 gets a processing order of its destination rows (grouped by community),
    per batch / over the whole group."""
    cap_dst, cap_src, cap_nnz = cr_block_capacities(cfg, n_nodes, batch_size)
    return [BlockSet(n_batches, cfg.fanout[l], cap_dst[l], cap_src[l], cap_nnz[l], l >= 1 or transpose_input, device, gather_ids=(l == 0),
                     row_order=(order_input and l == 0), group_order=(group_order_input and l == 0))
            for l in range(cfg.n_layers)]


# --------------------------------------------------------------------------- step 1
def cr_build_batches_workspace_bytes(n_train: int, n_comm: int) -> int:
    n = C.c_size_t(0)
    _check(lib().cr_build_batches_workspace_bytes(n_train, n_comm, C.byref(n)))
    return n.value


def cr_build_batches(policy, mix_count, batch_size, seed, epoch, train_ids, comm, n_comm, ws, out_perm,
                     stream=None) -> int:
    cfg = cr_batch_cfg(policy, mix_count, batch_size, epoch, seed)
    nb = C.c_int64(0)
    _check(lib().cr_build_batches(C.byref(cfg), _ptr(train_ids), train_ids.numel(), _ptr(comm), n_comm,
                                  _ptr(ws), ws.numel() * ws.element_size(), _ptr(out_perm), C.byref(nb),
                                  _stream(stream)))
    return nb.value


CR_STATIC_MAX_TRAIN, CR_STATIC_MAX_COMM = 262144, 65536


def cr_build_batches_static(policy, mix_count, batch_size, seed, epoch, train_ids, comm, n_comm, out_perm, stream=None) -> int:
    """cr_build_batches without a workspace argument (the library's fixed scratch array; allocates nothing)."""
    cfg = cr_batch_cfg(policy, mix_count, batch_size, epoch, seed)
    nb = C.c_int64(0)
    _check(lib().cr_build_batches_static(C.byref(cfg), _ptr(train_ids), train_ids.numel(), _ptr(comm), n_comm,
                                         _ptr(out_perm), C.byref(nb), _stream(stream)))
    return nb.value


# --------------------------------------------------------------------------- step 2
def make_graph(indptr, indices, comm, n_comm, edge_intra=None) -> cr_graph:
    return cr_graph(indptr.numel() - 1, indices.numel(), _ptr(indptr), _ptr(indices), _ptr(comm), n_comm, 0, _ptr(edge_intra))


def cr_graph_edge_classes(graph: cr_graph, stream=None):
    """Allocates and fills the per-entry class bits of a graph; returns the tensor (int32 words); the caller stores
    its address in graph.edge_intra (and keeps the tensor alive)."""
    import torch
    words = max(1, -(-graph.n_entries // 32))
    bits = torch.zeros(words, dtype=torch.int32, device="cuda")
    _check(lib().cr_graph_edge_classes(C.byref(graph), _ptr(bits), _stream(stream)))
    return bits


def cr_sample_blocks_workspace_bytes(cfg, n_nodes, batch_size, n_batches) -> int:
    n = C.c_size_t(0)
    _check(lib().cr_sample_blocks_workspace_bytes(C.byref(cfg), n_nodes, batch_size, n_batches, C.byref(n)))
    return n.value


CR_DEDUP_DIRECT, CR_DEDUP_HASH = 0, 1


def cr_selftest_clock_approximation(result, stream=None):
    _check(lib().cr_selftest_clock_approximation(_ptr(result), _stream(stream)))


def cr_sample_blocks_dedup_table(cfg, n_nodes, batch_size) -> int:
    kind = C.c_int32(-1)
    _check(lib().cr_sample_blocks_dedup_table(C.byref(cfg), n_nodes, batch_size, C.byref(kind)))
    return kind.value


def cr_sample_blocks(graph: cr_graph, cfg: cr_sample_cfg, roots, n_roots_total, batch_size, n_batches, ws,
                     layers: List[BlockSet], stream=None):
    arr = (cr_block_set * len(layers))(*[b.c for b in layers])
    _check(lib().cr_sample_blocks(C.byref(graph), C.byref(cfg), _ptr(roots), n_roots_total, batch_size,
                                  n_batches, _ptr(ws), ws.numel() * ws.element_size(), arr, _stream(stream)))


# --------------------------------------------------------------------------- training on the sub-graph
def cr_gather_aggregate_fwd(blocks: BlockSet, g, H_src, dtype, ld_src, F, indirect, agg=None, agg_bf16=None,
                            self_bf16=None, ld_bf16=0, stream=None):
    H_ptr = H_src if isinstance(H_src, C.c_void_p) else _ptr(H_src)
    _check(lib().cr_gather_aggregate_fwd(C.byref(blocks.c), g, H_ptr, dtype, ld_src, F, int(indirect),
                                         _ptr(agg), _ptr(agg_bf16), _ptr(self_bf16), ld_bf16, _stream(stream)))


def cr_gather_aggregate_fwd_group(blocks, H_src, dtype, ld_src, F, agg_bf16, self_bf16, batch_stride_rows, ld_bf16, stream=None):
    """blocks: a BlockSet or a view of its first batches (anything with a .c descriptor)."""
    H_ptr = H_src if isinstance(H_src, C.c_void_p) else _ptr(H_src)
    _check(lib().cr_gather_aggregate_fwd_group(C.byref(blocks.c), H_ptr, dtype, ld_src, F, _ptr(agg_bf16), _ptr(self_bf16),
                                               batch_stride_rows, ld_bf16, _stream(stream)))


def cr_gather_aggregate_bwd(blocks: BlockSet, g, d_agg, d_self, ld_in, F, relu_out=None, ld_relu=0, d_src=None,
                            d_src_bf16=None, ld_bf16=0, stream=None, relu_dtype=CR_F32, in_dtype=CR_F32):
    """d_agg / d_self: tensors, or raw device addresses (ctypes.c_void_p) for views into a shared buffer."""
    as_ptr = lambda t: t if isinstance(t, C.c_void_p) else _ptr(t)
    _check(lib().cr_gather_aggregate_bwd(C.byref(blocks.c), g, as_ptr(d_agg), as_ptr(d_self), in_dtype, ld_in, F,
                                         _ptr(relu_out), relu_dtype, ld_relu, _ptr(d_src), _ptr(d_src_bf16), ld_bf16,
                                         _stream(stream)))


def cr_gcn_aggregate_fwd_group(blocks, norm, H_src, dtype, ld_src, F, agg_bf16, batch_stride_rows, ld_bf16, stream=None):
    """blocks: a BlockSet or a view of its first batches (anything with a cr_block_set in .c)."""
    as_ptr = lambda t: t if isinstance(t, C.c_void_p) else _ptr(t)
    _check(lib().cr_gcn_aggregate_fwd_group(C.byref(blocks.c), _ptr(norm), as_ptr(H_src), dtype, ld_src, F, _ptr(agg_bf16), batch_stride_rows,
                                            ld_bf16, _stream(stream)))


def cr_graph_gcn_norm(graph: cr_graph, stream=None):
    """Allocates and fills the per-node GCN normalisation of a graph: float tensor [n_nodes, 2]."""
    import torch
    norm = torch.zeros((graph.n_nodes, 2), dtype=torch.float32, device="cuda")
    _check(lib().cr_graph_gcn_norm(C.byref(graph), _ptr(norm), _stream(stream)))
    return norm


def cr_gcn_block_norm(blocks, g, norm, blk_norm, stream=None):
    _check(lib().cr_gcn_block_norm(C.byref(blocks.c), g, _ptr(norm), _ptr(blk_norm), _stream(stream)))


def cr_gcn_aggregate_fwd(blocks, g, norm, blk_norm, H_src, dtype, ld_src, F, indirect, agg=None, agg_bf16=None, ld_bf16=0, stream=None):
    H_ptr = H_src if isinstance(H_src, C.c_void_p) else _ptr(H_src)
    _check(lib().cr_gcn_aggregate_fwd(C.byref(blocks.c), g, _ptr(norm), _ptr(blk_norm), H_ptr, dtype, ld_src, F, int(indirect),
                                      _ptr(agg), _ptr(agg_bf16), ld_bf16, _stream(stream)))


def cr_gcn_aggregate_bwd(blocks, g, blk_norm, d_out, ld_in, F, relu_out=None, ld_relu=0, d_src=None, d_src_bf16=None, ld_bf16=0,
                         stream=None, relu_dtype=CR_F32, in_dtype=CR_F32):
    _check(lib().cr_gcn_aggregate_bwd(C.byref(blocks.c), g, _ptr(blk_norm), _ptr(d_out), in_dtype, ld_in, F, _ptr(relu_out), relu_dtype,
                                      ld_relu, _ptr(d_src), _ptr(d_src_bf16), ld_bf16, _stream(stream)))


def cr_sage_padded_dims(F_in, F_out):
    a, b = C.c_int32(0), C.c_int32(0)
    _check(lib().cr_sage_padded_dims(F_in, F_out, C.byref(a), C.byref(b)))
    return a.value, b.value


class SageLayer:
    """Device storage of one layer's parameters: float master + two bf16 shadows.  n_operands = 2: GraphSAGE
    (W = [W_self; W_neigh]); 1: a single aggregated input (GCN)."""

    def __init__(self, W_host, b_host, device="cuda", n_operands=2):
        import torch
        F2, F_out = W_host.shape
        self.n_operands = n_operands
        self.F_in, self.F_out = F2 // n_operands, F_out
        self.F_pad, self.N_pad = cr_sage_padded_dims(self.F_in, F_out)
        self.W = torch.from_numpy(W_host).to(device=device, dtype=torch.float32).contiguous()
        self.bias = torch.zeros(self.N_pad, dtype=torch.float32, device=device)
        self.bias[:F_out] = torch.from_numpy(b_host).to(device)
        self.W_bf16 = torch.zeros((n_operands * self.F_pad, self.N_pad), dtype=torch.int16, device=device)
        self.Wt_bf16 = torch.zeros((self.N_pad, n_operands * self.F_pad), dtype=torch.int16, device=device)
        self.c = cr_sage_layer(self.F_in, self.F_out, n_operands, 0, _ptr(self.W), _ptr(self.bias), _ptr(self.W_bf16),
                               _ptr(self.Wt_bf16))

    def refresh(self, stream=None):
        _check(lib().cr_sage_refresh_shadows(C.byref(self.c), _stream(stream)))

    def drop_bias(self):
        """Turns the layer into one without a bias term (the graph-attention projection)."""
        self.bias = None
        self.c.bias = None


def cr_sage_linear_fwd(layer: SageLayer, hdr_ptr, max_rows, h_self, agg, ld_in, relu, out=None, out_bf16=None,
                       stream=None):
    _check(lib().cr_sage_linear_fwd(C.byref(layer.c), hdr_ptr, max_rows, _ptr(h_self), _ptr(agg), ld_in,
                                    int(relu), _ptr(out), _ptr(out_bf16), _stream(stream)))


def cr_sage_linear_bwd_workspace_bytes(F_in, F_out, max_rows) -> int:
    n = C.c_size_t(0)
    _check(lib().cr_sage_linear_bwd_workspace_bytes(F_in, F_out, max_rows, C.byref(n)))
    return n.value


CR_XENT_SCRATCH_BYTES = 512


def cr_sage_linear_fwd_xent(layer: SageLayer, hdr_ptr, max_rows, h_self, agg, ld_in, logits, n_classes, labels, root_ids_ptr, loss,
                            row_loss, d_logits_bf16, scratch, stream=None):
    _check(lib().cr_sage_linear_fwd_xent(C.byref(layer.c), hdr_ptr, max_rows, _ptr(h_self), _ptr(agg), ld_in, _ptr(logits), n_classes,
                                         _ptr(labels), root_ids_ptr, _ptr(loss), _ptr(row_loss), _ptr(d_logits_bf16), _ptr(scratch),
                                         _stream(stream)))


def cr_sage_linear_bwd(layer: SageLayer, hdr_ptr, max_rows, h_self, agg, ld_in, dz_bf16, lr, weight_decay,
                       d_self, d_agg, ws, dW_out=None, db_out=None, stream=None, d_in_bf16=None):
    _check(lib().cr_sage_linear_bwd(C.byref(layer.c), hdr_ptr, max_rows, _ptr(h_self), _ptr(agg), ld_in,
                                    _ptr(dz_bf16), lr, weight_decay, _ptr(d_self), _ptr(d_agg), _ptr(d_in_bf16), _ptr(dW_out),
                                    _ptr(db_out), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))


def cr_sage_linear_bwd_input(layer: SageLayer, hdr_ptr, max_rows, dz_bf16, d_self, d_agg, stream=None, d_in_bf16=None):
    _check(lib().cr_sage_linear_bwd_input(C.byref(layer.c), hdr_ptr, max_rows, _ptr(dz_bf16), _ptr(d_self), _ptr(d_agg),
                                          _ptr(d_in_bf16), _stream(stream)))


def cr_sage_layer_bwd(layer: SageLayer, blocks: BlockSet, g, h_self, agg, ld_in, dz_bf16, lr, weight_decay, d_in_bf16,
                      relu_out_bf16, ld_relu, d_src_bf16, ld_bf16, ws, dW_out=None, db_out=None, stream=None):
    _check(lib().cr_sage_layer_bwd(C.byref(layer.c), C.byref(blocks.c), g, _ptr(h_self), _ptr(agg), ld_in, _ptr(dz_bf16), lr,
                                   weight_decay, _ptr(d_in_bf16), _ptr(relu_out_bf16), ld_relu, _ptr(d_src_bf16), ld_bf16,
                                   _ptr(dW_out), _ptr(db_out), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))


def cr_softmax_xent(hdr_ptr, max_rows, logits, ld, n_classes, labels, root_ids_ptr, loss, row_loss,
                    d_logits=None, d_logits_bf16=None, stream=None):
    _check(lib().cr_softmax_xent(hdr_ptr, max_rows, _ptr(logits), ld, n_classes, _ptr(labels), root_ids_ptr,
                                 _ptr(loss), _ptr(row_loss), _ptr(d_logits), _ptr(d_logits_bf16),
                                 _stream(stream)))


def cr_count_correct(hdr_ptr, max_rows, logits, ld, n_classes, labels, root_ids_ptr, count, stream=None):
    _check(lib().cr_count_correct(hdr_ptr, max_rows, _ptr(logits), ld, n_classes, _ptr(labels), root_ids_ptr, _ptr(count),
                                  _stream(stream)))


def cr_mean_accumulate(hdr_ptr, max_rows, value, acc, stream=None):
    _check(lib().cr_mean_accumulate(hdr_ptr, max_rows, _ptr(value), _ptr(acc), _stream(stream)))


class GatParams:
    """Device storage of one graph-attention layer's attention vectors and bias: float [3][N_pad] = a_l, a_r, bias."""

    def __init__(self, a_l, a_r, bias, heads, N_pad, slope=0.2, device="cuda"):
        import numpy as np
        import torch
        HD = len(bias)
        assert HD % heads == 0 and len(a_l) == HD and len(a_r) == HD and HD <= N_pad
        host = np.zeros((3, N_pad), dtype=np.float32)
        host[0, :HD], host[1, :HD], host[2, :HD] = a_l, a_r, bias
        self.heads, self.D, self.N_pad, self.slope = heads, HD // heads, N_pad, slope
        self.attn = torch.from_numpy(host).to(device)
        self.c = cr_gat_params(heads, HD // heads, slope, 0, _ptr(self.attn))


def cr_gather_rows_bf16(store, dtype, ld_src, F, ids_ptr, hdr_ptr, hdr_word, max_n, rows_out, ld_out, stream=None):
    store_ptr = store if isinstance(store, C.c_void_p) else _ptr(store)
    _check(lib().cr_gather_rows_bf16(store_ptr, dtype, ld_src, F, ids_ptr, hdr_ptr, hdr_word, max_n, _ptr(rows_out), ld_out,
                                     _stream(stream)))


def cr_gat_attention_fwd(blocks, g, params: GatParams, z_bf16, ld, relu, el, er, stat, out=None, out_bf16=None, stream=None):
    _check(lib().cr_gat_attention_fwd(C.byref(blocks.c), g, C.byref(params.c), _ptr(z_bf16), ld, int(relu), _ptr(el), _ptr(er),
                                      _ptr(stat), _ptr(out), _ptr(out_bf16), _stream(stream)))


def cr_gat_attention_bwd_workspace_bytes(cap_dst, ld, heads) -> int:
    n = C.c_size_t(0)
    _check(lib().cr_gat_attention_bwd_workspace_bytes(cap_dst, ld, heads, C.byref(n)))
    return n.value


def cr_gat_attention_bwd(blocks, g, params: GatParams, z_bf16, ld, el, stat, d_out_bf16, ld_dout, relu_out_bf16, lr, weight_decay,
                         dz_bf16, ws, d_attn_out=None, stream=None):
    _check(lib().cr_gat_attention_bwd(C.byref(blocks.c), g, C.byref(params.c), _ptr(z_bf16), ld, _ptr(el), _ptr(stat),
                                      _ptr(d_out_bf16), ld_dout, _ptr(relu_out_bf16), lr, weight_decay, _ptr(dz_bf16),
                                      _ptr(d_attn_out), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))


def cr_stage_rows(store_ptr, store_ld_bytes, ids_ptr, hdr_ptr, hdr_word, max_n, rows_out, row_bytes, stream=None):
    _check(lib().cr_stage_rows(store_ptr, store_ld_bytes, ids_ptr, hdr_ptr, hdr_word, max_n, _ptr(rows_out), row_bytes, _stream(stream)))


class FeatureCache:
    """Device storage of a software-managed feature cache (set-associative LRU, updated once per batch)."""

    def __init__(self, n_sets: int, ways: int, row_bytes: int, max_batch_nodes: int, device="cuda"):
        import torch
        self.n_sets, self.ways, self.row_bytes, self.max_n = n_sets, ways, row_bytes, max_batch_nodes
        slots = n_sets * ways
        i32 = lambda n: torch.zeros(n, dtype=torch.int32, device=device)
        self.keys, self.stamps = i32(slots), i32(slots)
        self.rows = torch.zeros((slots + max_batch_nodes, row_bytes), dtype=torch.uint8, device=device)
        self.set_count, self.set_list, self.counters = i32(n_sets), i32(n_sets * CR_CACHE_LIST_CAP), i32(8)
        self.slot_out = i32(max_batch_nodes)
        self.c = cr_feature_cache(n_sets, ways, row_bytes, max_batch_nodes, _ptr(self.keys), _ptr(self.stamps), _ptr(self.rows),
                                  _ptr(self.set_count), _ptr(self.set_list), _ptr(self.counters))
        self.reset()

    def reset(self, stream=None):
        _check(lib().cr_cache_reset(C.byref(self.c), _stream(stream)))

    def fetch(self, store_ptr, store_ld_bytes, ids_ptr, hdr_ptr, hdr_word, stamp, stream=None):
        """store_ptr / ids_ptr / hdr_ptr: raw addresses (ctypes.c_void_p) the GPU can read."""
        _check(lib().cr_cache_fetch(C.byref(self.c), store_ptr, store_ld_bytes, ids_ptr, hdr_ptr, hdr_word, self.max_n, stamp,
                                    _ptr(self.slot_out), _stream(stream)))

    def stats(self):
        """(look-ups, misses, misses served from the overflow area, status) since the last reset."""
        c = self.counters.cpu().numpy()
        return int(c[0]), int(c[1]), int(c[2]), int(c[3])


class HostBuffer:
    """Pinned host memory that kernels can read (cr_host_alloc); .array is a numpy view for the CPU side."""

    def __init__(self, shape, dtype):
        import numpy as np
        self.shape, self.dtype = tuple(shape), np.dtype(dtype)
        self.nbytes = int(np.prod(self.shape)) * self.dtype.itemsize
        h, d = C.c_void_p(), C.c_void_p()
        _check(lib().cr_host_alloc(self.nbytes, C.byref(h), C.byref(d)))
        self.host_ptr, self.device_ptr = h, d
        buf = (C.c_char * self.nbytes).from_address(h.value)
        self.array = np.frombuffer(buf, dtype=self.dtype).reshape(self.shape)

    def free(self):
        if self.host_ptr is not None and self.host_ptr.value:
            self.array = None
            _check(lib().cr_host_free(self.host_ptr))
            self.host_ptr = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass
