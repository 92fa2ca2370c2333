"""Epoch driver: sequences the C-ABI calls of Algorithm 1 (root partitioning, grouped sub-graph
sampling, then forward / loss / backward / SGD per mini-batch).  Call sequencing and buffer
ownership only -- every arithmetic step runs inside libcommrand.so.

`run_epoch_serial` (the default everywhere) issues every call on the current stream.  `run_epoch` is
the optional overlapped schedule: sampling and the layer-0 feature gather do not depend on the
weights, so it issues them on side streams (default priority) ahead of the training stream; block
storage and the layer-0 operand buffers are double-buffered for this and HIP events order the
hand-offs.  It gives the same weights bit for bit and measured no faster on one MI355X.

Beyond the GraphSAGE path the same driver runs GCN layers (`model="gcn"`), the validation pass and
training protocol of the paper (`evaluate`, `fit`), and a feature store in pinned host memory with or
without the software-managed cache in front of it (`host_features`, `cache_rows`).
"""
from __future__ import annotations

import ctypes as C
from typing import List, Optional

import numpy as np

from . import binding as B
from . import synth


class Trainer:
    def __init__(self, workload: synth.Workload, group_size: int = 16, lr: float = 0.01,
                 weight_decay: float = 5e-4, seed: int = 0, device: str = "cuda", weights=None,
                 relabel_input: bool = False, edge_classes: bool = True, host_features: bool = False,
                 cache_rows: int = 0, cache_ways: int = 16, model: str = "sage", gat_heads: int = 4, order_rows="auto",
                 fused_layer_bwd: bool = True, fused_top_loss: bool = True):
        import torch
        self.torch = torch
        self.fused_layer_bwd = fused_layer_bwd
        self.w = workload
        cfg = workload.cfg
        self.cfg = cfg
        self.L = len(cfg.fanouts)
        self.B = cfg.batch_size
        self.G = group_size
        self.lr, self.wd, self.seed = lr, weight_decay, seed
        assert model in ("sage", "gcn", "gat")
        self.model = model
        self.n_op = 2 if model == "sage" else 1
        assert model == "sage" or not (host_features or cache_rows), "the GCN and GAT paths read the resident table"
        # The layer-0 gather reads the feature table through per-edge global ids and the features take no
        # gradient, so nothing in a training step needs the input frontier de-duplicated or relabelled
        # (relabel_input=True asks for it anyway, e.g. to count the distinct input nodes of a batch).
        # A feature store on the host (and the cache in front of it) works on the batch's distinct input nodes,
        # so those set-ups do need the input frontier de-duplicated.
        # Graph attention projects every distinct input node once and needs the gradient per source row of every
        # layer, the first included: de-duplicated input frontier and a transposed input block.
        relabel_input = relabel_input or host_features or cache_rows > 0 or model == "gat"
        self.sample_flags = 0 if relabel_input else B.CR_SAMPLE_INPUT_GLOBAL_IDS
        if model == "gat":
            self.sample_flags |= B.CR_SAMPLE_TRANSPOSE_INPUT
        # the workload's arrays are numpy (synth.Workload: uploaded here) or already device tensors (synth_gpu.DeviceWorkload)
        def up(a, dtype):
            if isinstance(a, torch.Tensor):
                return a.to(device=device, dtype=dtype).contiguous()
            return torch.from_numpy(np.ascontiguousarray(a)).to(device=device, dtype=dtype)
        self.indptr = up(workload.indptr, torch.int64)
        self.indices = up(workload.indices, torch.int32)
        self.comm = up(workload.comm, torch.int32)
        self.labels = up(workload.labels, torch.int32)
        self.train_ids = up(workload.train_ids, torch.int32)
        feats = workload.features
        on_device = isinstance(feats, torch.Tensor)
        is_bf16 = feats.dtype == (torch.int16 if on_device else np.uint16)
        self.feat_dtype = B.CR_BF16 if is_bf16 else B.CR_F32
        self.ld_table = int(feats.shape[1])
        self.row_bytes = self.ld_table * (2 if is_bf16 else 4)
        self.host_store = None
        if host_features:      # the table stays in pinned host memory; kernels read it over the host link
            assert not on_device, "a host-resident store takes a numpy workload"
            self.host_store = B.HostBuffer(feats.shape, feats.dtype)
            self.host_store.array[:] = feats
            self.table = None
            self.table_ptr = self.host_store.device_ptr
        else:
            if on_device:
                self.table = feats.to(device).contiguous()
            else:
                self.table = torch.from_numpy(np.ascontiguousarray(feats.view(np.int16) if is_bf16 else feats)).to(device)
            self.table_ptr = C.c_void_p(self.table.data_ptr())
        self.graph = B.make_graph(self.indptr, self.indices, self.comm, cfg.n_comm)
        # context of this trainer's calls: kernels record data-dependent overflows in its device status words
        self.ctx = B.Context(device=torch.device(device).index or 0, status=torch.zeros(B.CR_CTX_STATUS_WORDS, dtype=torch.int64, device=device))
        self.ctx.make_current()
        if edge_classes:     # static per graph: one bit per adjacency entry, read by the biased selection
            self.edge_bits = B.cr_graph_edge_classes(self.graph)
            self.graph.edge_intra = self.edge_bits.data_ptr()
        self.n_nodes = cfg.n_nodes
        self.n_train = int(self.train_ids.numel())
        self.n_batches = -(-self.n_train // self.B)

        # parameters
        if model == "gat":
            # weights: per layer (W [F_in, heads*D], a_l, a_r, bias); `gat_heads` heads on hidden layers, one on the last
            weights = weights if weights is not None else synth.init_gat_weights(cfg, seed, gat_heads)
            assert cfg.hidden % 64 == 0 and cfg.hidden % gat_heads == 0, "GAT path: hidden width must be a multiple of 64 and of the head count"
            self.layers = [B.SageLayer(W, np.zeros(W.shape[1], dtype=np.float32), device, 1) for (W, _, _, _) in weights]
            for layer in self.layers:
                layer.drop_bias()
            self.gat = [B.GatParams(a_l, a_r, b, gat_heads if l < self.L - 1 else 1, self.layers[l].N_pad, 0.2, device)
                        for l, (_, a_l, a_r, b) in enumerate(weights)]
        else:
            weights = weights if weights is not None else synth.init_weights(cfg, seed, self.n_op)
            self.layers: List[B.SageLayer] = [B.SageLayer(W, b, device, self.n_op) for (W, b) in weights]
        for layer in self.layers:
            layer.refresh()

        # step 1
        self.perm = torch.zeros(max(1, self.n_train), dtype=torch.int32, device=device)
        self.ws_batches = torch.empty(B.cr_build_batches_workspace_bytes(self.n_train, cfg.n_comm), dtype=torch.uint8, device=device)

        # step 2: block storage for one group of batches
        scfg = B.make_sample_cfg(cfg.fanouts, 0.5, seed, 0)
        # Processing order of the input-side block's destination rows (grouped by community): the layer-0 gather then
        # works on rows that share feature rows next to each other.  It pays when a batch holds many rows per community
        # (measured: -13 % gather time on the arxiv-like graph, -11 % on the reddit-like one, nothing on the
        # products-like one with its 5000 communities), so "auto" asks for it from 32 rows per community on.
        cap_dst0 = B.cr_block_capacities(scfg, self.n_nodes, self.B)[0][0]
        group_possible = model in ("sage", "gcn") and not (host_features or cache_rows > 0)
        if order_rows == "auto":
            # per batch the order needs enough rows per community to pay; over a whole group (below) it always did
            order_rows = group_possible or (model != "gat" and cap_dst0 >= 32 * cfg.n_comm)
        self.order_rows = bool(order_rows) and model != "gat"
        if self.order_rows:
            self.sample_flags |= B.CR_SAMPLE_ROW_ORDER
        # GraphSAGE and GCN on a resident table go one step further: the layer-0 aggregation needs neither weights nor
        # gradients, so it runs once per sampled group, over the rows of all its batches in community order
        # (cr_gather_aggregate_fwd_group): a feature row is then fetched once for the group, not once per batch
        # (measured per batch: arxiv-like 31.8 -> 18.2 us, products-like 77.5 -> 55.6 us, papers-like 46.8 -> 30.4 us).
        # Results are the same bit for bit.
        self.group_gather = self.order_rows and group_possible
        self.block_slots = [B.alloc_block_sets(scfg, self.n_nodes, self.B, self.G, device, transpose_input=model == "gat",
                                               order_input=self.order_rows and not self.group_gather,
                                               group_order_input=self.group_gather) for _ in range(2)]
        self.blocks = self.block_slots[0]
        scfg.flags = self.sample_flags
        self.ws_sample = torch.empty(B.cr_sample_blocks_workspace_bytes(scfg, self.n_nodes, self.B, self.G), dtype=torch.uint8, device=device)

        # activations / gradients, sized by the per-batch capacities
        f32 = lambda r, c: torch.zeros((r, c), dtype=torch.float32, device=device)
        b16 = lambda r, c: torch.zeros((r, c), dtype=torch.int16, device=device)
        self.self0_bufs = [b16(self.blocks[0].cap_dst, self.layers[0].F_pad) for _ in range(2)]
        self.agg0_bufs = [b16(self.blocks[0].cap_dst, self.layers[0].F_pad) for _ in range(2)]
        self.self0 = self.self0_bufs[0]
        self.self0_all = self.agg0_all = None
        if self.group_gather:     # [slot][batch][row][column]: layer-0 operands of a whole group
            b16g = lambda: torch.zeros((self.G, self.blocks[0].cap_dst, self.layers[0].F_pad), dtype=torch.int16, device=device)
            self.agg0_all = [b16g(), b16g()]
            self.self0_all = [b16g(), b16g()] if model == "sage" else [None, None]      # (GCN's sum includes the destination's own row)
        self.group_gathered = [False, False]     # per block slot: the current group's layer-0 operands are in *_all
        self.agg = [b16(self.blocks[l].cap_dst, self.layers[l].F_pad if l == 0 else self.layers[l - 1].N_pad) for l in range(self.L)]
        # hidden activations are kept in bf16 only (next layer's self operand, aggregation input and
        # ReLU mask); the logits of the last layer stay in float for the loss
        self.out = [f32(self.blocks[l].cap_dst, self.layers[l].N_pad) if l == self.L - 1 else None for l in range(self.L)]
        self.out_b = [b16(self.blocks[l].cap_dst, self.layers[l].N_pad) if l < self.L - 1 else None for l in range(self.L)]
        self.dz = [b16(self.blocks[l].cap_dst, self.layers[l].N_pad) for l in range(self.L)]
        # input gradients [d_self | d_agg] of the layers above the first, kept in bf16: the scatter back over the
        # block reads them once per edge, so their width is what that kernel's traffic is made of
        self.d_in = [b16(self.blocks[l].cap_dst, self.n_op * self.layers[l].F_pad) if l >= 1 else None for l in range(self.L)]
        if model == "gcn":     # per-node normalisation of the graph, per-block normalisation scratch of every layer
            self.gcn_norm = B.cr_graph_gcn_norm(self.graph)
            self.blk_norm = [torch.zeros(self.blocks[l].cap_src + 2 * self.blocks[l].cap_dst, dtype=torch.float32, device=device)
                             for l in range(self.L)]
        if model == "gat":     # the dense part runs over the source rows of every block
            lay, blk = self.layers, self.blocks
            self.x0 = b16(blk[0].cap_src, lay[0].F_pad)                                   # bf16 rows of the distinct input nodes
            self.gat_z = [b16(blk[l].cap_src, lay[l].N_pad) for l in range(self.L)]       # projected source rows
            self.gat_dz = [b16(blk[l].cap_src, lay[l].N_pad) for l in range(self.L)]      # their gradients
            self.gat_el = [f32(blk[l].cap_src, self.gat[l].heads) for l in range(self.L)]
            self.gat_er = [f32(blk[l].cap_src, self.gat[l].heads) for l in range(self.L)]
            self.gat_stat = [f32(blk[l].cap_dst, 4 * self.gat[l].heads) for l in range(self.L)]
            self.gat_din = [b16(blk[l].cap_src, lay[l].F_pad) if l >= 1 else None for l in range(self.L)]   # dL/d (output of layer l-1)
            self.ws_gat = [torch.empty(B.cr_gat_attention_bwd_workspace_bytes(blk[l].cap_dst, lay[l].N_pad, self.gat[l].heads),
                                       dtype=torch.uint8, device=device) for l in range(self.L)]
        rows_of = lambda l: self.blocks[l].cap_src if model == "gat" else self.blocks[l].cap_dst
        self.ws_bwd = [torch.empty(B.cr_sage_linear_bwd_workspace_bytes(self.layers[l].F_in, self.layers[l].F_out, rows_of(l)),
                                   dtype=torch.uint8, device=device) for l in range(self.L)]
        self.loss = torch.zeros(1, dtype=torch.float32, device=device)
        self.row_loss = torch.zeros(self.B, dtype=torch.float32, device=device)
        self.xent_scratch = torch.zeros(B.CR_XENT_SCRATCH_BYTES, dtype=torch.uint8, device=device)
        self.fused_top_loss = fused_top_loss and model in ("sage", "gcn")
        self.agg[0] = self.agg0_bufs[0]
        self.gather0_events = []          # (start, stop) pairs around the layer-0 gather when timing is on
        self.time_gather0 = False
        # software-managed cache of feature rows (set-associative LRU) and / or a staging area for the distinct
        # input rows of one batch when the store is on the host
        self.cache, self.cache_stamp, self.staged = None, 0, None
        cap_src0 = self.blocks[0].cap_src
        if cache_rows > 0:
            assert self.row_bytes % 16 == 0
            self.cache = B.FeatureCache(max(1, cache_rows // cache_ways), cache_ways, self.row_bytes, cap_src0, device)
        elif host_features:
            self.staged = torch.zeros((cap_src0, self.row_bytes), dtype=torch.uint8, device=device)
        self.stream_sample = torch.cuda.Stream(device=device)
        self.stream_gather = torch.cuda.Stream(device=device)
        self.stream_weights = torch.cuda.Stream(device=device)
        self.weights_on_side_stream = False     # set by run_epoch(weights_on_side_stream=True)
        self.order_now = self.order_rows
        self.ev_weights = [None] * self.L        # event: layer l's weights are updated and its operands are free again

    # ------------------------------------------------------------------ step 1
    def build_batches(self, policy: int, mix_count: int, epoch: int) -> int:
        # every root policy gains: random and community-mixing batches from the locality of the order, batches that
        # follow the community order already (NORAND) from gathering a whole group in one launch
        self.order_now = self.order_rows
        return B.cr_build_batches(policy, mix_count, self.B, self.seed, epoch, self.train_ids, self.comm, self.cfg.n_comm,
                                  self.ws_batches, self.perm)

    # ------------------------------------------------------------------ step 2
    def sample_group(self, first_batch: int, n_batches: int, p_intra: float, epoch: int, flags: Optional[int] = None, slot: int = 0):
        """Samples mini-batches first_batch .. first_batch+n_batches-1 of the current permutation into
        block storage `slot` (on the current stream)."""
        assert 1 <= n_batches <= self.G
        self.ctx.make_current()
        self.blocks = self.block_slots[slot]
        flags = self.sample_flags if flags is None else flags
        flags = self._apply_row_order(self.blocks[0], flags)
        scfg = B.make_sample_cfg(self.cfg.fanouts, p_intra, self.seed, epoch, first_batch, flags)
        start = first_batch * self.B
        n_roots = min(self.n_train, start + n_batches * self.B) - start
        roots = C.c_void_p(self.perm.data_ptr() + 4 * start)
        layers = self.blocks
        if n_batches != self.G:           # a short last group: same storage, fewer batches
            layers = [_view_block_set(b, n_batches) for b in self.blocks]
        arr = (B.cr_block_set * self.L)(*[b.c for b in layers])
        B._check(B.lib().cr_sample_blocks(C.byref(self.graph), C.byref(scfg), roots, n_roots, self.B, n_batches,
                                          B._ptr(self.ws_sample), self.ws_sample.numel(), arr, B._stream()))
        self._gather_group(slot, layers[0], n_batches)

    def _apply_row_order(self, blk0, flags: int) -> int:
        """Switches the input-side block's row order (per batch or over the group) on or off for the group about to be
        sampled (the gathers read the same descriptor, so both always agree); returns the sampling flags to use."""
        if blk0.row_order is None and blk0.group_order is None:
            return flags & ~B.CR_SAMPLE_ROW_ORDER
        on = bool(self.order_now) and bool(flags & B.CR_SAMPLE_ROW_ORDER)
        if blk0.row_order is not None:
            blk0.c.row_order = blk0.row_order.data_ptr() if on else None
        if blk0.group_order is not None:
            blk0.c.group_order = blk0.group_order.data_ptr() if on else None
        return (flags | B.CR_SAMPLE_ROW_ORDER) if on else (flags & ~B.CR_SAMPLE_ROW_ORDER)

    def _gather_group(self, slot: int, blk0, n_batches: int):
        """Layer-0 gather + aggregation of every batch of the group just sampled into block slot `slot`, in one launch
        (only when the group carries its order; otherwise the batches gather one by one in forward_batch)."""
        self.group_gathered[slot] = bool(self.group_gather and blk0.c.group_order)
        if not self.group_gathered[slot]:
            return
        if self.time_gather0:
            ev0, ev1 = self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)
            ev0.record()
        if self.model == "gcn":
            B.cr_gcn_aggregate_fwd_group(blk0, self.gcn_norm, self.table_ptr, self.feat_dtype, self.ld_table, self.cfg.n_feat,
                                         self.agg0_all[slot], self.block_slots[slot][0].cap_dst, self.layers[0].F_pad)
        else:
            B.cr_gather_aggregate_fwd_group(blk0, self.table_ptr, self.feat_dtype, self.ld_table, self.cfg.n_feat, self.agg0_all[slot],
                                            self.self0_all[slot], self.block_slots[slot][0].cap_dst, self.layers[0].F_pad)
        if self.time_gather0:
            ev1.record()
            self.gather0_events.append((ev0, ev1))

    # ------------------------------------------------------------------ training on one sub-graph
    def gather_layer0(self, g: int, slot: int = 0, buf: int = 0):
        """Feature gather + mean aggregation of mini-batch g of block slot `slot` into operand buffer `buf`."""
        blk, lay = self.block_slots[slot][0], self.layers[0]
        if self.group_gathered[slot]:          # done for the whole group right after sampling
            return
        if self.time_gather0:
            ev0, ev1 = self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)
            ev0.record()
        if self.cache is not None:
            # look the batch's distinct input nodes up, bring the missing rows in, then gather from the cache's rows
            # through the slots (a one-batch view of the block whose frontier array is the slot array)
            self.cache.fetch(self.table_ptr, self.row_bytes, blk.src_ids_ptr(g), blk.hdr_ptr(g), B.CR_HDR_N_SRC, self.cache_stamp)
            self.cache_stamp += 1
            view = _one_batch_view(blk, g, self.cache.slot_out)
            B.cr_gather_aggregate_fwd(view, 0, self.cache.rows, self.feat_dtype, self.ld_table, self.cfg.n_feat, True,
                                      None, self.agg0_bufs[buf], self.self0_bufs[buf], lay.F_pad)
        elif self.staged is not None:
            # no cache: every distinct input row crosses the host link once, then a dense gather
            B.cr_stage_rows(self.table_ptr, self.row_bytes, blk.src_ids_ptr(g), blk.hdr_ptr(g), B.CR_HDR_N_SRC, blk.cap_src,
                            self.staged, self.row_bytes)
            B.cr_gather_aggregate_fwd(blk, g, self.staged, self.feat_dtype, self.ld_table, self.cfg.n_feat, False,
                                      None, self.agg0_bufs[buf], self.self0_bufs[buf], lay.F_pad)
        else:
            B.cr_gather_aggregate_fwd(blk, g, self.table_ptr, self.feat_dtype, self.ld_table, self.cfg.n_feat, True,
                                      None, self.agg0_bufs[buf], self.self0_bufs[buf], lay.F_pad)
        if self.time_gather0:
            ev1.record()
            self.gather0_events.append((ev0, ev1))

    def forward_batch(self, g: int, slot: Optional[int] = None, buf: int = 0, gather0: bool = True, with_loss: bool = False):
        """Forward pass of mini-batch g of a sampled group (current stream); leaves the logits in self.out[L-1].
        with_loss: also the loss on the roots and its gradient (self.loss, self.dz[L-1]); returns whether they were taken."""
        if slot is not None:
            self.blocks = self.block_slots[slot]
        else:
            slot = self.block_slots.index(self.blocks)
        if self.group_gathered[slot]:
            self.agg[0] = self.agg0_all[slot][g]
            if self.self0_all[slot] is not None:
                self.self0 = self.self0_all[slot][g]
        else:
            self.self0, self.agg[0] = self.self0_bufs[buf], self.agg0_bufs[buf]
        L, blocks, layers = self.L, self.blocks, self.layers
        if self.model == "gcn":
            return self._forward_batch_gcn(g, with_loss, self.group_gathered[slot])
        if self.model == "gat":
            return self._forward_batch_gat(g)
        for l in range(L):
            blk, lay = blocks[l], layers[l]
            if l == 0:
                if gather0:
                    self.gather_layer0(g, slot, buf)
                # weight updates of the previous step that ran on the side stream: every layer's operands
                # (hidden activations, aggregates, dZ) are overwritten from here on
                self.wait_weights()
                h_self, ld_in = self.self0, lay.F_pad
            else:
                prev = layers[l - 1]
                B.cr_gather_aggregate_fwd(blk, g, self.out_b[l - 1], B.CR_BF16, prev.N_pad, prev.F_out, False,
                                          None, self.agg[l], None, prev.N_pad)
                h_self, ld_in = self.out_b[l - 1], prev.N_pad
            if with_loss and l == L - 1 and self.fused_top_loss:
                # the layer next to the loss and the loss itself in one launch
                B.cr_sage_linear_fwd_xent(lay, blk.hdr_ptr(g), blk.cap_dst, h_self, self.agg[l], ld_in, self.out[l], self.cfg.n_classes,
                                          self.labels, blk.src_ids_ptr(g), self.loss, self.row_loss, self.dz[l], self.xent_scratch)
                return True
            B.cr_sage_linear_fwd(lay, blk.hdr_ptr(g), blk.cap_dst, h_self, self.agg[l], ld_in, l < L - 1,
                                 self.out[l], self.out_b[l])
        return False

    def _forward_batch_gcn(self, g: int, with_loss: bool = False, gathered0: bool = False):
        """GCN layers: normalised aggregation over the block (the destination's own row included), one-operand layer."""
        L, blocks, layers = self.L, self.blocks, self.layers
        self.wait_weights()
        for l in range(L):
            blk, lay = blocks[l], layers[l]
            if l == 0 and gathered0:          # aggregated for the whole group right after sampling (self.agg[0])
                B.cr_sage_linear_fwd(lay, blk.hdr_ptr(g), blk.cap_dst, None, self.agg[0], lay.F_pad, l < L - 1, self.out[l], self.out_b[l])
                continue
            B.cr_gcn_block_norm(blk, g, self.gcn_norm, self.blk_norm[l])
            if l == 0:
                if self.time_gather0:
                    ev0, ev1 = self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)
                    ev0.record()
                B.cr_gcn_aggregate_fwd(blk, g, self.gcn_norm, self.blk_norm[0], self.table_ptr, self.feat_dtype, self.ld_table,
                                       self.cfg.n_feat, True, None, self.agg[0], lay.F_pad)
                if self.time_gather0:
                    ev1.record()
                    self.gather0_events.append((ev0, ev1))
                ld_in = lay.F_pad
            else:
                prev = layers[l - 1]
                B.cr_gcn_aggregate_fwd(blk, g, self.gcn_norm, self.blk_norm[l], self.out_b[l - 1], B.CR_BF16, prev.N_pad, prev.F_out,
                                       False, None, self.agg[l], prev.N_pad)
                ld_in = prev.N_pad
            if with_loss and l == L - 1 and self.fused_top_loss:
                B.cr_sage_linear_fwd_xent(lay, blk.hdr_ptr(g), blk.cap_dst, None, self.agg[l], ld_in, self.out[l], self.cfg.n_classes,
                                          self.labels, blk.src_ids_ptr(g), self.loss, self.row_loss, self.dz[l], self.xent_scratch)
                return True
            B.cr_sage_linear_fwd(lay, blk.hdr_ptr(g), blk.cap_dst, None, self.agg[l], ld_in, l < L - 1, self.out[l], self.out_b[l])
        return False

    def _backward_batch_gcn(self, g: int, dW_out, db_out):
        L, blocks, layers = self.L, self.blocks, self.layers
        for l in range(L - 1, -1, -1):
            blk, lay = blocks[l], layers[l]
            ld_in = lay.F_pad if l == 0 else layers[l - 1].N_pad
            grads = (None if dW_out is None else dW_out[l], None if db_out is None else db_out[l])
            B.cr_sage_linear_bwd(lay, blk.hdr_ptr(g), blk.cap_dst, None, self.agg[l], ld_in, self.dz[l], self.lr, self.wd,
                                 None, None, self.ws_bwd[l], *grads, d_in_bf16=self.d_in[l])
            if l >= 1:
                prev = layers[l - 1]
                B.cr_gcn_aggregate_bwd(blk, g, self.blk_norm[l], self.d_in[l], lay.F_pad, lay.F_in, self.out_b[l - 1], prev.N_pad,
                                       None, self.dz[l - 1], prev.N_pad, relu_dtype=B.CR_BF16, in_dtype=B.CR_BF16)

    # graph attention: project the source rows, then attend over the block (the dense layer runs on n_src rows)
    @staticmethod
    def _src_rows_hdr(blk, g):
        """Address of the header word that holds the block's number of source rows (the dense calls read one word)."""
        return C.c_void_p(blk.hdr_ptr(g).value + 4 * B.CR_HDR_N_SRC)

    def _forward_batch_gat(self, g: int):
        L, blocks, layers = self.L, self.blocks, self.layers
        self.wait_weights()
        for l in range(L):
            blk, lay, par = blocks[l], layers[l], self.gat[l]
            if l == 0:
                if self.time_gather0:
                    ev0, ev1 = self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)
                    ev0.record()
                B.cr_gather_rows_bf16(self.table_ptr, self.feat_dtype, self.ld_table, self.cfg.n_feat, blk.src_ids_ptr(g), blk.hdr_ptr(g),
                                      B.CR_HDR_N_SRC, blk.cap_src, self.x0, lay.F_pad)
                if self.time_gather0:
                    ev1.record()
                    self.gather0_events.append((ev0, ev1))
                x, ld_in = self.x0, lay.F_pad
            else:
                x, ld_in = self.out_b[l - 1], layers[l - 1].N_pad
            B.cr_sage_linear_fwd(lay, self._src_rows_hdr(blk, g), blk.cap_src, None, x, ld_in, False, None, self.gat_z[l])
            B.cr_gat_attention_fwd(blk, g, par, self.gat_z[l], lay.N_pad, l < L - 1, self.gat_el[l], self.gat_er[l], self.gat_stat[l],
                                   self.out[l], self.out_b[l])

    def _backward_batch_gat(self, g: int, dW_out, d_attn_out):
        L, blocks, layers = self.L, self.blocks, self.layers
        for l in range(L - 1, -1, -1):
            blk, lay, par = blocks[l], layers[l], self.gat[l]
            if l == L - 1:
                d_out, ld_dout = self.dz[l], lay.N_pad
            else:
                d_out, ld_dout = self.gat_din[l + 1], layers[l + 1].F_pad
            B.cr_gat_attention_bwd(blk, g, par, self.gat_z[l], lay.N_pad, self.gat_el[l], self.gat_stat[l], d_out, ld_dout,
                                   self.out_b[l] if l < L - 1 else None, self.lr, self.wd, self.gat_dz[l], self.ws_gat[l],
                                   None if d_attn_out is None else d_attn_out[l])
            x, ld_in = (self.x0, lay.F_pad) if l == 0 else (self.out_b[l - 1], layers[l - 1].N_pad)
            B.cr_sage_linear_bwd(lay, self._src_rows_hdr(blk, g), blk.cap_src, None, x, ld_in, self.gat_dz[l], self.lr, self.wd,
                                 None, None, self.ws_bwd[l], None if dW_out is None else dW_out[l], None, d_in_bf16=self.gat_din[l])

    def train_batch(self, g: int, dW_out=None, db_out=None, slot: Optional[int] = None, buf: int = 0, gather0: bool = True,
                    d_attn_out=None):
        """Forward, loss, backward and SGD for mini-batch g of a sampled group (current stream)."""
        have_loss = self.forward_batch(g, slot, buf, gather0, with_loss=True)
        L, blocks, layers = self.L, self.blocks, self.layers
        # loss on the roots
        top = blocks[L - 1]
        if not have_loss:
            B.cr_softmax_xent(top.hdr_ptr(g), top.cap_dst, self.out[L - 1], layers[L - 1].N_pad, self.cfg.n_classes,
                              self.labels, top.src_ids_ptr(g), self.loss, self.row_loss, None, self.dz[L - 1])
        # backward + SGD
        if self.model == "gcn":
            return self._backward_batch_gcn(g, dW_out, db_out)
        if self.model == "gat":
            return self._backward_batch_gat(g, dW_out, d_attn_out)
        side = self.stream_weights if self.weights_on_side_stream else None
        for l in range(L - 1, -1, -1):
            blk, lay = blocks[l], layers[l]
            if l == 0:
                h_self, ld_in = self.self0, lay.F_pad
            else:
                h_self, ld_in = self.out_b[l - 1], layers[l - 1].N_pad
            grads = (None if dW_out is None else dW_out[l], None if db_out is None else db_out[l])
            if side is None and l >= 1 and self.fused_layer_bwd:
                # the whole layer in two launches: (weight gradient | input gradient), (aggregation backward | SGD step)
                prev = layers[l - 1]
                B.cr_sage_layer_bwd(lay, blk, g, h_self, self.agg[l], ld_in, self.dz[l], self.lr, self.wd, self.d_in[l],
                                    self.out_b[l - 1], prev.N_pad, self.dz[l - 1], prev.N_pad, self.ws_bwd[l], *grads)
                continue
            if side is None:
                B.cr_sage_linear_bwd(lay, blk.hdr_ptr(g), blk.cap_dst, h_self, self.agg[l], ld_in, self.dz[l], self.lr, self.wd,
                                     None, None, self.ws_bwd[l], *grads, d_in_bf16=self.d_in[l])
            else:
                # the input gradients stay on the critical path; the weight gradient and the SGD step of this
                # layer go to the side stream, after the input-gradient product has read the old weights
                if l >= 1:
                    B.cr_sage_linear_bwd_input(lay, blk.hdr_ptr(g), blk.cap_dst, self.dz[l], None, None, d_in_bf16=self.d_in[l])
                ready = self.torch.cuda.Event()
                ready.record()
                with self.torch.cuda.stream(side):
                    side.wait_event(ready)
                    B.cr_sage_linear_bwd(lay, blk.hdr_ptr(g), blk.cap_dst, h_self, self.agg[l], ld_in, self.dz[l], self.lr, self.wd,
                                         None, None, self.ws_bwd[l], *grads)
                    self.ev_weights[l] = self.torch.cuda.Event()
                    self.ev_weights[l].record(side)
            if l >= 1:
                prev = layers[l - 1]
                d_agg = C.c_void_p(self.d_in[l].data_ptr() + 2 * lay.F_pad)      # second half of every row
                B.cr_gather_aggregate_bwd(blk, g, d_agg, self.d_in[l], 2 * lay.F_pad, lay.F_in, self.out_b[l - 1],
                                          prev.N_pad, None, self.dz[l - 1], prev.N_pad, relu_dtype=B.CR_BF16, in_dtype=B.CR_BF16)

    def wait_weights(self, layers=None):
        """Makes the current stream wait for the side-stream weight updates of the given layers (all by default)."""
        cur = self.torch.cuda.current_stream()
        for l in (range(self.L) if layers is None else layers):
            if self.ev_weights[l] is not None:
                cur.wait_event(self.ev_weights[l])
                self.ev_weights[l] = None

    # ------------------------------------------------------------------ one epoch
    def run_epoch_serial(self, policy: int, mix_count: int, p_intra: float, epoch: int, max_batches: Optional[int] = None):
        """Everything on the current stream, one call after the other."""
        nb = self.build_batches(policy, mix_count, epoch)
        if max_batches is not None:
            nb = min(nb, max_batches)
        done = 0
        while done < nb:
            n = min(self.G, nb - done)
            self.sample_group(done, n, p_intra, epoch)
            for g in range(n):
                self.train_batch(g)
            done += n
        return nb

    def run_epoch(self, policy: int, mix_count: int, p_intra: float, epoch: int, max_batches: Optional[int] = None,
                  on_group=None, gather_on_side_stream: bool = False, weights_on_side_stream: bool = False):
        """Overlapped schedule: root partitioning and sampling of the next group of mini-batches run on a
        side stream while the current group trains; with gather_on_side_stream the layer-0 gather of the
        next mini-batch runs on a second side stream as well; with weights_on_side_stream every layer's
        weight gradient + SGD step leaves the critical path of the backward pass for a third one.  Same
        calls, same arguments, same results as run_epoch_serial.  on_group(n, slot), if given, is called
        after a group's work is enqueued."""
        torch = self.torch
        self.weights_on_side_stream = weights_on_side_stream
        main = torch.cuda.current_stream()
        ss = self.stream_sample
        sg = self.stream_gather if gather_on_side_stream else main
        ev = lambda: torch.cuda.Event()
        ss.wait_stream(main)
        sg.wait_stream(main)
        with torch.cuda.stream(ss):
            nb = self.build_batches(policy, mix_count, epoch)
        if max_batches is not None:
            nb = min(nb, max_batches)
        groups = [(first, min(self.G, nb - first)) for first in range(0, nb, self.G)]
        sampled = [None, None]           # event: block slot holds a freshly sampled group
        slot_free = [None, None]         # event: training and gathering no longer read the slot
        gathered = [None, None]          # event: layer-0 operand buffer holds a batch
        buf_free = [None, None]          # event: training no longer reads the operand buffer

        def enqueue_sample(k):
            first, n = groups[k]
            slot = k % 2
            with torch.cuda.stream(ss):
                if slot_free[slot] is not None:
                    ss.wait_event(slot_free[slot])
                self.sample_group(first, n, p_intra, epoch, slot=slot)
                sampled[slot] = ev()
                sampled[slot].record(ss)

        if groups:
            enqueue_sample(0)
        step = 0
        for k, (first, n) in enumerate(groups):
            slot = k % 2
            if k + 1 < len(groups):
                enqueue_sample(k + 1)
            with torch.cuda.stream(sg):
                sg.wait_event(sampled[slot])
            main.wait_event(sampled[slot])
            for g in range(n):
                buf = step % 2
                with torch.cuda.stream(sg):
                    for e in buf_free[buf] or ():
                        sg.wait_event(e)
                    self.gather_layer0(g, slot, buf)
                    gathered[buf] = ev()
                    gathered[buf].record(sg)
                main.wait_event(gathered[buf])
                self.train_batch(g, slot=slot, buf=buf, gather0=False)
                e = ev()
                e.record(main)
                buf_free[buf] = [e] + ([self.ev_weights[0]] if self.ev_weights[0] is not None else [])
                step += 1
            if on_group is not None:
                on_group(n, slot)
            self.wait_weights()             # side-stream weight updates still read this slot's headers
            done = ev()
            done.record(main)               # training of the group is enqueued up to here ...
            with torch.cuda.stream(sg):
                fin = ev()
                fin.record(sg)              # ... and so is its gathering
            with torch.cuda.stream(ss):
                ss.wait_event(fin)
            slot_free[slot] = done
        main.wait_stream(ss)
        main.wait_stream(sg)
        self.wait_weights()
        self.weights_on_side_stream = False
        return nb

    # ------------------------------------------------------------------ validation pass and training protocol
    def evaluate(self, node_ids, epoch: int = 0, p_intra: float = 0.5):
        """Forward-only pass over `node_ids` (device int32 tensor) in mini-batches of the training batch size,
        neighbours sampled uniformly with the same fanouts.  Returns (mean loss, accuracy).  Validation batches
        are numbered after the epoch's training batches, so they draw their own random streams."""
        torch = self.torch
        n = int(node_ids.numel())
        if n == 0:
            return float("nan"), float("nan")
        nb = -(-n // self.B)
        batch_loss = torch.zeros(1, dtype=torch.float32, device=node_ids.device)
        mean_loss = torch.zeros(3, dtype=torch.float64, device=node_ids.device)     # sum of loss x rows, rows, mean over all rows
        correct = torch.zeros(1, dtype=torch.int32, device=node_ids.device)
        top_l = self.L - 1
        for first in range(0, nb, self.G):
            cnt = min(self.G, nb - first)
            scfg = B.make_sample_cfg(self.cfg.fanouts, p_intra, self.seed, epoch, self.n_batches + first,
                                     self._apply_row_order(self.block_slots[0][0], self.sample_flags))
            start = first * self.B
            n_roots = min(n, start + cnt * self.B) - start
            layers = self.block_slots[0] if cnt == self.G else [_view_block_set(b, cnt) for b in self.block_slots[0]]
            arr = (B.cr_block_set * self.L)(*[b.c for b in layers])
            B._check(B.lib().cr_sample_blocks(C.byref(self.graph), C.byref(scfg), C.c_void_p(node_ids.data_ptr() + 4 * start), n_roots,
                                              self.B, cnt, B._ptr(self.ws_sample), self.ws_sample.numel(), arr, B._stream()))
            self._gather_group(0, layers[0], cnt)
            for g in range(cnt):
                self.forward_batch(g, slot=0, buf=0)
                top = self.block_slots[0][top_l]
                B.cr_softmax_xent(top.hdr_ptr(g), top.cap_dst, self.out[top_l], self.layers[top_l].N_pad, self.cfg.n_classes,
                                  self.labels, top.src_ids_ptr(g), batch_loss, self.row_loss)
                B.cr_mean_accumulate(top.hdr_ptr(g), top.cap_dst, batch_loss, mean_loss)
                B.cr_count_correct(top.hdr_ptr(g), top.cap_dst, self.out[top_l], self.layers[top_l].N_pad, self.cfg.n_classes,
                                   self.labels, top.src_ids_ptr(g), correct)
        return float(mean_loss.cpu()[2]), float(int(correct.cpu()[0]) / n)

    def fit(self, policy: int, mix_count: int, p_intra: float, val_ids, max_epochs: int = 100, patience: int = 6,
            lr_patience: int = 3, lr_factor: float = 0.1, first_epoch: int = 0):
        """The paper's protocol: up to max_epochs epochs, early stop when the validation loss has not improved for
        `patience` epochs, learning rate cut after `lr_patience` epochs on a plateau.  Returns a protocol.History."""
        from . import protocol
        torch = self.torch
        sched = protocol.PlateauScheduler(self.lr, lr_patience, lr_factor)
        stop = protocol.EarlyStopping(patience)
        hist = protocol.History()
        for e in range(first_epoch, first_epoch + max_epochs):
            torch.cuda.synchronize()
            t0 = _now()
            self.run_epoch_serial(policy, mix_count, p_intra, e)
            torch.cuda.synchronize()
            hist.epoch_ms.append((_now() - t0) * 1e3)
            hist.train_loss.append(float(self.loss.cpu()[0]))
            vl, va = self.evaluate(val_ids, e)
            hist.val_loss.append(vl)
            hist.val_acc.append(va)
            hist.lr.append(self.lr)
            self.check_async_status()
            self.lr = sched.step(vl)
            if stop.step(vl, e):
                hist.stopped_early = True
                break
        return hist

    def check_async_status(self):
        """Polls what the kernels recorded since the last poll (one small read-back; once per epoch in fit): raises if a
        sampled block did not fit its arrays."""
        st, required = self.ctx.poll_error()
        if st != B.CR_OK:
            raise B.CrError(st, f"{B.lib().cr_last_error().decode()} (required: {required})")

    def input_node_stats(self, policy: int, mix_count: int, p_intra: float, epoch: int, max_groups: int = 4):
        """Distinct input nodes and gathered rows per batch over the first groups of an epoch (sampled once more
        with the input frontier de-duplicated; bookkeeping, not part of a training step).  Returns
        (mean distinct input nodes, distinct / gathered rows)."""
        nb = self.build_batches(policy, mix_count, epoch)
        n_src = rows = seen = 0
        for first in range(0, min(nb, max_groups * self.G), self.G):
            n = min(self.G, nb - first)
            self.sample_group(first, n, p_intra, epoch, flags=self.sample_flags & ~B.CR_SAMPLE_INPUT_GLOBAL_IDS)
            h = self.headers()[0][:n]
            n_src += int(h[:, 1].sum())
            rows += int(h[:, 2].sum() + h[:, 0].sum())
            seen += n
        return n_src / max(1, seen), n_src / max(1, rows)

    def headers(self):
        """Host copy of the current group's block headers: [layer][batch] -> (n_dst, n_src, nnz, status)."""
        return [b.hdr.cpu().numpy()[:, :4].copy() for b in self.blocks]


def _now():
    import time
    return time.perf_counter()


class _BlockSetView:
    """A block set restricted to its first n batches (same device storage)."""

    def __init__(self, c):
        self.c = c


def _one_batch_view(b: B.BlockSet, g: int, frontier) -> _BlockSetView:
    """Batch g of a block set as a block set of its own, with `frontier` (device int32[cap_src]) in place of src_ids."""
    off = lambda t, stride: None if t is None else C.c_void_p(t.data_ptr() + 4 * g * stride)
    c = B.cr_block_set(1, b.fanout, b.cap_dst, b.cap_src, b.cap_nnz, 0, off(b.hdr, B.CR_HDR_WORDS), B._ptr(frontier),
                       off(b.indptr, b.cap_dst + 1), off(b.indices, b.cap_nnz), None, None, None,
                       off(b.row_order, b.cap_dst) if b.c.row_order else None)
    return _BlockSetView(c)


def _view_block_set(b: B.BlockSet, n_batches: int) -> _BlockSetView:
    c = B.cr_block_set(n_batches, b.fanout, b.cap_dst, b.cap_src, b.cap_nnz, 0, B._ptr(b.hdr), B._ptr(b.src_ids),
                       B._ptr(b.indptr), B._ptr(b.indices), B._ptr(b.t_indptr), B._ptr(b.t_indices), B._ptr(b.gather_ids),
                       b.c.row_order, b.c.group_order)
    return _BlockSetView(c)
