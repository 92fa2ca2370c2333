"""One training step of the L-layer GraphSAGE-mean model written with the oracle's pieces only
(test infrastructure).

Two compositions of the same pieces:
  mirror=False  the precision model of the plain definition: the operands of every dense product are rounded to
                bf16 (the matrix cores take bf16), everything between the products -- hidden activations,
                aggregates, gradients -- stays in float64;
  mirror=True   additionally rounds what the GPU path STORES in bf16 between its kernels: hidden activations
                (self operand, aggregation input, ReLU mask), the input gradients d_self / d_agg, and the bias
                gradient summed from the rounded dZ.
The GPU path is compared with both: with the mirror at a tight tolerance (only the accumulation order differs, and
bf16 values that sat on a rounding boundary), with the plain composition at the bf16 tolerance; a third composition in
exact float64 (round_operands=False) measures how far each bf16 model is from the unrounded result.
"""
import time

import numpy as np

import oracle


class StageTimers(dict):
    """Seconds per stage of the path, accumulated over calls (used by the benchmark's cpu_baseline leg)."""

    def add(self, stage, t0):
        self[stage] = self.get(stage, 0.0) + (time.perf_counter() - t0)


def oracle_forward(graph, table, n_feat, roots, fanouts, p, seed, epoch, batch, params, pos_map=None, strict=False,
                   mirror=True, timers=None, round_operands=True, table_is_frontier=False):
    """Sampling and forward pass only; returns (blocks, h_self, aggs, outs).  table_is_frontier: `table` holds the
    feature rows of this batch's input frontier only, in frontier order (for graphs whose whole table is not on the host)."""
    L = len(fanouts)
    tm = timers if timers is not None else StageTimers()
    t0 = time.perf_counter()
    blocks = oracle.sample_blocks(graph, roots, fanouts, p, strict, seed, epoch, batch, pos_map)
    tm.add("sample_blocks", t0)
    h_self, aggs, outs = [None] * L, [None] * L, [None] * L
    for l in range(L):
        blk = blocks[l]
        W, b = params[l]
        t0 = time.perf_counter()
        if l == 0:
            aggs[0], h_self[0] = oracle.gather_mean(blk, table, indirect=not table_is_frontier, F=n_feat, want_self=True)
            tm.add("gather_aggregate_fwd_layer0", t0)
        else:
            if mirror:      # hidden activations live in bf16 on the GPU
                prev = np.ascontiguousarray(oracle.round_bf16(outs[l - 1]).astype(np.float32))
                aggs[l] = oracle.gather_mean(blk, prev, indirect=False)
            else:
                aggs[l] = oracle.gather_mean(blk, np.ascontiguousarray(outs[l - 1]), indirect=False)
            h_self[l] = outs[l - 1][:blk.n_dst]
            tm.add("gather_aggregate_fwd_hidden", t0)
        t0 = time.perf_counter()
        outs[l] = oracle.sage_linear_fwd(h_self[l], aggs[l], W, b, l < L - 1, round_operands)
        tm.add("sage_linear_fwd", t0)
    return blocks, h_self, aggs, outs


def oracle_train_step(graph, table, n_feat, labels, roots, fanouts, p, seed, epoch, batch, params, lr, wd,
                      pos_map=None, strict=False, mirror=True, timers=None, round_operands=True, table_is_frontier=False):
    """params: list of (W float64 [2F_in, F_out], b float64 [F_out]); returns dict with loss, logits,
    grads and the updated params (inputs are not modified).  round_operands=False (with mirror=False) is the step in
    exact float64 arithmetic, nothing rounded anywhere: the yardstick for what each bf16 model costs in accuracy."""
    L = len(fanouts)
    tm = timers if timers is not None else StageTimers()
    blocks, h_self, aggs, outs = oracle_forward(graph, table, n_feat, roots, fanouts, p, seed, epoch, batch, params, pos_map, strict,
                                                mirror, tm, round_operands, table_is_frontier)
    t0 = time.perf_counter()
    loss, dz = oracle.softmax_xent(outs[L - 1], labels[np.asarray(roots)])
    tm.add("softmax_xent", t0)
    grads, new_params, dzs = [None] * L, [None] * L, [None] * L
    for l in range(L - 1, -1, -1):
        W, b = params[l]
        dzs[l] = dz
        t0 = time.perf_counter()
        dW, db, d_self, d_agg = oracle.sage_linear_bwd(h_self[l], aggs[l], W, outs[l], dz, False, round_operands, need_dx=l > 0)
        if mirror:
            db = oracle.round_bf16(dz).sum(axis=0)          # the GPU sums the operand it feeds the matrix cores
        grads[l] = (dW, db)
        new_params[l] = oracle.sgd_step(W, dW, b, db, lr, wd)
        tm.add("sage_linear_bwd_sgd", t0)
        if l > 0:
            t0 = time.perf_counter()
            if mirror:
                d_agg, d_self = oracle.round_bf16(d_agg), oracle.round_bf16(d_self)     # the GPU path stores them in bf16
            d_src = oracle.gather_mean_bwd(blocks[l], d_agg, d_self)
            dz = d_src * ((oracle.round_bf16(outs[l - 1]) if mirror else outs[l - 1]) > 0)
            tm.add("gather_aggregate_bwd", t0)
    return dict(blocks=blocks, loss=loss, logits=outs[L - 1], outs=outs, grads=grads, params=new_params, timers=tm, dzs=dzs,
                h_self=h_self, aggs=aggs)


def oracle_train_step_gcn(graph, table, n_feat, labels, roots, fanouts, p, seed, epoch, batch, params, lr, wd, pos_map=None):
    """The same step for GCN layers: params are (W float64 [F_in, F_out], b).  The dense part goes through the
    two-operand oracle with a zero self operand and zero W_self rows (adds exact zeros)."""
    L = len(fanouts)
    deg = np.diff(graph[0])
    blocks = oracle.sample_blocks(graph, roots, fanouts, p, False, seed, epoch, batch, pos_map)
    aggs, outs = [None] * L, [None] * L
    two = lambda W: np.vstack([np.zeros_like(W), W])
    for l in range(L):
        W, b = params[l]
        if l == 0:
            aggs[0] = oracle.gcn_aggregate(blocks[0], table, deg, indirect=True, F=n_feat)
        else:
            prev = np.ascontiguousarray(oracle.round_bf16(outs[l - 1]).astype(np.float32))
            aggs[l] = oracle.gcn_aggregate(blocks[l], prev, deg, indirect=False)
        outs[l] = oracle.sage_linear_fwd(np.zeros_like(aggs[l]), aggs[l], two(W), b, l < L - 1, True)
    loss, dz = oracle.softmax_xent(outs[L - 1], labels[np.asarray(roots)])
    grads, new_params = [None] * L, [None] * L
    for l in range(L - 1, -1, -1):
        W, b = params[l]
        F_in = W.shape[0]
        dW2, _, _, d_agg = oracle.sage_linear_bwd(np.zeros_like(aggs[l]), aggs[l], two(W), outs[l], dz, False, True, need_dx=l > 0)
        dW = dW2[F_in:]
        db = oracle.round_bf16(dz).sum(axis=0)
        grads[l] = (dW, db)
        W_new2, b_new = oracle.sgd_step(two(W), dW2, b, db, lr, wd)
        new_params[l] = (W_new2[F_in:], b_new)
        if l > 0:
            d_src = oracle.gcn_aggregate_bwd(blocks[l], oracle.round_bf16(d_agg), deg)
            dz = d_src * (oracle.round_bf16(outs[l - 1]) > 0)
    return dict(blocks=blocks, loss=loss, logits=outs[L - 1], outs=outs, grads=grads, params=new_params)


def oracle_train_step_gat(graph, table, n_feat, labels, roots, fanouts, p, seed, epoch, batch, params, heads, lr, wd,
                          pos_map=None, slope=0.2):
    """The same step for graph-attention layers: params are (W float64 [F_in, heads_l*D_l], a_l, a_r, bias) with
    `heads` heads on hidden layers and one on the last.  Precision points of the GPU path: bf16 operands into
    every contraction, projected rows z and hidden activations stored in bf16, gradients handed from one
    kernel to the next (d logits, d z, d input) stored in bf16."""
    L = len(fanouts)
    rb = oracle.round_bf16
    two = lambda W: np.vstack([np.zeros_like(W), W])
    blocks = oracle.sample_blocks(graph, roots, fanouts, p, False, seed, epoch, batch, pos_map)
    H = [heads if l < L - 1 else 1 for l in range(L)]
    xs, zs, outs = [None] * L, [None] * L, [None] * L
    for l in range(L):
        W, a_l, a_r, b = params[l]
        blk = blocks[l]
        if l == 0:
            xs[0] = oracle._as_float_table(table)[blk.src_ids.astype(np.int64), :n_feat]
        else:
            xs[l] = rb(outs[l - 1])
        proj = oracle.sage_linear_fwd(np.zeros_like(xs[l]), xs[l], two(W), np.zeros(W.shape[1]), False, True)
        zs[l] = rb(proj)
        out, _ = oracle.gat_attention_fwd(blk, zs[l], a_l, a_r, b, H[l], slope)
        outs[l] = np.maximum(out, 0.0) if l < L - 1 else out
    loss, d_logits = oracle.softmax_xent(outs[L - 1], labels[np.asarray(roots)])
    d_out = rb(d_logits)
    grads, new_params = [None] * L, [None] * L
    for l in range(L - 1, -1, -1):
        W, a_l, a_r, b = params[l]
        F_in = W.shape[0]
        g = d_out * (rb(outs[l]) > 0) if l < L - 1 else d_out
        d_z, d_al, d_ar, d_b = oracle.gat_attention_bwd(blocks[l], zs[l], a_l, a_r, H[l], g, slope)
        dz_b = rb(d_z)
        dW2, _, _, d_x = oracle.sage_linear_bwd(np.zeros_like(xs[l]), xs[l], two(W), np.zeros((len(xs[l]), W.shape[1])), dz_b,
                                                False, True, need_dx=l > 0)
        dW = dW2[F_in:]
        grads[l] = (dW, d_al, d_ar, d_b)
        new_params[l] = (W - lr * (dW + wd * W), a_l - lr * (d_al + wd * a_l), a_r - lr * (d_ar + wd * a_r), b - lr * d_b)
        if l > 0:
            d_out = rb(d_x)
    return dict(blocks=blocks, loss=loss, logits=outs[L - 1], outs=outs, grads=grads, params=new_params)
