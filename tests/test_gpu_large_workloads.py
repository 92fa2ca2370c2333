"""GPU parity at the sizes the benchmark's numbers come from, in the benchmark's launch configuration (groups of 32
mini-batches of 1024 roots, three layers, input-side block in global ids, layer-0 gather once per group over the
group-wide community order):

  reddit-like   : 233 K nodes, ~114 M adjacency entries (mean degree 490: most destination rows take the long-row
                  paths of the selection), 2408-byte float rows gathered in five 512-byte column panels, 41 classes
  products-like : 2.45 M nodes, ~124 M adjacency entries, 400-byte float rows (not 128-byte aligned), 5000 communities
  papers-like   : the FULL shape, 111 M nodes, ~3.2 G adjacency entries (offsets beyond 2^31), 256-byte bf16 rows,
                  100,000 communities, 172 classes; the graph is too large for the direct-address de-duplication
                  table, so the open-addressing table is the one that runs

The workloads are generated on the GPU (set-up) and the graph arrays are copied to the host for the oracle.  Root
partitioning is compared in full; two batches of the group are compared with the oracle in full (every array of every
block, the layer-0 aggregate of every row), invariants are checked on all 32; one whole training step is compared with
the oracle's step.
"""
import numpy as np
import pytest

import oracle
from gpu_util import assert_close, bf16_tensor_to_float, relu_flip_allowance, rms_rel_err
from oracle_step import oracle_train_step
from paper_2504_18082_amd import synth

pytestmark = pytest.mark.gpu
GROUP = 32
RTOL_BF16 = 2e-2        # element-wise, downstream of bf16 products
RTOL_RMS = 5e-3         # root-mean-square of the difference over the root-mean-square of the tensor


class Large:
    """One generated workload: device tensors for the GPU path, host copies of the graph for the oracle."""

    def __init__(self, name):
        import torch
        from paper_2504_18082_amd import synth_gpu
        print(f"generating {name} on the GPU", flush=True)
        self.dw = synth_gpu.make_workload_gpu(name, seed=0)
        torch.cuda.synchronize()
        d = self.dw
        self.cfg = d.cfg
        print(f"{name}: {d.n_entries} adjacency entries; copying the graph to the host", flush=True)
        self.indptr = d.indptr.cpu().numpy()
        self.indices = d.indices.cpu().numpy()
        self.comm = d.comm.cpu().numpy()
        self.labels = d.labels.cpu().numpy()
        self.train_ids = d.train_ids.cpu().numpy()
        self.graph = (self.indptr, self.indices, self.comm)
        self.deg = np.diff(self.indptr)

    def rows_of_table(self, ids):
        """Feature rows of the given nodes, from the device table, as the oracle's table type (float32 or raw bf16)."""
        import torch
        rows = self.dw.features[torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int64)).cuda()].cpu().numpy()
        return rows.view(np.uint16) if rows.dtype == np.int16 else rows


@pytest.fixture(scope="module", params=["reddit", "products", "papers"])
def large(request):
    import torch
    lw = Large(request.param)
    yield lw
    del lw
    torch.cuda.empty_cache()


def test_bench_configuration(large):
    import torch
    from paper_2504_18082_amd import binding as B
    from paper_2504_18082_amd.trainer import Trainer
    lw, cfg = large, large.cfg
    L = len(cfg.fanouts)
    seed, epoch = 0, 2
    scfg = B.make_sample_cfg(cfg.fanouts, 0.5, seed, epoch)
    kind = B.cr_sample_blocks_dedup_table(scfg, cfg.n_nodes, cfg.batch_size)
    if cfg.name == "papers":
        assert lw.dw.n_entries > 2 ** 31, "the papers-like graph must exercise offsets beyond 31 bits"
        assert kind == B.CR_DEDUP_HASH
        assert cfg.n_comm > 4096
    else:
        assert kind == B.CR_DEDUP_DIRECT

    # ---- root partitioning, in full (RAND and a mixing COMM-RAND setting)
    tr = Trainer(lw.dw, group_size=GROUP, lr=0.01, seed=seed)
    assert tr.group_gather, "the benchmark's configuration gathers layer 0 once per group"
    mix = B.cr_mix_count_from_percent(12.5, lw.dw.n_comm_in_train)
    for policy, m in ((B.CR_ROOTS_COMM_RAND, mix), (B.CR_ROOTS_RAND, 1)):
        print(f"{cfg.name}: root partitioning policy {policy} mix {m}", flush=True)
        tr.build_batches(policy, m, epoch)
        perm = tr.perm.cpu().numpy()
        assert np.array_equal(perm, oracle.build_batches(policy, m, seed, epoch, lw.train_ids, lw.comm, cfg.n_comm))

    # ---- one group of 32 batches, as the benchmark samples it (RAND roots are current)
    first = GROUP                                      # second group of the epoch
    for p, full_batches in ((0.5, (0, 31)), (1.0, (17,)), (0.9, (5,))):
        print(f"{cfg.name}: sampling a group of {GROUP} at p={p}", flush=True)
        tr.sample_group(first, GROUP, p, epoch)
        torch.cuda.synchronize()
        assert tr.ctx.poll_error() == (B.CR_OK, 0)
        hdrs = tr.headers()
        blocks = tr.blocks
        # invariants on every batch: sizes chain, counts = min(fanout, degree), ids are neighbours (sampled)
        for g in range(GROUP):
            roots = perm[(first + g) * cfg.batch_size:(first + g + 1) * cfg.batch_size]
            for l in range(L - 1, -1, -1):
                n_dst, n_src, nnz, status = hdrs[l][g]
                assert status == 0
                dst = blocks[l].src_ids[g, :n_dst].cpu().numpy()
                if l == L - 1:
                    assert np.array_equal(dst, roots)
                else:
                    assert n_dst == hdrs[l + 1][g][1] and np.array_equal(dst, blocks[l + 1].src_ids[g, :n_dst].cpu().numpy())
                indptr = blocks[l].indptr[g, :n_dst + 1].cpu().numpy()
                assert indptr[0] == 0 and indptr[-1] == nnz
                assert np.array_equal(np.diff(indptr), np.minimum(lw.deg[dst], cfg.fanouts[l]))
                if l >= 1:
                    src = blocks[l].src_ids[g, :n_src].cpu().numpy()
                    assert len(np.unique(src)) == n_src
                    idx = blocks[l].indices[g, :nnz].cpu().numpy()
                    assert idx.min(initial=0) >= 0 and idx.max(initial=0) < n_src
                else:
                    assert n_src == -1
        # full comparison with the oracle
        pos = np.full(cfg.n_nodes, -1, dtype=np.int32)
        for g in full_batches:
            print(f"{cfg.name}: oracle sampling for batch {first + g} at p={p}", flush=True)
            roots = perm[(first + g) * cfg.batch_size:(first + g + 1) * cfg.batch_size]
            want = oracle.sample_blocks(lw.graph, roots, cfg.fanouts, p, False, seed, epoch, first + g, pos)
            if cfg.name == "papers":
                touched = lw.indptr[want[0].src_ids[:want[0].n_dst].astype(np.int64)]
                assert (touched > 2 ** 31).any(), "the compared rows must include adjacency offsets beyond 31 bits"
            for l, ob in enumerate(want):
                blk = blocks[l]
                if l == 0:
                    assert hdrs[0][g].tolist() == [ob.n_dst, -1, ob.nnz, 0]
                    assert np.array_equal(blk.indptr[g, :ob.n_dst + 1].cpu().numpy(), ob.indptr)
                    assert np.array_equal(blk.gather_ids[g, :ob.nnz].cpu().numpy(), ob.src_ids[ob.indices])
                    assert np.array_equal(blk.src_ids[g, :ob.n_dst].cpu().numpy(), ob.src_ids[:ob.n_dst])
                    continue
                assert hdrs[l][g].tolist() == [ob.n_dst, ob.n_src, ob.nnz, 0]
                assert np.array_equal(blk.src_ids[g, :ob.n_src].cpu().numpy(), ob.src_ids)
                assert np.array_equal(blk.indptr[g, :ob.n_dst + 1].cpu().numpy(), ob.indptr)
                assert np.array_equal(blk.indices[g, :ob.nnz].cpu().numpy(), ob.indices)
                assert np.array_equal(blk.t_indptr[g, :ob.n_src + 1].cpu().numpy(), ob.t_indptr)
                assert np.array_equal(blk.t_indices[g, :ob.nnz].cpu().numpy(), ob.t_indices)
            # the grouped layer-0 gather (bf16 operand outputs), every row of this batch, against orc_gather_mean
            assert tr.group_gathered[0]
            # (the oracle reads the rows of this block's frontier, fetched from the device table in frontier order, with
            # dense addressing, instead of a host copy of the whole table)
            table = np.ascontiguousarray(lw.rows_of_table(want[0].src_ids))
            agg_ref, self_ref = oracle.gather_mean(want[0], table, indirect=False, F=cfg.n_feat, want_self=True)
            agg = bf16_tensor_to_float(tr.agg0_all[0][g])[:want[0].n_dst, :cfg.n_feat]
            selfb = bf16_tensor_to_float(tr.self0_all[0][g])[:want[0].n_dst, :cfg.n_feat]
            # the kernel sums in float and rounds once to bf16 (2^-9 relative); sums that cancel are judged against the
            # magnitude of what was added up
            scale = np.sqrt(np.mean(agg_ref * agg_ref))
            assert_close(agg, agg_ref, 2.0 ** -8, f"{cfg.name} layer-0 aggregate batch {g}", scale)
            np.testing.assert_array_equal(selfb.astype(np.float64), oracle.round_bf16(self_ref))
    del tr
    torch.cuda.empty_cache()


def test_input_frontier_deduplicated_at_scale(large):
    """The same group with the input frontier de-duplicated (what a feature cache, a host-resident store or graph
    attention need): at the papers-like size the largest table of the open-addressing path, at the products-like size
    the direct-address table."""
    import torch
    from paper_2504_18082_amd import binding as B
    from paper_2504_18082_amd.trainer import Trainer
    lw, cfg = large, large.cfg
    seed, epoch, first = 0, 1, 0
    tr = Trainer(lw.dw, group_size=GROUP, lr=0.01, seed=seed, relabel_input=True)
    tr.build_batches(B.CR_ROOTS_RAND, 1, epoch)
    perm = tr.perm.cpu().numpy()
    tr.sample_group(first, GROUP, 0.5, epoch)
    torch.cuda.synchronize()
    hdrs = tr.headers()
    for g in range(GROUP):
        n_dst, n_src, nnz, status = hdrs[0][g]
        assert status == 0
        src = tr.blocks[0].src_ids[g, :n_src].cpu().numpy()
        assert len(np.unique(src)) == n_src
        idx = tr.blocks[0].indices[g, :nnz].cpu().numpy()
        assert np.array_equal(tr.blocks[0].gather_ids[g, :nnz].cpu().numpy(), src[idx])
    g = 5
    print(f"{cfg.name}: oracle sampling for batch {first + g} (de-duplicated input frontier)", flush=True)
    pos = np.full(cfg.n_nodes, -1, dtype=np.int32)
    roots = perm[(first + g) * cfg.batch_size:(first + g + 1) * cfg.batch_size]
    want = oracle.sample_blocks(lw.graph, roots, cfg.fanouts, 0.5, False, seed, epoch, first + g, pos)
    ob, blk = want[0], tr.blocks[0]
    assert hdrs[0][g].tolist() == [ob.n_dst, ob.n_src, ob.nnz, 0]
    assert np.array_equal(blk.src_ids[g, :ob.n_src].cpu().numpy(), ob.src_ids)
    assert np.array_equal(blk.indices[g, :ob.nnz].cpu().numpy(), ob.indices)
    del tr
    torch.cuda.empty_cache()


def test_one_training_step(large):
    """One whole step (forward, loss, backward, SGD) of the first batch of a group of 32 against the oracle's step
    (the composition that mirrors the bf16 storage points; the oracle's source built with OpenMP to keep the test
    short: same sums in the same order).  papers-like: 172 classes, the loss runs in its separate kernels."""
    import torch
    from paper_2504_18082_amd import binding as B
    from paper_2504_18082_amd.trainer import Trainer
    from gpu_util import assert_weight_step
    lw, cfg = large, large.cfg
    seed, epoch, p, lr, wd = 0, 4, 0.9, 0.01, 5e-4
    weights = synth.init_weights(cfg, seed)
    tr = Trainer(lw.dw, group_size=GROUP, lr=lr, weight_decay=wd, seed=seed, weights=weights)
    mix = B.cr_mix_count_from_percent(25.0, lw.dw.n_comm_in_train)
    tr.build_batches(B.CR_ROOTS_COMM_RAND, mix, epoch)
    perm = tr.perm.cpu().numpy()
    tr.sample_group(0, GROUP, p, epoch)
    dW_out = [torch.zeros_like(l.W) for l in tr.layers]
    db_out = [torch.zeros(l.F_out, dtype=torch.float32, device="cuda") for l in tr.layers]
    g = 3
    tr.train_batch(g, dW_out, db_out)
    torch.cuda.synchronize()
    roots = perm[g * cfg.batch_size:(g + 1) * cfg.batch_size]
    params = [(W.astype(np.float64), b.astype(np.float64)) for W, b in weights]
    print(f"{cfg.name}: oracle training step", flush=True)
    # the oracle samples first (the step below samples the same blocks again), then gets the rows of its input frontier
    pos = np.full(cfg.n_nodes, -1, dtype=np.int32)
    blocks = oracle.sample_blocks(lw.graph, roots, cfg.fanouts, p, False, seed, epoch, g, pos)
    table = np.ascontiguousarray(lw.rows_of_table(blocks[0].src_ids))
    oracle.use_all_cores(True)
    try:
        ref = oracle_train_step(lw.graph, table, cfg.n_feat, lw.labels, roots, cfg.fanouts, p, seed, epoch, g,
                                params, lr, wd, pos, mirror=True, table_is_frontier=True)
    finally:
        oracle.use_all_cores(False)
    # Element by element at the bf16 tolerance; in the root-mean-square sense far tighter.  (Against this composition
    # the differences are accumulation order and bf16 values that sat on a rounding boundary: with 60 K rows summed into
    # every element of a weight gradient a few per cent of the stored bf16 gradients fall the other way.)
    assert abs(float(tr.loss.cpu()[0]) - ref["loss"]) <= 1e-3 * abs(ref["loss"])
    logits = tr.out[tr.L - 1].cpu().numpy()[:len(roots), :cfg.n_classes]
    assert_close(logits, ref["logits"], RTOL_BF16, f"{cfg.name} logits")
    report = {"logits": rms_rel_err(logits, ref["logits"])}
    for l in range(tr.L):
        dW, db = dW_out[l].cpu().numpy(), db_out[l].cpu().numpy()
        allow_dW = allow_db = None
        if l < tr.L - 1:        # ReLU decisions on activations within rounding of zero may differ: allow exactly their share
            n_rows, n_cols = ref["outs"][l].shape
            allow_dW, allow_db, flips = relu_flip_allowance(
                bf16_tensor_to_float(tr.out_b[l])[:n_rows, :n_cols], oracle.round_bf16(ref["outs"][l]),
                bf16_tensor_to_float(tr.dz[l])[:n_rows, :n_cols], ref["dzs"][l], np.hstack([ref["h_self"][l], ref["aggs"][l]]))
            print(f"{cfg.name}: layer {l}: {flips} of {n_rows * n_cols} ReLU decisions at the boundary differ", flush=True)
        assert_close(dW, ref["grads"][l][0], RTOL_BF16, f"{cfg.name} dW layer {l}", extra=allow_dW)
        assert_close(db, ref["grads"][l][1], RTOL_BF16, f"{cfg.name} db layer {l}", extra=allow_db)
        assert_weight_step(tr.layers[l].W.cpu().numpy(), params[l][0], ref["params"][l][0], params[l][0], RTOL_BF16,
                           f"{cfg.name} W change layer {l}", extra=None if allow_dW is None else lr * allow_dW)
        report[f"dW{l}"], report[f"db{l}"] = rms_rel_err(dW, ref["grads"][l][0]), rms_rel_err(db, ref["grads"][l][1])
    print(f"{cfg.name}: rms |gpu - oracle| / rms oracle:", {k: float(f"{v:.3g}") for k, v in report.items()}, flush=True)
    assert max(report.values()) <= RTOL_RMS, report
    del tr
    torch.cuda.empty_cache()
