"""GPU parity: cr_gather_aggregate_fwd / _bwd against the oracle on oracle-sampled blocks."""
import ctypes as C

import numpy as np
import pytest

import oracle
from paper_2504_18082_amd import synth
from gpu_util import assert_close, bf16_tensor_to_float

pytestmark = pytest.mark.gpu
RTOL = 1e-5          # fp32 aggregation
RTOL_BF16 = 2.0 ** -8  # one rounding to bf16 of an fp32-exact value (half an ulp = 2^-9), with margin


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available()
    return torch


def _features(rng, n, F, dtype):
    ld = (F + 7) // 8 * 8 if dtype == "bf16" else (F + 3) // 4 * 4
    x = np.zeros((n, ld), dtype=np.float32)
    x[:, :F] = rng.standard_normal((n, F), dtype=np.float32)
    return synth.float_to_bf16_bits(x) if dtype == "bf16" else x


@pytest.mark.parametrize("F,dtype", [(64, "f32"), (100, "f32"), (128, "f32"), (256, "f32"), (602, "f32"),
                                     (1024, "f32"), (7, "f32"), (128, "bf16"), (200, "bf16"), (512, "bf16"), (1000, "bf16")])
def test_gather_fwd_indirect(torch_mod, tiny_workload, F, dtype):
    torch = torch_mod
    from paper_2504_18082_amd import binding as B
    w = tiny_workload
    rng = np.random.default_rng(F)
    table = _features(rng, w.cfg.n_nodes, F, dtype)
    roots = w.train_ids[:300]
    blocks = oracle.sample_blocks(w.graph, roots, [10, 5], 0.9, False, 0, 0, 0)
    blk = blocks[0]                                  # ~1.7K rows: several tiles and a ragged tail
    print(f"case F={F} dtype={dtype} n_dst={blk.n_dst} nnz={blk.nnz}", flush=True)
    want_agg, want_self = oracle.gather_mean(blk, table, indirect=True, F=F, want_self=True)
    if dtype == "bf16":
        abs_table = (table & np.uint16(0x7FFF))
    else:
        abs_table = np.abs(table)
    term_scale = oracle.gather_mean(blk, abs_table, indirect=True, F=F)      # mean |term| per element

    bs = B.BlockSet.from_host(blk, 10, gather_ids=(F % 2 == 0))     # both index paths: per-edge ids / src_ids[indices]
    dev_table = torch.from_numpy(table.view(np.int16) if dtype == "bf16" else table).cuda()
    ldb = (F + 31) // 32 * 32
    agg = torch.full((bs.cap_dst, F), np.nan, dtype=torch.float32, device="cuda")
    agg_b = torch.full((bs.cap_dst, ldb), 0x7FC0, dtype=torch.int16, device="cuda")
    self_b = torch.full((bs.cap_dst, ldb), 0x7FC0, dtype=torch.int16, device="cuda")
    B.cr_gather_aggregate_fwd(bs, 0, dev_table, B.CR_BF16 if dtype == "bf16" else B.CR_F32, table.shape[1], F, True,
                              agg, agg_b, self_b, ldb)
    torch.cuda.synchronize()
    assert_close(agg.cpu().numpy(), want_agg, RTOL, "agg", term_scale)
    ab = bf16_tensor_to_float(agg_b)
    assert_close(ab[:, :F], want_agg, RTOL_BF16, "agg_bf16", RTOL / RTOL_BF16 * term_scale)
    assert np.all(ab[:, F:] == 0)
    sb = bf16_tensor_to_float(self_b)
    np.testing.assert_array_equal(sb[:, :F].astype(np.float64), oracle.round_bf16(want_self))
    assert np.all(sb[:, F:] == 0)


def test_gather_fwd_direct_and_empty_rows(torch_mod, tiny_workload):
    torch = torch_mod
    from paper_2504_18082_amd import binding as B
    w = tiny_workload
    # strict sampling at p=1 leaves some rows empty; isolated nodes too
    roots = w.train_ids[:500]
    blk = oracle.sample_hop(w.graph, roots, 5, 1.0, True, 0, 0, 0, 1)
    deg = np.diff(blk.indptr)
    assert (deg == 0).any()
    rng = np.random.default_rng(0)
    H = rng.standard_normal((blk.n_src, 64), dtype=np.float32)
    want = oracle.gather_mean(blk, H, indirect=False)
    bs = B.BlockSet.from_host(blk, 5)
    agg = torch.full((bs.cap_dst, 64), np.nan, dtype=torch.float32, device="cuda")
    B.cr_gather_aggregate_fwd(bs, 0, torch.from_numpy(H).cuda(), B.CR_F32, 64, 64, False, agg)
    torch.cuda.synchronize()
    got = agg.cpu().numpy()
    assert_close(got, want, RTOL, "agg direct")
    assert np.all(got[deg == 0] == 0.0)


def test_rows_beyond_n_dst_are_untouched(torch_mod, tiny_workload):
    torch = torch_mod
    from paper_2504_18082_amd import binding as B
    w = tiny_workload
    blk = oracle.sample_hop(w.graph, w.train_ids[:100], 5, 0.5, False, 0, 0, 0, 0)
    bs = B.BlockSet.from_host(blk, 5)
    bs.hdr[0, 0] = 37            # pretend only 37 rows exist
    table = torch.from_numpy(np.ascontiguousarray(w.features)).cuda()
    agg = torch.full((bs.cap_dst, 64), -7.0, dtype=torch.float32, device="cuda")
    B.cr_gather_aggregate_fwd(bs, 0, table, B.CR_F32, 64, 64, True, agg)
    torch.cuda.synchronize()
    got = agg.cpu().numpy()
    assert np.all(got[37:] == -7.0) and not np.any(got[:37] == -7.0)
    # empty block: nothing happens, nothing faults
    bs.hdr[0, 0] = 0
    agg.fill_(-7.0)
    B.cr_gather_aggregate_fwd(bs, 0, table, B.CR_F32, 64, 64, True, agg)
    torch.cuda.synchronize()
    assert np.all(agg.cpu().numpy() == -7.0)


@pytest.mark.parametrize("F", [64, 100, 256, 300])
def test_gather_bwd(torch_mod, tiny_workload, F):
    torch = torch_mod
    from paper_2504_18082_amd import binding as B
    w = tiny_workload
    roots = w.train_ids[:700]
    blk = oracle.transpose_block(oracle.sample_hop(w.graph, roots, 10, 0.9, False, 1, 2, 3, 1))
    print(f"case bwd F={F} n_dst={blk.n_dst} n_src={blk.n_src} nnz={blk.nnz}", flush=True)
    rng = np.random.default_rng(F)
    ld_in = (F + 31) // 32 * 32
    d_agg = np.zeros((blk.n_dst, ld_in), dtype=np.float32)
    d_self = np.zeros((blk.n_dst, ld_in), dtype=np.float32)
    d_agg[:, :F] = rng.standard_normal((blk.n_dst, F), dtype=np.float32)
    d_self[:, :F] = rng.standard_normal((blk.n_dst, F), dtype=np.float32)
    relu_out = rng.standard_normal((blk.n_src, ld_in), dtype=np.float32)
    want = oracle.gather_mean_bwd(blk, d_agg[:, :F], d_self[:, :F])
    want_masked = want * (relu_out[:, :F] > 0)

    bs = B.BlockSet.from_host(blk, 10)
    up = lambda a: torch.from_numpy(a).cuda()
    d_src = torch.full((bs.cap_src, F), np.nan, dtype=torch.float32, device="cuda")
    B.cr_gather_aggregate_bwd(bs, 0, up(d_agg), up(d_self), ld_in, F, d_src=d_src)
    torch.cuda.synchronize()
    assert_close(d_src.cpu().numpy(), want, RTOL, "d_src")
    d_src_b = torch.full((bs.cap_src, ld_in), 0x7FC0, dtype=torch.int16, device="cuda")
    B.cr_gather_aggregate_bwd(bs, 0, up(d_agg), up(d_self), ld_in, F, up(relu_out), ld_in, d_src, d_src_b, ld_in)
    torch.cuda.synchronize()
    assert_close(d_src.cpu().numpy(), want_masked, RTOL, "d_src masked")
    # the mask may also come from a bf16 copy of the forward output
    relu_b = torch.from_numpy(synth.float_to_bf16_bits(relu_out).view(np.int16)).cuda()
    d_src2 = torch.full((bs.cap_src, F), np.nan, dtype=torch.float32, device="cuda")
    B.cr_gather_aggregate_bwd(bs, 0, up(d_agg), up(d_self), ld_in, F, relu_b, ld_in, d_src2, None, 0, relu_dtype=B.CR_BF16)
    torch.cuda.synchronize()
    want_masked_b = want * (synth.bf16_bits_to_float(synth.float_to_bf16_bits(relu_out))[:, :F] > 0)
    assert_close(d_src2.cpu().numpy(), want_masked_b, RTOL, "d_src masked by bf16")
    got_b = bf16_tensor_to_float(d_src_b)
    assert_close(got_b[:, :F], want_masked, RTOL_BF16, "d_src bf16")
    assert np.all(got_b[:, F:] == 0)
    # bf16 input gradients, [d_self | d_agg] side by side in one array: the oracle gets the same rounded values
    both = np.concatenate([d_self, d_agg], axis=1)
    both_b = torch.from_numpy(synth.float_to_bf16_bits(both).view(np.int16)).cuda()
    rounded = synth.bf16_bits_to_float(synth.float_to_bf16_bits(both))
    want_b = oracle.gather_mean_bwd(blk, rounded[:, ld_in:ld_in + F], rounded[:, :F]) * (relu_out[:, :F] > 0)
    d_src3 = torch.full((bs.cap_src, F), np.nan, dtype=torch.float32, device="cuda")
    d_src3_b = torch.full((bs.cap_src, ld_in), 0x7FC0, dtype=torch.int16, device="cuda")
    B.cr_gather_aggregate_bwd(bs, 0, C.c_void_p(both_b.data_ptr() + 2 * ld_in), both_b, 2 * ld_in, F, up(relu_out), ld_in, d_src3,
                              d_src3_b, ld_in, in_dtype=B.CR_BF16)
    torch.cuda.synchronize()
    assert_close(d_src3.cpu().numpy(), want_b, RTOL, "d_src from bf16 inputs")
    got_b3 = bf16_tensor_to_float(d_src3_b)
    assert_close(got_b3[:, :F], want_b, RTOL_BF16, "d_src bf16 from bf16 inputs")
    assert np.all(got_b3[:, F:] == 0)
    # without the self path
    B.cr_gather_aggregate_bwd(bs, 0, up(d_agg), None, ld_in, F, d_src=d_src)
    torch.cuda.synchronize()
    assert_close(d_src.cpu().numpy(), oracle.gather_mean_bwd(blk, d_agg[:, :F]), RTOL, "d_src no self")


@pytest.mark.parametrize("F,in_bf16", [(64, False), (256, True), (600, True)])
def test_gather_bwd_hub_sources(torch_mod, F, in_bf16):
    """A hand-made block in which a few source rows are used by very many destinations (segments of the transposed
    block far longer than a pass, and longer than the lanes of a row group) beside sources used once or not at all."""
    torch = torch_mod
    from paper_2504_18082_amd import binding as B
    rng = np.random.default_rng(F)
    n_dst, n_src, fanout = 500, 3000, 6
    hubs = np.array([0, 1, 777], dtype=np.int32)           # two hubs are destinations themselves, one is not
    rows = []
    for v in range(n_dst):
        nb = set(rng.choice(np.arange(2, n_src - 1), size=int(rng.integers(0, fanout - 2)), replace=False).tolist())
        if v % 2 == 0: nb.add(0)
        if v % 3 == 0: nb.add(1)
        if v % 5 != 0: nb.add(777)
        rows.append(np.array(sorted(nb), dtype=np.int32))
    indptr = np.zeros(n_dst + 1, dtype=np.int32)
    indptr[1:] = np.cumsum([len(r) for r in rows])
    indices = np.concatenate(rows).astype(np.int32)
    blk = oracle.transpose_block(oracle.Block(n_dst, np.arange(n_src, dtype=np.int32), indptr, indices, np.zeros_like(indices)))
    uses = np.diff(blk.t_indptr)
    assert uses[0] == 250 and uses[777] == 400 and uses[n_src - 1] == 0
    print(f"case bwd hubs F={F} bf16={in_bf16} nnz={blk.nnz}", flush=True)
    ld_in = (F + 31) // 32 * 32
    both = np.zeros((n_dst, 2 * ld_in), dtype=np.float32)
    both[:, :F] = rng.standard_normal((n_dst, F), dtype=np.float32)
    both[:, ld_in:ld_in + F] = rng.standard_normal((n_dst, F), dtype=np.float32)
    if in_bf16:
        both = synth.bf16_bits_to_float(synth.float_to_bf16_bits(both))
    want = oracle.gather_mean_bwd(blk, both[:, ld_in:ld_in + F], both[:, :F])
    bs = B.BlockSet.from_host(blk, fanout)
    d_src = torch.full((bs.cap_src, F), np.nan, dtype=torch.float32, device="cuda")
    if in_bf16:
        dev = torch.from_numpy(synth.float_to_bf16_bits(both).view(np.int16)).cuda()
        B.cr_gather_aggregate_bwd(bs, 0, C.c_void_p(dev.data_ptr() + 2 * ld_in), dev, 2 * ld_in, F, d_src=d_src, in_dtype=B.CR_BF16)
    else:
        dev = torch.from_numpy(both).cuda()
        B.cr_gather_aggregate_bwd(bs, 0, C.c_void_p(dev.data_ptr() + 4 * ld_in), dev, 2 * ld_in, F, d_src=d_src)
    torch.cuda.synchronize()
    got = d_src.cpu().numpy()
    assert_close(got[:n_src], want, RTOL, "d_src with hub sources")
    assert np.all(got[n_src - 1] == 0)                      # a source nobody uses and that is no destination


@pytest.mark.parametrize("F,dtype,gcn", [(128, "f32", False), (602, "f32", False), (256, "bf16", False), (100, "f32", True)])
def test_gather_fwd_with_a_processing_order(torch_mod, tiny_workload, F, dtype, gcn):
    """A block set that carries a row order (any permutation of the destination rows) gives bit-identical outputs:
    the order only says which workgroup handles a row and when."""
    torch = torch_mod
    from paper_2504_18082_amd import binding as B
    w = tiny_workload
    rng = np.random.default_rng(F + 1)
    table = _features(rng, w.cfg.n_nodes, F, dtype)
    roots = w.train_ids[:700]
    blk = oracle.sample_blocks(w.graph, roots, [10, 5], 0.9, False, 0, 0, 0)[0]
    print(f"case order F={F} dtype={dtype} gcn={gcn} n_dst={blk.n_dst}", flush=True)
    dev_table = torch.from_numpy(table.view(np.int16) if dtype == "bf16" else table).cuda()
    ldb = (F + 31) // 32 * 32
    if gcn:
        indptr = torch.from_numpy(w.indptr.astype(np.int64)).cuda()
        indices = torch.from_numpy(w.indices.astype(np.int32)).cuda()
        comm = torch.from_numpy(w.comm.astype(np.int32)).cuda()
        norm = B.cr_graph_gcn_norm(B.make_graph(indptr, indices, comm, w.cfg.n_comm))
    results = []
    for order in (None, rng.permutation(blk.n_dst), np.arange(blk.n_dst)[::-1]):
        blk.row_order = order
        bs = B.BlockSet.from_host(blk, 10, gather_ids=True)
        agg = torch.full((bs.cap_dst, F), np.nan, dtype=torch.float32, device="cuda")
        agg_b = torch.full((bs.cap_dst, ldb), 0x7FC0, dtype=torch.int16, device="cuda")
        self_b = torch.full((bs.cap_dst, ldb), 0x7FC0, dtype=torch.int16, device="cuda")
        dt = B.CR_BF16 if dtype == "bf16" else B.CR_F32
        if gcn:
            blk_norm = torch.zeros(bs.cap_src + 2 * bs.cap_dst, dtype=torch.float32, device="cuda")
            B.cr_gcn_block_norm(bs, 0, norm, blk_norm)
            B.cr_gcn_aggregate_fwd(bs, 0, norm, blk_norm, dev_table, dt, table.shape[1], F, True, agg, agg_b, ldb)
        else:
            B.cr_gather_aggregate_fwd(bs, 0, dev_table, dt, table.shape[1], F, True, agg, agg_b, self_b, ldb)
        torch.cuda.synchronize()
        results.append((agg.cpu().numpy().copy(), agg_b.cpu().numpy().copy(), self_b.cpu().numpy().copy()))
    blk.row_order = None
    assert not np.isnan(results[0][0][:blk.n_dst]).any()
    for other in results[1:]:
        for a, b in zip(results[0], other):
            np.testing.assert_array_equal(a, b)
