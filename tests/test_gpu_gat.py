"""GPU parity of the graph-attention layer on sampled blocks (cr_gather_rows_bf16, cr_gat_attention_fwd / _bwd)
against the oracle.  Inputs are bf16-representable, so the two sides see the same numbers; the kernels compute in
float: scores are 64-term sums (relative error ~1e-6), the exponential passes an absolute score error e on as a
relative error e, hence 1e-4 on float outputs; bf16 outputs add half a bf16 ulp (2^-9)."""
import numpy as np
import pytest

import oracle
from paper_2504_18082_amd import synth
from gpu_util import assert_close, assert_weight_step, bf16_tensor_to_float

pytestmark = pytest.mark.gpu
RTOL = 1e-4
RTOL_BF16 = 2.0 ** -8


def bf16_exact(x):
    return synth.bf16_bits_to_float(synth.float_to_bf16_bits(np.asarray(x, dtype=np.float32)))


def dev_bf16(torch, x):
    return torch.from_numpy(synth.float_to_bf16_bits(np.ascontiguousarray(x, dtype=np.float32)).view(np.int16)).cuda()


@pytest.mark.parametrize("F,dtype", [(128, "f32"), (602, "f32"), (100, "f32"), (128, "bf16"), (50, "bf16")])
def test_gather_rows_bf16(F, dtype):
    import ctypes as C
    import torch
    from paper_2504_18082_amd import binding as B
    rng = np.random.default_rng(F)
    n_nodes, n = 5000, 1777
    ld = (F + 7) // 8 * 8 if dtype == "bf16" else (F + 3) // 4 * 4
    x = np.zeros((n_nodes, ld), dtype=np.float32)
    x[:, :F] = rng.standard_normal((n_nodes, F), dtype=np.float32)
    table = synth.float_to_bf16_bits(x) if dtype == "bf16" else x
    ids = rng.choice(n_nodes, size=n, replace=False).astype(np.int32)
    print(f"case gather_rows_bf16 F={F} dtype={dtype}", flush=True)
    ld_out = (F + 31) // 32 * 32
    hdr = torch.tensor([0, n, 0, 0, 0, 0, 0, 0], dtype=torch.int32, device="cuda")
    dev_ids = torch.from_numpy(ids).cuda()
    dev_table = torch.from_numpy(table.view(np.int16) if dtype == "bf16" else table).cuda()
    out = torch.full((n + 5, ld_out), 0x7FC0, dtype=torch.int16, device="cuda")
    B.cr_gather_rows_bf16(dev_table, B.CR_BF16 if dtype == "bf16" else B.CR_F32, ld, F, C.c_void_p(dev_ids.data_ptr()),
                          C.c_void_p(hdr.data_ptr()), B.CR_HDR_N_SRC, n + 5, out, ld_out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint16)
    want = synth.float_to_bf16_bits(x[ids])
    np.testing.assert_array_equal(got[:n, :F], want[:, :F])          # rounding to nearest even is exact work
    assert np.all(got[:n, F:] == 0)
    assert np.all(got[n:] == 0x7FC0)                                  # rows past the count are not touched


CASES = [(4, 64, 256), (1, 41, 64), (2, 16, 64), (8, 64, 512), (1, 172, 192), (3, 32, 128)]


def _setup(torch, w, heads, D, ld, seed, empty_row=True):
    from paper_2504_18082_amd import binding as B
    rng = np.random.default_rng(seed)
    roots = w.train_ids[:500]
    blk = oracle.transpose_block(oracle.sample_hop(w.graph, roots, 10, 0.9, False, 1, 2, 3, 1))
    HD = heads * D
    z = np.zeros((blk.n_src, ld), dtype=np.float32)
    z[:, :HD] = bf16_exact(rng.standard_normal((blk.n_src, HD)))
    a_l = (rng.standard_normal(HD) / np.sqrt(D)).astype(np.float32)
    a_r = (rng.standard_normal(HD) / np.sqrt(D)).astype(np.float32)
    bias = (0.1 * rng.standard_normal(HD)).astype(np.float32)
    bs = B.BlockSet.from_host(blk, 10)
    par = B.GatParams(a_l, a_r, bias, heads, ld)
    return rng, blk, z, a_l, a_r, bias, bs, par


@pytest.mark.parametrize("heads,D,ld", CASES)
@pytest.mark.parametrize("relu", [False, True])
def test_gat_attention_fwd(tiny_workload, heads, D, ld, relu):
    import torch
    from paper_2504_18082_amd import binding as B
    rng, blk, z, a_l, a_r, bias, bs, par = _setup(torch, tiny_workload, heads, D, ld, heads * 100 + D)
    HD = heads * D
    deg = np.diff(blk.indptr)
    print(f"case gat fwd heads={heads} D={D} ld={ld} relu={relu} n_dst={blk.n_dst} n_src={blk.n_src} nnz={blk.nnz} "
          f"empty rows={(deg == 0).sum()}", flush=True)
    want, _ = oracle.gat_attention_fwd(blk, z[:, :HD], a_l, a_r, bias, heads)
    if relu:
        want = np.maximum(want, 0.0)
    z_dev = dev_bf16(torch, z)
    el = torch.full((bs.cap_src, heads), np.nan, dtype=torch.float32, device="cuda")
    er = torch.full((bs.cap_src, heads), np.nan, dtype=torch.float32, device="cuda")
    stat = torch.full((bs.cap_dst, heads, 4), np.nan, dtype=torch.float32, device="cuda")
    out = torch.full((bs.cap_dst, ld), np.nan, dtype=torch.float32, device="cuda")
    out_b = torch.full((bs.cap_dst, ld), 0x7FC0, dtype=torch.int16, device="cuda")
    B.cr_gat_attention_fwd(bs, 0, par, z_dev, ld, relu, el, er, stat, out, out_b)
    torch.cuda.synchronize()
    z3 = z[:, :HD].astype(np.float64).reshape(-1, heads, D)
    assert_close(el.cpu().numpy()[:blk.n_src], (z3 * a_l.astype(np.float64).reshape(heads, D)).sum(-1), 1e-5, "el")
    assert_close(er.cpu().numpy()[:blk.n_src], (z3 * a_r.astype(np.float64).reshape(heads, D)).sum(-1), 1e-5, "er")
    got = out.cpu().numpy()
    assert_close(got[:blk.n_dst, :HD], want, RTOL, "gat out")
    assert np.all(got[:blk.n_dst, HD:] == 0)
    gb = bf16_tensor_to_float(out_b)
    assert_close(gb[:blk.n_dst, :HD], want, RTOL_BF16, "gat out bf16")
    assert np.all(gb[:blk.n_dst, HD:] == 0)


@pytest.mark.parametrize("heads,D,ld", CASES)
@pytest.mark.parametrize("relu", [False, True])
def test_gat_attention_bwd(tiny_workload, heads, D, ld, relu):
    import torch
    from paper_2504_18082_amd import binding as B
    rng, blk, z, a_l, a_r, bias, bs, par = _setup(torch, tiny_workload, heads, D, ld, heads * 100 + D + 7)
    HD = heads * D
    print(f"case gat bwd heads={heads} D={D} ld={ld} relu={relu} n_dst={blk.n_dst} n_src={blk.n_src} nnz={blk.nnz}", flush=True)
    z_dev = dev_bf16(torch, z)
    el = torch.zeros((bs.cap_src, heads), dtype=torch.float32, device="cuda")
    er = torch.zeros((bs.cap_src, heads), dtype=torch.float32, device="cuda")
    stat = torch.zeros((bs.cap_dst, heads, 4), dtype=torch.float32, device="cuda")
    out_b = torch.zeros((bs.cap_dst, ld), dtype=torch.int16, device="cuda")
    B.cr_gat_attention_fwd(bs, 0, par, z_dev, ld, relu, el, er, stat, None, out_b)
    torch.cuda.synchronize()
    out_host = bf16_tensor_to_float(out_b)[:blk.n_dst, :HD]

    ld_dout = ld + 64                                   # a wider gradient array (the dense layer's input gradient)
    d_out = np.zeros((blk.n_dst, ld_dout), dtype=np.float32)
    d_out[:, :HD] = bf16_exact(rng.standard_normal((blk.n_dst, HD)))
    g = d_out[:, :HD].astype(np.float64)
    if relu:
        g = g * (out_host > 0)                         # the mask is taken on the stored forward output
    want_dz, want_al, want_ar, want_b = oracle.gat_attention_bwd(blk, z[:, :HD], a_l, a_r, heads, g)

    lr, wd = 0.05, 1e-3
    ws = torch.empty(B.cr_gat_attention_bwd_workspace_bytes(bs.cap_dst, ld, heads), dtype=torch.uint8, device="cuda")
    dz = torch.full((bs.cap_src, ld), 0x7FC0, dtype=torch.int16, device="cuda")
    d_attn = torch.full((3, ld), np.nan, dtype=torch.float32, device="cuda")
    B.cr_gat_attention_bwd(bs, 0, par, z_dev, ld, el, stat, dev_bf16(torch, d_out), ld_dout, out_b if relu else None, lr, wd, dz, ws, d_attn)
    torch.cuda.synchronize()
    got_dz = bf16_tensor_to_float(dz)
    assert_close(got_dz[:blk.n_src, :HD], want_dz, RTOL_BF16, "gat dz")
    assert np.all(got_dz[:blk.n_src, HD:] == 0)
    ga = d_attn.cpu().numpy()
    # the parameter gradients are sums over all rows: judge them against the magnitude of what was added up
    assert_close(ga[0, :HD], want_al, 1e-3, "d a_l")
    assert_close(ga[1, :HD], want_ar, 1e-3, "d a_r")
    assert_close(ga[2, :HD], want_b, 1e-4, "d bias", np.abs(g).sum(axis=0))
    new = par.attn.cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(new[0, :HD], a_l - lr * (ga[0, :HD].astype(np.float64) + wd * a_l), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(new[1, :HD], a_r - lr * (ga[1, :HD].astype(np.float64) + wd * a_r), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(new[2, :HD], bias - lr * ga[2, :HD].astype(np.float64), rtol=1e-6, atol=1e-7)
    assert np.all(new[:, HD:] == 0)


def test_gat_backward_is_bit_reproducible(tiny_workload):
    import torch
    from paper_2504_18082_amd import binding as B
    heads, D, ld = 4, 64, 256
    results = []
    for _ in range(2):
        rng, blk, z, a_l, a_r, bias, bs, par = _setup(torch, tiny_workload, heads, D, ld, 99)
        z_dev = dev_bf16(torch, z)
        el = torch.zeros((bs.cap_src, heads), dtype=torch.float32, device="cuda")
        er = torch.zeros((bs.cap_src, heads), dtype=torch.float32, device="cuda")
        stat = torch.zeros((bs.cap_dst, heads, 4), dtype=torch.float32, device="cuda")
        out_b = torch.zeros((bs.cap_dst, ld), dtype=torch.int16, device="cuda")
        B.cr_gat_attention_fwd(bs, 0, par, z_dev, ld, True, el, er, stat, None, out_b)
        d_out = bf16_exact(rng.standard_normal((blk.n_dst, ld)))
        ws = torch.empty(B.cr_gat_attention_bwd_workspace_bytes(bs.cap_dst, ld, heads), dtype=torch.uint8, device="cuda")
        dz = torch.zeros((bs.cap_src, ld), dtype=torch.int16, device="cuda")
        d_attn = torch.zeros((3, ld), dtype=torch.float32, device="cuda")
        B.cr_gat_attention_bwd(bs, 0, par, z_dev, ld, el, stat, dev_bf16(torch, d_out), ld, out_b, 0.1, 0.0, dz, ws, d_attn)
        torch.cuda.synchronize()
        results.append((dz.cpu().numpy().copy(), d_attn.cpu().numpy().copy(), par.attn.cpu().numpy().copy()))
    for a, b in zip(results[0], results[1]):
        np.testing.assert_array_equal(a, b)


def test_gat_train_steps_match_oracle(tiny_workload):
    """Three consecutive GAT training steps (sampling with a transposed input block, row gather, projection,
    attention, loss, backward through attention and projection, SGD on every parameter)."""
    import torch
    from paper_2504_18082_amd.trainer import Trainer
    from oracle_step import oracle_train_step_gat
    w, seed, epoch, p, lr, wd, heads = tiny_workload, 0, 3, 0.9, 0.05, 5e-4, 4
    cfg = w.cfg
    weights = synth.init_gat_weights(cfg, seed, heads)
    tr = Trainer(w, group_size=2, lr=lr, weight_decay=wd, seed=seed, weights=weights, model="gat", gat_heads=heads)
    tr.build_batches(oracle.COMM_RAND, 6, epoch)
    perm = oracle.build_batches(oracle.COMM_RAND, 6, seed, epoch, w.train_ids, w.comm, cfg.n_comm)
    params = [tuple(a.astype(np.float64) for a in t) for t in weights]
    pos = np.full(cfg.n_nodes, -1, dtype=np.int32)
    dW_out = [torch.zeros_like(l.W) for l in tr.layers]
    d_attn = [torch.zeros_like(gp.attn) for gp in tr.gat]
    done = 0
    while done < 3:
        n = min(2, 3 - done)
        tr.sample_group(done, n, p, epoch)
        for g in range(n):
            b = done + g
            print(f"gat step batch={b}", flush=True)
            W_before = [l.W.cpu().numpy() for l in tr.layers]
            attn_before = [tr.gat[l].attn.cpu().numpy() for l in range(tr.L)]
            tr.train_batch(g, dW_out, None, d_attn_out=d_attn)
            torch.cuda.synchronize()
            roots = perm[b * cfg.batch_size:(b + 1) * cfg.batch_size]
            ref = oracle_train_step_gat(w.graph, w.features, cfg.n_feat, w.labels, roots, cfg.fanouts, p, seed, epoch, b, params, heads,
                                        lr, wd, pos)
            hdrs = tr.headers()
            for l in range(tr.L):       # the sampled blocks, the transposed input block included
                assert tuple(hdrs[l][g][:3]) == (ref["blocks"][l].n_dst, ref["blocks"][l].n_src, ref["blocks"][l].nnz)
            assert abs(float(tr.loss.cpu()[0]) - ref["loss"]) <= 1e-3 * abs(ref["loss"])
            assert_close(tr.out[tr.L - 1].cpu().numpy()[:len(roots), :cfg.n_classes], ref["logits"], 2e-2, f"logits batch {b}")
            for l in range(tr.L):
                HD = tr.layers[l].F_out
                dW, d_al, d_ar, d_b = ref["grads"][l]
                assert_close(dW_out[l].cpu().numpy(), dW, 2e-2, f"dW layer {l} batch {b}")
                ga = d_attn[l].cpu().numpy()
                assert_close(ga[0, :HD], d_al, 2e-2, f"d a_l layer {l} batch {b}")
                assert_close(ga[1, :HD], d_ar, 2e-2, f"d a_r layer {l} batch {b}")
                assert_close(ga[2, :HD], d_b, 2e-2, f"d bias layer {l} batch {b}")
                assert_weight_step(tr.layers[l].W.cpu().numpy(), W_before[l], ref["params"][l][0], params[l][0], 2e-2, f"W change layer {l} batch {b}")
                new = tr.gat[l].attn.cpu().numpy()
                for k in range(3):
                    assert_weight_step(new[k, :HD], attn_before[l][k, :HD], ref["params"][l][1 + k], params[l][1 + k], 2e-2,
                                       f"attn[{k}] change layer {l} batch {b}")
            params = [(tr.layers[l].W.cpu().numpy().astype(np.float64),) +
                      tuple(tr.gat[l].attn.cpu().numpy()[k, :tr.layers[l].F_out].astype(np.float64) for k in range(3))
                      for l in range(tr.L)]
        done += n


def test_transposed_input_block_matches_oracle(tiny_workload):
    """CR_SAMPLE_TRANSPOSE_INPUT: the input-side block comes with its transpose, bit for bit the oracle's."""
    import torch
    from paper_2504_18082_amd.trainer import Trainer
    w, seed, epoch, p = tiny_workload, 5, 1, 0.9
    cfg = w.cfg
    tr = Trainer(w, group_size=2, seed=seed, model="gat")
    tr.build_batches(oracle.RAND, 1, epoch)
    perm = oracle.build_batches(oracle.RAND, 1, seed, epoch, w.train_ids, w.comm, cfg.n_comm)
    tr.sample_group(0, 2, p, epoch)
    torch.cuda.synchronize()
    for g in range(2):
        roots = perm[g * cfg.batch_size:(g + 1) * cfg.batch_size]
        blk = oracle.transpose_block(oracle.sample_blocks(w.graph, roots, cfg.fanouts, p, False, seed, epoch, g)[0])
        bs = tr.blocks[0]
        np.testing.assert_array_equal(bs.t_indptr[g, :blk.n_src + 1].cpu().numpy(), blk.t_indptr)
        np.testing.assert_array_equal(bs.t_indices[g, :blk.nnz].cpu().numpy(), blk.t_indices)


def test_gat_fit_on_tiny(tiny_workload):
    import torch
    from paper_2504_18082_amd.trainer import Trainer
    w = tiny_workload
    tr = Trainer(w, group_size=8, lr=0.1, seed=0, model="gat")
    val = torch.from_numpy(w.val_ids).cuda()
    loss0, acc0 = tr.evaluate(val, 0)
    hist = tr.fit(oracle.COMM_RAND, 6, 0.9, val, max_epochs=10, patience=6, lr_patience=3)
    print("gat val acc", [round(v, 4) for v in hist.val_acc], flush=True)
    assert min(hist.val_loss) < 0.8 * loss0 and max(hist.val_acc) > 3.0 / w.cfg.n_classes


def test_gat_forward_at_benchmark_size(arxiv_workload):
    """The GAT forward pass in the measured configuration (arxiv-like workload, groups of 16 mini-batches of 1024 roots,
    three layers, ~130 K distinct input nodes per batch), checked on sampled outputs: the neighbours chosen for a node
    depend on (seed, epoch, batch, layer, node) only, so the oracle can compute the logits of a few roots of the batch
    from their own three-hop trees."""
    import torch
    from paper_2504_18082_amd.trainer import Trainer
    from oracle_step import oracle_train_step_gat
    w, seed, epoch, p, heads, g = arxiv_workload, 0, 2, 0.5, 4, 9
    cfg = w.cfg
    weights = synth.init_gat_weights(cfg, seed, heads)
    tr = Trainer(w, group_size=16, lr=0.05, seed=seed, weights=weights, model="gat", gat_heads=heads)
    tr.build_batches(oracle.RAND, 1, epoch)
    perm = oracle.build_batches(oracle.RAND, 1, seed, epoch, w.train_ids, w.comm, cfg.n_comm)
    tr.sample_group(0, 16, p, epoch)
    print("gat forward at benchmark size", flush=True)
    tr.forward_batch(g)
    torch.cuda.synchronize()
    hdr = tr.headers()[0][g]
    assert hdr[3] == 0 and hdr[1] > 50_000                     # a full-size input frontier
    logits = tr.out[tr.L - 1].cpu().numpy()
    roots = perm[g * cfg.batch_size:(g + 1) * cfg.batch_size]
    assert np.array_equal(tr.blocks[tr.L - 1].src_ids[g, :len(roots)].cpu().numpy(), roots)
    params = [tuple(a.astype(np.float64) for a in t) for t in weights]
    pick = np.arange(0, len(roots), 128)
    ref = oracle_train_step_gat(w.graph, w.features, cfg.n_feat, w.labels, roots[pick], cfg.fanouts, p, seed, epoch, g, params, heads,
                                0.0, 0.0)
    assert_close(logits[pick, :cfg.n_classes], ref["logits"], 2e-2, "logits of sampled roots")
