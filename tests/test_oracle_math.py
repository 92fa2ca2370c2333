"""Pins for the oracle's aggregation / projection / loss / backward (Eq. 1 in GraphSAGE-mean form)."""
import numpy as np
import scipy.sparse as sp

import oracle
from paper_2504_18082_amd import synth


def dense_mean_operator(blk):
    A = np.zeros((blk.n_dst, blk.n_src))
    for v in range(blk.n_dst):
        cols = blk.indices[blk.indptr[v]:blk.indptr[v + 1]]
        for c in cols:
            A[v, c] += 1.0 / len(cols)
    return A


def small_block(w, n_roots=96, fanout=5, layer=1):
    return oracle.transpose_block(oracle.sample_hop(w.graph, w.train_ids[:n_roots], fanout, 0.9, False, 0, 0, 0, layer))


def test_gather_mean_equals_dense_operator(tiny_workload):
    w = tiny_workload
    blk = small_block(w)
    rng = np.random.default_rng(0)
    H = rng.standard_normal((blk.n_src, 24)).astype(np.float32)
    agg, self_rows = oracle.gather_mean(blk, H, indirect=False, want_self=True)
    np.testing.assert_allclose(agg, dense_mean_operator(blk) @ H.astype(np.float64), rtol=1e-13, atol=1e-13)
    np.testing.assert_array_equal(self_rows, H[:blk.n_dst].astype(np.float64))
    # indirect mode reads the feature table through the frontier ids
    agg0, self0 = oracle.gather_mean(blk, w.features, indirect=True, F=w.cfg.n_feat, want_self=True)
    X = w.features[blk.src_ids, :w.cfg.n_feat].astype(np.float64)
    np.testing.assert_allclose(agg0, dense_mean_operator(blk) @ X, rtol=1e-13, atol=1e-13)
    np.testing.assert_array_equal(self0, X[:blk.n_dst])


def test_gather_mean_bf16_table(tiny_workload):
    w = tiny_workload
    blk = small_block(w)
    bits = synth.float_to_bf16_bits(w.features)
    agg = oracle.gather_mean(blk, bits, indirect=True, F=w.cfg.n_feat)
    X = synth.bf16_bits_to_float(bits)[blk.src_ids, :w.cfg.n_feat].astype(np.float64)
    np.testing.assert_allclose(agg, dense_mean_operator(blk) @ X, rtol=1e-13, atol=1e-13)
    # storage conversion agrees with the oracle's own operand rounding
    x = np.random.default_rng(3).standard_normal(4096).astype(np.float32) * 37.0
    np.testing.assert_array_equal(synth.bf16_bits_to_float(synth.float_to_bf16_bits(x)).astype(np.float64), oracle.round_bf16(x))
    # known roundings: ties to even on the 8-bit mantissa
    np.testing.assert_array_equal(oracle.round_bf16([1.0, 1.00390625, 1.01171875, -3.0e-40 * 0 + 257.0, 258.0 + 1.0]),
                                  [1.0, 1.0, 1.015625, 256.0, 260.0])


def test_full_fanout_all_nodes_equals_normalised_adjacency_spmm():
    # Eq. 1 with A' = D^-1 A: fanout >= max degree and every node a root
    cfg = synth.scaled(synth.CONFIGS["tiny"], 0.05, "tiny_small")
    w = synth.make_workload(cfg, seed=1)
    N = cfg.n_nodes
    deg = np.diff(w.indptr)
    blk = oracle.sample_hop(w.graph, np.arange(N, dtype=np.int32), int(deg.max()) + 3, 0.9, False, 0, 0, 0, 0)
    assert blk.n_src == N and np.array_equal(blk.src_ids, np.arange(N))
    A = sp.csr_matrix((np.ones(len(w.indices)), w.indices, w.indptr), shape=(N, N))
    Dinv = sp.diags(1.0 / np.maximum(deg, 1))
    X = w.features[:, :cfg.n_feat].astype(np.float64)
    agg = oracle.gather_mean(blk, w.features, indirect=True, F=cfg.n_feat)
    np.testing.assert_allclose(agg, (Dinv @ A) @ X, rtol=1e-12, atol=1e-12)
    assert np.all(agg[deg == 0] == 0.0)


def test_gather_backward_is_the_transpose(tiny_workload):
    w = tiny_workload
    blk = small_block(w)
    rng = np.random.default_rng(1)
    d_agg = rng.standard_normal((blk.n_dst, 16))
    d_self = rng.standard_normal((blk.n_dst, 16))
    A = dense_mean_operator(blk)
    want = A.T @ d_agg
    np.testing.assert_allclose(oracle.gather_mean_bwd(blk, d_agg), want, rtol=1e-12, atol=1e-12)
    want[:blk.n_dst] += d_self
    np.testing.assert_allclose(oracle.gather_mean_bwd(blk, d_agg, d_self), want, rtol=1e-12, atol=1e-12)
    # adjoint identity <A x, y> = <x, A^T y>
    x = rng.standard_normal((blk.n_src, 16)).astype(np.float32)
    lhs = np.sum(oracle.gather_mean(blk, x, indirect=False) * d_agg)
    rhs = np.sum(x.astype(np.float64) * oracle.gather_mean_bwd(blk, d_agg))
    assert abs(lhs - rhs) < 1e-10 * max(1.0, abs(lhs))


def test_isolated_row_aggregates_to_zero():
    indptr = np.array([0, 0, 2, 3], dtype=np.int64)          # node 0 has no neighbours
    indices = np.array([0, 2, 1], dtype=np.int32)
    comm = np.zeros(3, dtype=np.int32)
    blk = oracle.sample_hop((indptr, indices, comm), [0, 1], 3, 0.5, False, 0, 0, 0, 0)
    H = np.arange(12, dtype=np.float32).reshape(3, 4) + 1
    agg = oracle.gather_mean(blk, H, indirect=True)
    assert np.all(agg[0] == 0.0) and np.allclose(agg[1], (H[0] + H[2]) / 2)
    d = oracle.gather_mean_bwd(blk, np.ones((2, 4)))
    assert np.allclose(d[blk.src_ids.tolist().index(1)], 0.0)      # node 1 feeds no one
    assert np.allclose(d[blk.src_ids.tolist().index(2)], 0.5)


def test_linear_forward_matches_numpy():
    rng = np.random.default_rng(2)
    M, Fi, Fo = 37, 19, 11
    hs, ag = rng.standard_normal((M, Fi)), rng.standard_normal((M, Fi))
    W, b = rng.standard_normal((2 * Fi, Fo)), rng.standard_normal(Fo)
    z = np.concatenate([hs, ag], axis=1) @ W + b
    np.testing.assert_allclose(oracle.sage_linear_fwd(hs, ag, W, b, False, False), z, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.sage_linear_fwd(hs, ag, W, b, True, False), np.maximum(z, 0), rtol=1e-12, atol=1e-12)
    r = oracle.round_bf16
    zr = np.concatenate([r(hs), r(ag)], axis=1) @ r(W) + b
    np.testing.assert_allclose(oracle.sage_linear_fwd(hs, ag, W, b, False, True), zr, rtol=1e-12, atol=1e-12)
    assert np.abs(zr - z).max() > 1e-4          # rounding really happened


def test_linear_backward_matches_numpy():
    rng = np.random.default_rng(3)
    M, Fi, Fo = 29, 13, 7
    hs, ag = rng.standard_normal((M, Fi)), rng.standard_normal((M, Fi))
    W, b = rng.standard_normal((2 * Fi, Fo)), rng.standard_normal(Fo)
    out = oracle.sage_linear_fwd(hs, ag, W, b, True, False)
    d_out = rng.standard_normal((M, Fo))
    dW, db, d_self, d_agg = oracle.sage_linear_bwd(hs, ag, W, out, d_out, True, False)
    dz = d_out * (out > 0)
    A = np.concatenate([hs, ag], axis=1)
    np.testing.assert_allclose(dW, A.T @ dz, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(db, dz.sum(0), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(d_self, dz @ W[:Fi].T, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(d_agg, dz @ W[Fi:].T, rtol=1e-12, atol=1e-12)


def test_softmax_xent_closed_forms():
    n, Cn = 9, 7
    labels = np.arange(n, dtype=np.int32) % Cn
    loss, d = oracle.softmax_xent(np.full((n, Cn), 3.25), labels)
    assert abs(loss - np.log(Cn)) < 1e-14
    rng = np.random.default_rng(4)
    z = rng.standard_normal((n, Cn)) * 3
    loss, d = oracle.softmax_xent(z, labels)
    np.testing.assert_allclose(d.sum(axis=1), 0.0, atol=1e-15)
    p = np.exp(z - z.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    assert abs(loss - (-np.log(p[np.arange(n), labels]).mean())) < 1e-13
    # padded logits: columns >= n_classes are ignored and get zero gradient
    zp = np.concatenate([z, rng.standard_normal((n, 3)) + 50], axis=1)
    loss_p, dp = oracle.softmax_xent(zp, labels, n_classes=Cn)
    assert abs(loss_p - loss) < 1e-14 and np.all(dp[:, Cn:] == 0) and np.allclose(dp[:, :Cn], d)


def two_layer_loss(blocks, X, labels, params):
    """Forward of a 2-layer SAGE-mean net with the oracle's pieces (no operand rounding)."""
    (W0, b0), (W1, b1) = params
    agg0, self0 = oracle.gather_mean(blocks[0], X, indirect=True, want_self=True)
    h1 = oracle.sage_linear_fwd(self0, agg0, W0, b0, True, False)
    # the loss below needs double-precision hidden activations: aggregate them directly
    A1 = dense_mean_operator(blocks[1])
    agg1 = A1 @ h1
    logits = oracle.sage_linear_fwd(h1[:blocks[1].n_dst], agg1, W1, b1, False, False)
    loss, dlogits = oracle.softmax_xent(logits, labels)
    return loss, (agg0, self0, h1, agg1, logits, dlogits)


def test_gradients_match_finite_differences(tiny_workload):
    w = tiny_workload
    roots = w.train_ids[:24]
    blocks = oracle.sample_blocks(w.graph, roots, [4, 3], 0.9, False, 0, 0, 0)
    Fin, Hd, Cn = 6, 5, 4
    X = np.ascontiguousarray(w.features[:, :Fin])
    labels = (w.labels[roots] % Cn).astype(np.int32)
    rng = np.random.default_rng(5)
    params = [(rng.standard_normal((2 * Fin, Hd)) * 0.5, rng.standard_normal(Hd) * 0.1),
              (rng.standard_normal((2 * Hd, Cn)) * 0.5, rng.standard_normal(Cn) * 0.1)]
    loss, (agg0, self0, h1, agg1, logits, dlogits) = two_layer_loss(blocks, X, labels, params)
    # analytic backward, all from the oracle
    dW1, db1, d_self1, d_agg1 = oracle.sage_linear_bwd(h1[:blocks[1].n_dst], agg1, params[1][0], logits, dlogits, False, False)
    d_h1 = oracle.gather_mean_bwd(blocks[1], d_agg1, d_self1)
    dW0, db0, _, _ = oracle.sage_linear_bwd(self0, agg0, params[0][0], h1, d_h1, True, False, need_dx=False)
    eps = 1e-6
    for (li, which, grad) in ((0, 0, dW0), (0, 1, db0), (1, 0, dW1), (1, 1, db1)):
        arr = params[li][which]
        flat = arr.reshape(-1)
        for idx in rng.choice(flat.size, size=min(flat.size, 12), replace=False):
            old = flat[idx]
            flat[idx] = old + eps
            lp, _ = two_layer_loss(blocks, X, labels, params)
            flat[idx] = old - eps
            lm, _ = two_layer_loss(blocks, X, labels, params)
            flat[idx] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad.reshape(-1)[idx]) < 1e-6 * max(1.0, abs(fd)), (li, which, idx, fd, grad.reshape(-1)[idx])
    # one small SGD step without decay lowers the loss
    newp = []
    for (W, b), (dW, db) in zip(params, ((dW0, db0), (dW1, db1))):
        newp.append(oracle.sgd_step(W, dW, b, db, 1e-2, 0.0))
    loss2, _ = two_layer_loss(blocks, X, labels, newp)
    assert loss2 < loss
    # weight decay shrinks weights, leaves the bias alone
    W, b = oracle.sgd_step(np.ones((2, 2)), np.zeros((2, 2)), np.ones(2), np.zeros(2), 0.1, 0.5)
    assert np.allclose(W, 0.95) and np.allclose(b, 1.0)


def test_count_correct_matches_numpy_argmax():
    rng = np.random.default_rng(6)
    z = rng.standard_normal((200, 13))
    z[5, 3] = z[5, 7] = 9.0                       # a tie: the lower index wins, as numpy's argmax does
    labels = rng.integers(0, 13, size=200).astype(np.int32)
    labels[5] = 3
    assert oracle.count_correct(z, labels) == int((np.argmax(z, axis=1) == labels).sum())
    zp = np.concatenate([z, np.full((200, 3), 50.0)], axis=1)            # padded columns are ignored
    assert oracle.count_correct(zp, labels, n_classes=13) == oracle.count_correct(z, labels)
    assert oracle.count_correct(np.eye(4), np.arange(4, dtype=np.int32)) == 4
