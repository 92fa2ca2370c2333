"""Pins of the oracle's GCN propagation on sampled blocks (Section 6.4): the full-neighbourhood block equals the
textbook D~^-1/2 (A + I) D~^-1/2 H, the backward is the transpose, rows whose neighbours were all taken are exact,
and under uniform sampling the block estimate is unbiased."""
import numpy as np

import oracle
from paper_2504_18082_amd import synth


def small_graph(seed=0, n=300):
    cfg = synth.scaled(synth.CONFIGS["tiny"], n / 10_000)
    cfg.n_comm = 6
    return synth.make_workload(cfg, seed)


def dense_gcn_operator(indptr, indices):
    n = len(indptr) - 1
    A = np.zeros((n, n))
    rows = np.repeat(np.arange(n), np.diff(indptr))
    A[rows, indices] = 1.0
    A += np.eye(n)
    d = A.sum(axis=1)
    return A / np.sqrt(np.outer(d, d))


def test_full_neighbourhood_is_the_textbook_operator():
    w = small_graph()
    n = w.cfg.n_nodes
    deg = np.diff(w.indptr)
    roots = np.arange(n, dtype=np.int32)
    blk = oracle.sample_hop(w.graph, roots, int(deg.max()) + 1, 0.5, False, 1, 0, 0, 0)
    assert blk.n_src == n and blk.nnz == len(w.indices)          # every neighbour of every node was taken
    rng = np.random.default_rng(0)
    H = rng.standard_normal((n, 7)).astype(np.float32)
    want = dense_gcn_operator(w.indptr, w.indices) @ H.astype(np.float64)
    np.testing.assert_allclose(oracle.gcn_aggregate(blk, H, deg, indirect=True), want, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.gcn_aggregate(blk, H, deg, indirect=False), want, rtol=1e-12, atol=1e-12)  # local = global here


def test_backward_is_the_transpose():
    w = small_graph(1)
    deg = np.diff(w.indptr)
    roots = w.train_ids[:60]
    blk = oracle.sample_hop(w.graph, roots, 4, 0.9, False, 3, 1, 2, 1)
    rng = np.random.default_rng(1)
    H = rng.standard_normal((blk.n_src, 5))
    G = rng.standard_normal((blk.n_dst, 5))
    lhs = np.sum(oracle.gcn_aggregate(blk, H.astype(np.float32), deg, indirect=False) * G)
    rhs = np.sum(H.astype(np.float32).astype(np.float64) * oracle.gcn_aggregate_bwd(blk, G, deg))
    assert abs(lhs - rhs) <= 1e-10 * (abs(lhs) + 1.0)
    # and, being linear, the forward pass of a one-hot input is a column of the same operator
    e = np.zeros((blk.n_src, 1), dtype=np.float32)
    e[blk.n_dst + 3 if blk.n_src > blk.n_dst + 3 else 0] = 1.0
    col = oracle.gcn_aggregate(blk, e, deg, indirect=False)[:, 0]
    k = int(np.argmax(e[:, 0]))
    one = np.zeros((blk.n_dst, blk.n_dst))
    np.fill_diagonal(one, 1.0)
    np.testing.assert_allclose(oracle.gcn_aggregate_bwd(blk, one, deg)[k], col, rtol=1e-12, atol=1e-15)


def test_rows_with_all_neighbours_are_exact_and_sampling_is_unbiased():
    w = small_graph(2)
    n = w.cfg.n_nodes
    deg = np.diff(w.indptr)
    rng = np.random.default_rng(2)
    H = rng.standard_normal((n, 3)).astype(np.float32)
    exact = dense_gcn_operator(w.indptr, w.indices) @ H.astype(np.float64)
    roots = np.arange(0, n, 3, dtype=np.int32)
    fanout = 3
    mean = np.zeros((len(roots), 3))
    trials = 400
    for t in range(trials):
        blk = oracle.sample_hop(w.graph, roots, fanout, 0.5, False, 7, t, 0, 0)
        out = oracle.gcn_aggregate(blk, H, deg, indirect=True)
        small = deg[roots] <= fanout
        np.testing.assert_allclose(out[small], exact[roots][small], rtol=1e-12, atol=1e-12)
        mean += out / trials
    # Monte-Carlo mean against the exact rows: the estimator's noise shrinks like 1/sqrt(trials)
    err = np.abs(mean - exact[roots]).max()
    spread = np.abs(exact[roots]).max()
    assert err < 0.15 * spread
    # a wrong scale (forgetting deg/|N_s|) would be off by far more on the high-degree rows
    big = deg[roots] >= 3 * fanout
    assert big.any()
