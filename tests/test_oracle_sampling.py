"""Pins for the oracle's biased neighbourhood sampling (Algorithm 1 Step-2, Section 4.2)."""
import itertools
from collections import Counter

import numpy as np
from scipy import stats

import oracle
from paper_2504_18082_amd import synth


def chosen_neighbours(graph, blk, row):
    return blk.src_ids[blk.indices[blk.indptr[row]:blk.indptr[row + 1]]]


def test_rows_are_valid_distinct_neighbours_with_the_right_count(tiny_workload):
    w = tiny_workload
    roots = w.train_ids[:300]
    for p in (0.5, 0.9, 1.0):
        blk = oracle.sample_hop(w.graph, roots, 5, p, False, 0, 1, 2, 1)
        for i, v in enumerate(roots):
            adj = w.indices[w.indptr[v]:w.indptr[v + 1]]
            got = chosen_neighbours(w.graph, blk, i)
            assert len(got) == min(5, len(adj))
            assert len(set(got.tolist())) == len(got) and set(got.tolist()) <= set(adj.tolist())
            slots = blk.slots[blk.indptr[i]:blk.indptr[i + 1]]
            assert np.all(np.diff(slots) > 0) and np.array_equal(adj[slots], got)   # emitted in slot order


def test_low_degree_rows_keep_their_whole_adjacency(tiny_workload):
    w = tiny_workload
    deg = np.diff(w.indptr)
    rows = np.nonzero((deg > 0) & (deg <= 4))[0][:50].astype(np.int32)
    for p in (0.5, 0.9, 1.0):
        blk = oracle.sample_hop(w.graph, rows, 4, p, False, 3, 0, 0, 0)
        for i, v in enumerate(rows):
            assert np.array_equal(chosen_neighbours(w.graph, blk, i), w.indices[w.indptr[v]:w.indptr[v + 1]])


def test_selection_is_the_k_smallest_keys():
    g = synth.star_graph(6, 6)
    for p in (0.5, 0.9, 1.0):
        q = oracle.q_intra(p)
        blk = oracle.sample_hop(g, [0], 4, p, False, 5, 2, 7, 1)
        keys = []
        for j in range(12):
            r = oracle.slot_word(5, 2, 7, 1, 0, j)
            keys.append((oracle.slot_key(r, g[2][g[1][j]] == 0, q), j))
        want = sorted(j for _, j in sorted(keys)[:4])
        assert blk.slots.tolist() == want


def test_p_half_is_uniform_without_replacement():
    # 5-neighbour star, fanout 2: all C(5,2) = 10 subsets equally likely
    g = synth.star_graph(3, 2)
    n = 20000
    counts = Counter(tuple(oracle.sample_hop(g, [0], 2, 0.5, False, 77, e, 0, 0).slots.tolist()) for e in range(n))
    assert set(counts) == set(itertools.combinations(range(5), 2))
    chi2, pval = stats.chisquare(list(counts.values()))
    assert pval > 1e-4, (chi2, pval)


def test_weighted_sampling_matches_successive_sampling_closed_form():
    # 3 intra + 3 inter neighbours at p = 0.9: weights 9:1 (Section 5, "9 times higher")
    g = synth.star_graph(3, 3)
    wts = np.array([0.9] * 3 + [0.1] * 3)
    n = 40000
    # fanout 1: P(i) = w_i / W
    c1 = Counter(int(oracle.sample_hop(g, [0], 1, 0.9, False, 5, e, 0, 0).slots[0]) for e in range(n))
    chi2, pval = stats.chisquare([c1[i] for i in range(6)], f_exp=n * wts / wts.sum())
    assert pval > 1e-4, (chi2, pval)
    # fanout 2: P({i,j}) = w_i/W * w_j/(W-w_i) + w_j/W * w_i/(W-w_j)
    W = wts.sum()
    pairs = list(itertools.combinations(range(6), 2))
    prob = np.array([wts[i] / W * wts[j] / (W - wts[i]) + wts[j] / W * wts[i] / (W - wts[j]) for i, j in pairs])
    assert abs(prob.sum() - 1.0) < 1e-12
    c2 = Counter(tuple(oracle.sample_hop(g, [0], 2, 0.9, False, 6, e, 1, 1).slots.tolist()) for e in range(n))
    chi2, pval = stats.chisquare([c2[pr] for pr in pairs], f_exp=n * prob)
    assert pval > 1e-4, (chi2, pval)


def test_full_bias_takes_intra_first_and_strict_never_takes_inter(tiny_workload):
    w = tiny_workload
    roots = w.train_ids[:400]
    fill = oracle.sample_hop(w.graph, roots, 5, 1.0, False, 0, 0, 0, 1)
    strict = oracle.sample_hop(w.graph, roots, 5, 1.0, True, 0, 0, 0, 1)
    saw_short = False
    for i, v in enumerate(roots):
        adj = w.indices[w.indptr[v]:w.indptr[v + 1]]
        n_intra = int((w.comm[adj] == w.comm[v]).sum())
        a = chosen_neighbours(w.graph, fill, i)
        b = chosen_neighbours(w.graph, strict, i)
        assert len(a) == min(5, len(adj))
        assert int((w.comm[a] == w.comm[v]).sum()) == min(5, n_intra)
        assert len(b) == min(5, n_intra) and np.all(w.comm[b] == w.comm[v])
        assert set(b.tolist()) <= set(a.tolist())
        saw_short |= len(b) < len(a)
    assert saw_short


def test_frontier_is_dst_prefix_plus_first_appearance_order(tiny_workload):
    w = tiny_workload
    roots = w.train_ids[100:356]
    blk = oracle.sample_hop(w.graph, roots, 10, 0.9, False, 4, 2, 1, 0)
    assert np.array_equal(blk.src_ids[:len(roots)], roots)
    assert len(set(blk.src_ids.tolist())) == blk.n_src
    # independent re-derivation from the chosen slots
    seen = {int(v): i for i, v in enumerate(roots)}
    order = list(roots)
    for i, v in enumerate(roots):
        for s in blk.slots[blk.indptr[i]:blk.indptr[i + 1]]:
            u = int(w.indices[w.indptr[v] + s])
            if u not in seen:
                seen[u] = len(order)
                order.append(u)
    assert np.array_equal(blk.src_ids, np.array(order, dtype=np.int32))
    e = 0
    for i, v in enumerate(roots):
        for s in blk.slots[blk.indptr[i]:blk.indptr[i + 1]]:
            assert blk.src_ids[blk.indices[e]] == w.indices[w.indptr[v] + s]
            e += 1
    assert e == blk.nnz == blk.indptr[-1]


def test_multi_hop_chain_and_transpose(tiny_workload):
    w = tiny_workload
    roots = w.train_ids[:256]
    blocks = oracle.sample_blocks(w.graph, roots, [10, 5], 0.9, False, 0, 0, 0)
    assert np.array_equal(blocks[1].src_ids[:256], roots)
    assert blocks[0].n_dst == blocks[1].n_src and np.array_equal(blocks[0].src_ids[:blocks[0].n_dst], blocks[1].src_ids)
    assert blocks[1].indptr[-1] <= 256 * 5 and blocks[0].indptr[-1] <= blocks[0].n_dst * 10
    b = blocks[1]
    dense = np.zeros((b.n_dst, b.n_src), dtype=np.int32)
    for v in range(b.n_dst):
        dense[v, b.indices[b.indptr[v]:b.indptr[v + 1]]] += 1
    dense_t = np.zeros((b.n_src, b.n_dst), dtype=np.int32)
    for s in range(b.n_src):
        cols = b.t_indices[b.t_indptr[s]:b.t_indptr[s + 1]]
        assert np.all(np.diff(cols) >= 0)
        np.add.at(dense_t[s], cols, 1)
    assert np.array_equal(dense.T, dense_t)


def test_determinism_and_counter_sensitivity(tiny_workload):
    w = tiny_workload
    roots = w.train_ids[:128]
    base = oracle.sample_hop(w.graph, roots, 5, 0.9, False, 1, 2, 3, 1)
    again = oracle.sample_hop(w.graph, roots, 5, 0.9, False, 1, 2, 3, 1)
    assert np.array_equal(base.indices, again.indices) and np.array_equal(base.src_ids, again.src_ids)
    for args in ((2, 2, 3, 1), (1, 3, 3, 1), (1, 2, 4, 1), (1, 2, 3, 0)):
        other = oracle.sample_hop(w.graph, roots, 5, 0.9, False, *args)
        assert not np.array_equal(base.slots, other.slots)


def test_input_footprint_shrinks_with_more_bias(tiny_workload):
    # Section 6.1.1 discussion: more community bias (either knob) = fewer input nodes per batch
    w = tiny_workload
    B = w.cfg.batch_size
    pos = np.full(w.cfg.n_nodes, -1, dtype=np.int32)

    def mean_inputs(policy, mix, p):
        tot = []
        for epoch in range(2):
            perm = oracle.build_batches(policy, mix, 0, epoch, w.train_ids, w.comm, w.cfg.n_comm)
            for b, s in enumerate(range(0, len(perm), B)):
                blocks = oracle.sample_blocks(w.graph, perm[s:s + B], w.cfg.fanouts, p, False, 0, epoch, b, pos, transpose=False)
                tot.append(blocks[0].n_src)
        return float(np.mean(tot))

    by_p = [mean_inputs(oracle.RAND, 1, p) for p in (0.5, 0.9, 1.0)]
    assert by_p[0] > by_p[1] > by_p[2], by_p
    by_policy = [mean_inputs(oracle.RAND, 1, 1.0), mean_inputs(oracle.COMM_RAND, 12, 1.0),
                 mean_inputs(oracle.COMM_RAND, 1, 1.0), mean_inputs(oracle.NORAND, 1, 1.0)]
    assert by_policy[0] > by_policy[1] > by_policy[2] and by_policy[2] >= by_policy[3] * 0.98, by_policy


def test_rejects_bad_arguments(tiny_workload):
    import pytest
    w = tiny_workload
    with pytest.raises(ValueError):
        oracle.sample_hop(w.graph, [0], 0, 0.5, False, 0, 0, 0, 0)
    with pytest.raises(ValueError):
        oracle.sample_hop(w.graph, [0], 2, 0.3, False, 0, 0, 0, 0)
