"""Pins for the oracle's root-node partitioning (Algorithm 1 Step-1, Section 4.1, Table 1)."""
import itertools
from collections import Counter

import numpy as np
from scipy import stats

import oracle
from oracle import COMM_RAND, NORAND, RAND


def runs(seq):
    """Number of maximal runs of equal values."""
    seq = np.asarray(seq)
    return int(1 + np.count_nonzero(seq[1:] != seq[:-1])) if seq.size else 0


def test_every_policy_gives_a_permutation(tiny_workload):
    w = tiny_workload
    for policy, mix in ((NORAND, 1), (RAND, 1), (COMM_RAND, 1), (COMM_RAND, 6), (COMM_RAND, 25), (COMM_RAND, 50)):
        perm = oracle.build_batches(policy, mix, 0, 3, w.train_ids, w.comm, w.cfg.n_comm)
        assert np.array_equal(np.sort(perm), w.train_ids)      # every training node in exactly one batch


def test_norand_is_static_identity(tiny_workload):
    w = tiny_workload
    for epoch in (0, 1, 9):
        assert np.array_equal(oracle.build_batches(NORAND, 1, 5, epoch, w.train_ids, w.comm, w.cfg.n_comm), w.train_ids)


def test_rand_equals_plain_sort_by_key_and_full_mix(tiny_workload):
    w = tiny_workload
    seed, epoch = 11, 4
    keys = [oracle.shuffle_key(seed, epoch, 1, int(v)) for v in w.train_ids]
    expect = np.array([v for _, v in sorted(zip(keys, w.train_ids.tolist()))], dtype=np.int32)
    got = oracle.build_batches(RAND, 1, seed, epoch, w.train_ids, w.comm, w.cfg.n_comm)
    assert np.array_equal(got, expect)
    # mixing all communities is the fully random end of the knob
    for mix in (w.cfg.n_comm, w.cfg.n_comm + 7):
        assert np.array_equal(oracle.build_batches(COMM_RAND, mix, seed, epoch, w.train_ids, w.comm, w.cfg.n_comm), got)


def test_mix0_keeps_communities_contiguous(tiny_workload):
    w = tiny_workload
    perm = oracle.build_batches(COMM_RAND, 1, 2, 1, w.train_ids, w.comm, w.cfg.n_comm)
    c_train = len(np.unique(w.comm[w.train_ids]))
    assert runs(w.comm[perm]) == c_train
    # community order = communities sorted by their own key
    order = [int(c) for c in w.comm[perm][np.r_[True, w.comm[perm][1:] != w.comm[perm][:-1]]]]
    keyed = sorted((oracle.shuffle_key(2, 1, 0, c), c) for c in np.unique(w.comm[w.train_ids]).tolist())
    assert order == [c for _, c in keyed]
    # inside a community: nodes sorted by their own key
    first = order[0]
    members = perm[w.comm[perm] == first].tolist()
    assert members == [v for _, v in sorted((oracle.shuffle_key(2, 1, 1, v), v) for v in members)]


def test_super_blocks_are_unions_of_consecutive_shuffled_communities(tiny_workload):
    w = tiny_workload
    seed, epoch, mix = 9, 6, 7
    perm = oracle.build_batches(COMM_RAND, mix, seed, epoch, w.train_ids, w.comm, w.cfg.n_comm)
    present = np.unique(w.comm[w.train_ids]).tolist()
    pi = [c for _, c in sorted((oracle.shuffle_key(seed, epoch, 0, c), c) for c in present)]
    block_of = {c: r // mix for r, c in enumerate(pi)}
    blocks = np.array([block_of[int(c)] for c in w.comm[perm]])
    n_blocks = -(-len(present) // mix)
    assert runs(blocks) == n_blocks and np.all(np.diff(blocks) >= 0)
    for j in range(n_blocks):
        nodes = perm[blocks == j]
        want = w.train_ids[np.isin(w.comm[w.train_ids], pi[j * mix:(j + 1) * mix])]
        assert np.array_equal(np.sort(nodes), want)
        assert nodes.tolist() == [v for _, v in sorted((oracle.shuffle_key(seed, epoch, 1, int(v)), int(v)) for v in nodes)]


def test_determinism_and_epoch_sensitivity(tiny_workload):
    w = tiny_workload
    a = oracle.build_batches(COMM_RAND, 3, 1, 5, w.train_ids, w.comm, w.cfg.n_comm)
    b = oracle.build_batches(COMM_RAND, 3, 1, 5, w.train_ids, w.comm, w.cfg.n_comm)
    c = oracle.build_batches(COMM_RAND, 3, 1, 6, w.train_ids, w.comm, w.cfg.n_comm)
    d = oracle.build_batches(COMM_RAND, 3, 2, 5, w.train_ids, w.comm, w.cfg.n_comm)
    assert np.array_equal(a, b) and not np.array_equal(a, c) and not np.array_equal(a, d)


def test_absent_communities_and_unordered_membership():
    # community ids need not be contiguous in node order; communities without training nodes are ignored
    comm = np.array([3, 0, 3, 5, 0, 5, 3, 1, 1, 0], dtype=np.int32)
    train = np.array([0, 1, 2, 3, 4, 5, 6, 9], dtype=np.int32)        # community 1, 2, 4 absent
    perm = oracle.build_batches(COMM_RAND, 1, 3, 0, train, comm, 6)
    assert sorted(perm.tolist()) == train.tolist()
    assert runs(comm[perm]) == 3
    perm2 = oracle.build_batches(COMM_RAND, 2, 3, 0, train, comm, 6)
    pi = [c for _, c in sorted((oracle.shuffle_key(3, 0, 0, c), c) for c in (0, 3, 5))]
    first_block = set(np.nonzero(np.isin(comm, pi[:2]))[0].tolist()) & set(train.tolist())
    assert set(perm2[:len(first_block)].tolist()) == first_block


def test_exact_distribution_brute_force():
    # 3 communities x 2 nodes, no mixing: 3! * (2!)^3 = 48 equally likely orders
    comm = np.array([0, 0, 1, 1, 2, 2], dtype=np.int32)
    train = np.arange(6, dtype=np.int32)
    valid = set()
    for corder in itertools.permutations(range(3)):
        for flips in itertools.product((0, 1), repeat=3):
            seq = []
            for c in corder:
                pair = [2 * c, 2 * c + 1]
                seq += pair[::-1] if flips[c] else pair
            valid.add(tuple(seq))
    assert len(valid) == 48
    n_epochs = 24000
    counts = Counter(tuple(oracle.build_batches(COMM_RAND, 1, 123, e, train, comm, 3).tolist()) for e in range(n_epochs))
    assert set(counts) == valid
    chi2, pval = stats.chisquare([counts[k] for k in sorted(valid)])
    assert pval > 1e-4, (chi2, pval)
    # mixing two of three: the lone community's pair stays together at one end, the other four mix freely
    counts = Counter(tuple(oracle.build_batches(COMM_RAND, 2, 123, e, train, comm, 3).tolist()) for e in range(n_epochs))
    # outcomes: choose the ordered community triple (6), 4! orders of the super-block, 2 of the lone pair
    assert len(counts) == 3 * 24 * 2 and all(
        (seq[4] // 2 == seq[5] // 2) and len({x // 2 for x in seq[:4]}) == 2 for seq in counts)
    chi2, pval = stats.chisquare(list(counts.values()))
    assert pval > 1e-4, (chi2, pval)
    # RAND: all 6! orders, uniformly
    counts = Counter(tuple(oracle.build_batches(RAND, 1, 123, e, train, comm, 3).tolist()) for e in range(n_epochs))
    assert len(counts) == 720
    chi2, pval = stats.chisquare(list(counts.values()))
    assert pval > 1e-4, (chi2, pval)


def test_community_diversity_per_batch_grows_with_mixing(tiny_workload):
    # Section 4.1: more mixed communities = more randomisation, less community bias
    w = tiny_workload
    B = w.cfg.batch_size

    def mean_comms(policy, mix):
        tot = []
        for epoch in range(3):
            perm = oracle.build_batches(policy, mix, 0, epoch, w.train_ids, w.comm, w.cfg.n_comm)
            tot += [len(np.unique(w.comm[perm[s:s + B]])) for s in range(0, len(perm), B)]
        return float(np.mean(tot))

    seq = [mean_comms(NORAND, 1), mean_comms(COMM_RAND, 1), mean_comms(COMM_RAND, 6), mean_comms(COMM_RAND, 12),
           mean_comms(COMM_RAND, 25), mean_comms(RAND, 1)]
    assert seq[0] <= seq[1] + 1e-9
    assert all(seq[i] < seq[i + 1] for i in range(1, len(seq) - 1)), seq


def test_rejects_bad_arguments(tiny_workload):
    import pytest
    w = tiny_workload
    with pytest.raises(ValueError):
        oracle.build_batches(COMM_RAND, 0, 0, 0, w.train_ids, w.comm, w.cfg.n_comm)
    with pytest.raises(ValueError):
        oracle.build_batches(7, 1, 0, 0, w.train_ids, w.comm, w.cfg.n_comm)
