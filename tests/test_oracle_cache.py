"""Pins of the oracle's software-cache model (Section 6.5, software-managed caches): textbook LRU as the
one-set / one-node-per-batch special case, closed forms for an unbounded cache and for the cyclic pattern, and
the batch-synchronous rules (a row touched in a batch is never evicted in it; overflow misses are not cached)."""
from collections import OrderedDict

import numpy as np

import oracle


def textbook_lru(trace, capacity):
    """Classic LRU over single accesses; returns the miss count."""
    lru, misses = OrderedDict(), 0
    for x in trace:
        if x in lru:
            lru.move_to_end(x)
        else:
            misses += 1
            if len(lru) >= capacity:
                lru.popitem(last=False)
            lru[x] = True
    return misses


def test_single_set_single_access_is_textbook_lru():
    rng = np.random.default_rng(0)
    for ways, universe in ((4, 7), (8, 12), (16, 40)):
        trace = rng.integers(0, universe, size=3000)
        model = oracle.FeatureCacheModel(1, ways)
        for t, x in enumerate(trace):
            model.fetch([int(x)], t)
        assert model.misses == textbook_lru(trace.tolist(), ways)
        assert model.queries == len(trace)


def test_sets_are_independent_lru_caches():
    # a 4-set cache over ids equals four textbook LRUs over the residue classes
    rng = np.random.default_rng(1)
    trace = rng.integers(0, 64, size=4000)
    model = oracle.FeatureCacheModel(4, 3)
    for t, x in enumerate(trace):
        model.fetch([int(x)], t)
    want = sum(textbook_lru([x for x in trace.tolist() if x % 4 == r], 3) for r in range(4))
    assert model.misses == want


def test_unbounded_cache_misses_are_first_touches():
    rng = np.random.default_rng(2)
    model = oracle.FeatureCacheModel(16, 64)               # 1024 rows for a universe of 500 ids
    seen = set()
    for t in range(50):
        ids = rng.choice(500, size=60, replace=False)
        _, n_miss = model.fetch(ids, t)
        assert n_miss == len(set(ids.tolist()) - seen)
        seen |= set(ids.tolist())
    assert model.misses == len(seen)


def test_cyclic_pattern_closed_forms():
    # W + 1 keys cycled through one W-way set: every access misses; W keys: only the first round misses
    W = 8
    for n_keys, want_rate in ((W + 1, 1.0), (W, None)):
        model = oracle.FeatureCacheModel(1, W)
        t = 0
        for _ in range(20):
            for x in range(n_keys):
                model.fetch([x], t)
                t += 1
        if want_rate is not None:
            assert model.misses == model.queries
        else:
            assert model.misses == W


def test_batch_rules():
    model = oracle.FeatureCacheModel(1, 4)
    slots, miss = model.fetch([10, 11, 12, 13], 0)
    assert miss == 4 and slots.tolist() == [0, 1, 2, 3]           # empty rows are taken in way order
    # a batch that hits 11 and 13 and brings 3 new nodes: only the two untouched rows can be replaced,
    # the third miss (in batch order) is served without being cached
    slots, miss = model.fetch([20, 13, 21, 11, 22], 1)
    assert miss == 3
    assert slots.tolist() == [0, 3, 2, 1, -1]
    assert model.keys.tolist() == [20, 11, 21, 13]
    # least recently used first: rows 1 and 3 (stamp 1, hit) and 0, 2 (stamp 1, filled) are all equally recent,
    # so way order decides
    slots, miss = model.fetch([30], 2)
    assert slots.tolist() == [0]
    # now row 0 has stamp 2; the oldest are rows 1, 2, 3 (stamp 1): way order again
    slots, _ = model.fetch([31, 32], 3)
    assert slots.tolist() == [1, 2]


def test_community_ordered_batches_miss_less():
    # the effect the paper measures, in miniature: batches drawn from one community at a time reuse the cache,
    # batches drawn uniformly do not
    rng = np.random.default_rng(3)
    n_nodes, comm_size, batch = 4000, 200, 100
    def miss_rate(pick):
        model = oracle.FeatureCacheModel(32, 8)            # 256 rows
        for t in range(200):
            model.fetch(pick(t), t)
        return model.misses / model.queries
    uniform = miss_rate(lambda t: rng.choice(n_nodes, size=batch, replace=False))
    by_comm = miss_rate(lambda t: (t // 8 % (n_nodes // comm_size)) * comm_size + rng.choice(comm_size, size=batch, replace=False))
    assert by_comm < 0.5 * uniform
