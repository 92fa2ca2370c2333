"""Pins of the oracle's graph-attention layer (Section 6.4; layer of Velickovic et al.): a hand-computed
neighbourhood, the dense masked-softmax formulation through a library softmax, the reduction to mean aggregation
when the attention vector is zero, the softmax's shift invariance, and central finite differences for every
gradient."""
import numpy as np
import pytest
from scipy.special import softmax

import oracle


def random_block(rng, n_dst, n_extra, max_deg, empty_rows=()):
    n_src = n_dst + n_extra
    indptr = [0]
    indices = []
    for v in range(n_dst):
        d = 0 if v in empty_rows else int(rng.integers(1, max_deg + 1))
        indices += list(rng.choice(n_src, size=d, replace=False))
        indptr.append(len(indices))
    return oracle.Block(n_dst, np.arange(n_src, dtype=np.int32), np.asarray(indptr, dtype=np.int32),
                        np.asarray(indices, dtype=np.int32), None)


def test_hand_computed_neighbourhood():
    # one destination (row 0), neighbours rows 1 and 2, one head of width 1, a_l = 1, a_r = 0: the scores are z_u.
    blk = oracle.Block(1, np.arange(3, dtype=np.int32), np.array([0, 2], dtype=np.int32), np.array([1, 2], dtype=np.int32), None)
    ln2 = np.log(2.0)
    out, alpha = oracle.gat_attention_fwd(blk, np.array([[7.0], [ln2], [0.0]]), [1.0], [0.0], [0.5], heads=1)
    np.testing.assert_allclose(alpha[0][:, 0], [2 / 3, 1 / 3], rtol=1e-14)
    np.testing.assert_allclose(out, [[2 / 3 * ln2 + 0.5]], rtol=1e-14)
    # a negative score goes through the leaky slope: -5 ln2 * 0.2 = -ln2, against 0: weights 1/3 and 2/3
    out, alpha = oracle.gat_attention_fwd(blk, np.array([[7.0], [-5 * ln2], [0.0]]), [1.0], [0.0], [0.0], heads=1)
    np.testing.assert_allclose(alpha[0][:, 0], [1 / 3, 2 / 3], rtol=1e-14)
    np.testing.assert_allclose(out, [[-5 * ln2 / 3]], rtol=1e-14)
    # the destination's own term: a_r = 1 adds z_v = 7 to both scores, which the softmax cancels
    out2, alpha2 = oracle.gat_attention_fwd(blk, np.array([[7.0], [ln2], [0.0]]), [1.0], [1.0], [0.5], heads=1)
    np.testing.assert_allclose(alpha2[0][:, 0], [2 / 3, 1 / 3], rtol=1e-13)


@pytest.mark.parametrize("heads,D", [(1, 5), (4, 3)])
def test_dense_masked_softmax_formulation(heads, D):
    rng = np.random.default_rng(heads)
    blk = random_block(rng, 17, 30, 6, empty_rows=(4,))
    z = rng.standard_normal((blk.n_src, heads * D))
    a_l, a_r, b = rng.standard_normal(heads * D), rng.standard_normal(heads * D), rng.standard_normal(heads * D)
    out, _ = oracle.gat_attention_fwd(blk, z, a_l, a_r, b, heads, slope=0.2)
    z3 = z.reshape(-1, heads, D)
    el = (z3 * a_l.reshape(heads, D)).sum(-1)               # [n_src, heads]
    er = (z3 * a_r.reshape(heads, D)).sum(-1)
    S = el[None, :, :] + er[:blk.n_dst, None, :]            # [n_dst, n_src, heads]
    S = np.where(S > 0, S, 0.2 * S)
    mask = np.zeros((blk.n_dst, blk.n_src), dtype=bool)
    mask[np.repeat(np.arange(blk.n_dst), np.diff(blk.indptr)), blk.indices] = True
    S = np.where(mask[:, :, None], S, -np.inf)
    want = np.tile(b, (blk.n_dst, 1))
    rows = mask.any(axis=1)
    A = softmax(S[rows], axis=1)                              # library softmax over the source axis
    want[rows] += np.einsum("vuh,uhd->vhd", A, z3).reshape(-1, heads * D)
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(out[4], b)                     # the row without neighbours


def test_zero_attention_vector_is_mean_aggregation():
    rng = np.random.default_rng(3)
    blk = random_block(rng, 12, 20, 5)
    z = rng.standard_normal((blk.n_src, 8))
    out, alpha = oracle.gat_attention_fwd(blk, z, np.zeros(8), np.zeros(8), np.zeros(8), heads=2)
    A = np.zeros((blk.n_dst, blk.n_src))
    for v in range(blk.n_dst):
        nb = blk.indices[blk.indptr[v]:blk.indptr[v + 1]]
        A[v, nb] = 1.0 / len(nb)
    np.testing.assert_allclose(out, A @ z, rtol=1e-13, atol=1e-13)
    # and it agrees with the oracle's own mean aggregation on the same block
    np.testing.assert_allclose(out, oracle.gather_mean(blk, z.astype(np.float32), indirect=False),
                               rtol=1e-6, atol=1e-6)


def test_identity_slope_makes_the_destination_term_cancel():
    # with slope 1 the LeakyReLU is the identity, the destination's term is a per-row constant, softmax drops it
    rng = np.random.default_rng(4)
    blk = random_block(rng, 9, 11, 4)
    z = rng.standard_normal((blk.n_src, 6))
    a_l, b = rng.standard_normal(6), rng.standard_normal(6)
    o1, _ = oracle.gat_attention_fwd(blk, z, a_l, rng.standard_normal(6), b, 3, slope=1.0)
    o2, _ = oracle.gat_attention_fwd(blk, z, a_l, np.zeros(6), b, 3, slope=1.0)
    np.testing.assert_allclose(o1, o2, rtol=1e-12, atol=1e-12)
    G = rng.standard_normal(o1.shape)
    _, _, d_ar, _ = oracle.gat_attention_bwd(blk, z, a_l, rng.standard_normal(6), 3, G, slope=1.0)
    np.testing.assert_allclose(d_ar, 0.0, atol=1e-12)


def test_neighbour_order_does_not_matter():
    rng = np.random.default_rng(5)
    blk = random_block(rng, 8, 10, 5)
    z = rng.standard_normal((blk.n_src, 4))
    a_l, a_r, b = rng.standard_normal(4), rng.standard_normal(4), rng.standard_normal(4)
    o1, _ = oracle.gat_attention_fwd(blk, z, a_l, a_r, b, 2)
    ind = blk.indices.copy()
    for v in range(blk.n_dst):
        ind[blk.indptr[v]:blk.indptr[v + 1]] = ind[blk.indptr[v]:blk.indptr[v + 1]][::-1]
    blk2 = oracle.Block(blk.n_dst, blk.src_ids, blk.indptr, ind, None)
    o2, _ = oracle.gat_attention_fwd(blk2, z, a_l, a_r, b, 2)
    np.testing.assert_allclose(o1, o2, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("heads,D", [(1, 4), (3, 2)])
def test_gradients_by_central_differences(heads, D):
    rng = np.random.default_rng(10 + heads)
    blk = random_block(rng, 7, 6, 4, empty_rows=(2,))
    HD = heads * D
    z = rng.standard_normal((blk.n_src, HD))
    a_l, a_r, b = rng.standard_normal(HD), rng.standard_normal(HD), rng.standard_normal(HD)
    R = rng.standard_normal((blk.n_dst, HD))
    loss = lambda z_, al_, ar_, b_: float(np.sum(oracle.gat_attention_fwd(blk, z_, al_, ar_, b_, heads)[0] * R))
    d_z, d_al, d_ar, d_b = oracle.gat_attention_bwd(blk, z, a_l, a_r, heads, R)
    h = 1e-6

    def numeric(x, f):
        g = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            xp, xm = x.copy(), x.copy()
            xp[i] += h
            xm[i] -= h
            g[i] = (f(xp) - f(xm)) / (2 * h)
        return g

    np.testing.assert_allclose(d_z, numeric(z, lambda x: loss(x, a_l, a_r, b)), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(d_al, numeric(a_l, lambda x: loss(z, x, a_r, b)), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(d_ar, numeric(a_r, lambda x: loss(z, a_l, x, b)), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(d_b, numeric(b, lambda x: loss(z, a_l, a_r, x)), rtol=1e-6, atol=1e-7)
