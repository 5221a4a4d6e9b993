"""Pins of the oracle's collective-ready layouts (Alg. 1 and Alg. 2 of the
paper): the hidden-column shard a TP rank sends in the fused AG-Dispatch, and
the per-stage accumulation of the fused RS-Combine.  They are pinned to what
the mathematics fixes: the shards of all TP ranks tile the full send buffer,
a library gather gives the same rows, and the stages / column blocks add up to
the plain combine (which has its own pins)."""
import numpy as np
import pytest

import oracle


def routing(rng, T, E, k):
    ids = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    w = rng.random((T, k), dtype=np.float32) + 0.1
    return ids, w


@pytest.mark.parametrize("T,k,H,E,lo,hi,m", [(37, 3, 64, 10, 2, 7, 4), (5, 2, 48, 4, 0, 4, 3),
                                             (64, 8, 128, 32, 8, 16, 8), (9, 1, 16, 3, 1, 2, 1)])
def test_shards_tile_the_full_send_buffer(T, k, H, E, lo, hi, m):
    rng = np.random.default_rng(T * 131 + m)
    ids, _ = routing(rng, T, E, k)
    x = rng.standard_normal((T, H)).astype(np.float32)
    c, o, perm, inv, xs = oracle.dispatch(ids, x, lo, hi)
    shards = []
    for r in range(m):
        cr, orr, pr, ir, xr = oracle.dispatch_shard(ids, x, lo, hi, r, m)
        # the expert map does not depend on the rank
        assert np.array_equal(cr, c) and np.array_equal(orr, o)
        assert np.array_equal(pr, perm) and np.array_equal(ir, inv)
        # a library gather of the same rows and columns
        assert np.array_equal(xr, x[perm // k][:, r * (H // m):(r + 1) * (H // m)])
        shards.append(xr)
    assert np.array_equal(np.concatenate(shards, axis=1), xs)


def test_shard_of_one_rank_is_plain_dispatch():
    rng = np.random.default_rng(3)
    ids, _ = routing(rng, 20, 6, 2)
    x = rng.standard_normal((20, 32)).astype(np.float32)
    a = oracle.dispatch(ids, x, 0, 6)
    b = oracle.dispatch_shard(ids, x, 0, 6, 0, 1)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


def test_empty_range_gives_empty_shard():
    rng = np.random.default_rng(4)
    ids = np.zeros((7, 2), np.int32)          # every assignment goes to expert 0
    x = rng.standard_normal((7, 16)).astype(np.float32)
    c, o, perm, inv, xs = oracle.dispatch_shard(ids, x, 1, 3, 1, 2)
    assert c.tolist() == [0, 0] and o.tolist() == [0, 0, 0]
    assert perm.size == 0 and xs.shape == (0, 8) and (inv == -1).all()


@pytest.mark.parametrize("T,k,H,E,n_nodes,m", [(33, 4, 64, 16, 4, 2), (50, 8, 96, 32, 8, 4),
                                               (7, 2, 24, 6, 3, 3)])
def test_stages_and_blocks_add_up_to_the_plain_combine(T, k, H, E, n_nodes, m):
    """Stage i returns the rows of the experts hosted by node i.  Accumulating
    the stages per column block and laying the blocks side by side must give
    the combine of all experts at once."""
    rng = np.random.default_rng(T + 17 * m)
    ids, w = routing(rng, T, E, k)
    x = rng.standard_normal((T, H)).astype(np.float32)
    per = E // n_nodes
    # full combine over all experts, with arbitrary expert outputs
    c, o, perm, inv_all, _ = oracle.dispatch(ids, x, 0, E)
    ys_all = rng.standard_normal((T * k, H))
    ref = oracle.combine(ys_all, inv_all, w).astype(np.float64)
    direct = np.zeros((T, H))
    for t in range(T):
        for j in range(k):
            direct[t] += float(w[t, j]) * ys_all[inv_all[t * k + j]]
    np.testing.assert_allclose(ref, direct, rtol=0, atol=1e-6 * np.abs(direct).max())
    blocks = []
    for r in range(m):
        blk = None
        for i in range(n_nodes):
            ci, oi, pi, inv_i, _ = oracle.dispatch(ids, x, i * per, (i + 1) * per)
            # rows of node i are the rows of its experts, in the same order
            ys_i = ys_all[inv_all[pi]]
            blk = oracle.combine_stage(ys_i[:, r * (H // m):(r + 1) * (H // m)], inv_i, w, blk)
        blocks.append(blk)
    got = np.concatenate(blocks, axis=1).astype(np.float64)
    # every stage stores fp32: n_nodes roundings of magnitude <= max|out| * 2^-24
    np.testing.assert_allclose(got, direct, rtol=0, atol=n_nodes * 1.2e-7 * np.abs(direct).max())


def test_first_stage_overwrites_and_later_stages_add():
    rng = np.random.default_rng(9)
    ids, w = routing(rng, 12, 5, 2)
    x = rng.standard_normal((12, 8)).astype(np.float32)
    c, o, perm, inv, _ = oracle.dispatch(ids, x, 0, 5)
    ys = rng.standard_normal((24, 8))
    first = oracle.combine_stage(ys, inv, w, None)
    assert np.array_equal(first, oracle.combine(ys, inv, w))
    second = oracle.combine_stage(ys, inv, w, first)
    np.testing.assert_allclose(second, 2.0 * first.astype(np.float64), rtol=3e-7)
    # a stage with no local assignment leaves the block unchanged
    none = np.full_like(inv, -1)
    assert np.array_equal(oracle.combine_stage(ys, none, w, first), first)
    assert np.array_equal(oracle.combine_stage(ys, none, w, None), np.zeros_like(first))
