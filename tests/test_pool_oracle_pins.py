"""Pins for the pooling / unpooling oracle (Sec. 3, "Pooling and unpooling"): a
hand-worked fixture, closed forms, and -- for every backward pass -- the
adjoint identity <forward(x), g> = <x, backward(g)>, which ties the backward
code to the forward code without retyping either.  CPU only."""
import json
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _random_clusters(rng, n_in, n_out):
    cid = rng.integers(0, n_out, size=n_in).astype(np.int32)
    cid[:n_out] = np.arange(n_out)          # no empty cluster
    rng.shuffle(cid)
    return cid


def test_hand_worked_fixture(oracle):
    fx = json.load(open(os.path.join(GOLD, "pool_hand.json")))
    cid, n_out = np.array(fx["cluster_id"], np.int32), fx["n_out"]
    x, w = np.array(fx["x"], np.float32), np.array(fx["w"], np.float32)
    assert oracle.pool_forward(oracle.POOL_AVG, x, cid, n_out).tolist() == fx["avg"]
    y, arg = oracle.pool_forward(oracle.POOL_MAX, x, cid, n_out)
    assert y.tolist() == fx["max"] and arg.tolist() == fx["argmax"]
    assert oracle.pool_forward(oracle.POOL_WEIGHTED, x, cid, n_out, w).tolist() == fx["weighted"]
    assert oracle.pool_forward(oracle.POOL_SUM, x, cid, n_out).tolist() == fx["sum"]
    assert oracle.unpool_forward(np.array(fx["y"], np.float32), cid).tolist() == fx["unpool"]
    assert oracle.unpool_backward(x, cid, n_out).tolist() == fx["sum"]
    gy = np.array(fx["gy"], np.float32)
    assert oracle.pool_backward(oracle.POOL_AVG, gy, cid, 6).tolist() == fx["avg_backward"]
    assert oracle.pool_backward(oracle.POOL_MAX, gy, cid, 6, argmax=arg).tolist() == fx["max_backward"]
    assert oracle.pool_backward(oracle.POOL_WEIGHTED, gy, cid, 6, weight=w).tolist() == fx["weighted_backward"]


def test_closed_forms(oracle):
    rng = np.random.default_rng(3)
    n_in, n_out, C = 500, 120, 7
    cid = _random_clusters(rng, n_in, n_out)
    x = rng.normal(size=(n_in, C)).astype(np.float32)
    sizes = np.bincount(cid, minlength=n_out)
    avg = oracle.pool_forward(oracle.POOL_AVG, x, cid, n_out)
    summ = oracle.pool_forward(oracle.POOL_SUM, x, cid, n_out)
    mx, arg = oracle.pool_forward(oracle.POOL_MAX, x, cid, n_out)
    # numpy scatter-add in fp64 as the independent sum
    ref = np.zeros((n_out, C))
    np.add.at(ref, cid, x.astype(np.float64))
    np.testing.assert_allclose(summ, ref, rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(avg, ref / sizes[:, None], rtol=1e-6, atol=1e-6)
    refmax = np.full((n_out, C), -np.inf)
    np.maximum.at(refmax, cid, x.astype(np.float64))
    assert np.array_equal(mx, refmax.astype(np.float32))
    assert np.all(mx >= avg - 1e-6)
    # argmax points into the right cluster, at a member holding the max, and at the FIRST such member
    for c in range(0, n_out, 7):
        for k in range(C):
            v = arg[c, k]
            assert cid[v] == c and x[v, k] == mx[c, k]
            assert not np.any(x[(cid == c) & (np.arange(n_in) < v), k] == mx[c, k])
    # constants are fixed points of avg, weighted and max pooling; uniform weights reduce weighted to avg
    one = np.full((n_in, C), 2.5, np.float32)
    w = rng.uniform(0.1, 2.0, size=n_in).astype(np.float32)
    for mode, kw in ((oracle.POOL_AVG, {}), (oracle.POOL_WEIGHTED, {"weight": w})):
        assert np.allclose(oracle.pool_forward(mode, one, cid, n_out, **kw), 2.5, atol=1e-6)
    assert np.array_equal(oracle.pool_forward(oracle.POOL_MAX, one, cid, n_out)[0], np.full((n_out, C), 2.5, np.float32))
    np.testing.assert_allclose(oracle.pool_forward(oracle.POOL_WEIGHTED, x, cid, n_out, np.full(n_in, 0.7, np.float32)),
                               avg, rtol=1e-5, atol=1e-6)
    # pooling is invariant to relabelling the vertices
    perm = rng.permutation(n_in)
    np.testing.assert_allclose(oracle.pool_forward(oracle.POOL_AVG, x[perm], cid[perm], n_out), avg, rtol=1e-6, atol=1e-6)
    # unpool then average-pool is the identity on cluster features
    y = rng.normal(size=(n_out, C)).astype(np.float32)
    up = oracle.unpool_forward(y, cid)
    assert np.array_equal(up, y[cid])
    np.testing.assert_allclose(oracle.pool_forward(oracle.POOL_AVG, up, cid, n_out), y, rtol=1e-6, atol=1e-6)


@pytest.mark.parametrize("mode", ["avg", "weighted", "max", "unpool"])
def test_backward_is_the_adjoint_of_forward(oracle, mode):
    rng = np.random.default_rng(11)
    n_in, n_out, C = 300, 70, 5
    cid = _random_clusters(rng, n_in, n_out)
    x = rng.normal(size=(n_in, C)).astype(np.float32)
    g = rng.normal(size=(n_out, C)).astype(np.float32)
    w = rng.uniform(0.2, 3.0, size=n_in).astype(np.float32)
    if mode == "avg":
        lhs = np.vdot(oracle.pool_forward(oracle.POOL_AVG, x, cid, n_out).astype(np.float64), g)
        rhs = np.vdot(x.astype(np.float64), oracle.pool_backward(oracle.POOL_AVG, g, cid, n_in))
    elif mode == "weighted":
        lhs = np.vdot(oracle.pool_forward(oracle.POOL_WEIGHTED, x, cid, n_out, w).astype(np.float64), g)
        rhs = np.vdot(x.astype(np.float64), oracle.pool_backward(oracle.POOL_WEIGHTED, g, cid, n_in, weight=w))
    elif mode == "max":
        y, arg = oracle.pool_forward(oracle.POOL_MAX, x, cid, n_out)
        lhs = np.vdot(y.astype(np.float64), g)      # max pooling is linear once the argmax is fixed
        rhs = np.vdot(x.astype(np.float64), oracle.pool_backward(oracle.POOL_MAX, g, cid, n_in, argmax=arg))
    else:
        gx = rng.normal(size=(n_in, C)).astype(np.float32)
        lhs = np.vdot(oracle.unpool_forward(g, cid).astype(np.float64), gx)
        rhs = np.vdot(g.astype(np.float64), oracle.unpool_backward(gx, cid, n_out))
    assert abs(lhs - rhs) <= 1e-4 * (1 + abs(lhs))


def test_max_backward_matches_finite_differences(oracle):
    rng = np.random.default_rng(5)
    n_in, n_out, C = 40, 9, 3
    cid = _random_clusters(rng, n_in, n_out)
    x = rng.normal(size=(n_in, C)).astype(np.float32)
    g = rng.normal(size=(n_out, C)).astype(np.float32)
    y, arg = oracle.pool_forward(oracle.POOL_MAX, x, cid, n_out)
    gx = oracle.pool_backward(oracle.POOL_MAX, g, cid, n_in, argmax=arg)
    eps = 1e-3
    for v in range(0, n_in, 3):
        for k in range(C):
            xp = x.copy()
            xp[v, k] += eps
            xm = x.copy()
            xm[v, k] -= eps
            fp = np.vdot(oracle.pool_forward(oracle.POOL_MAX, xp, cid, n_out)[0].astype(np.float64), g)
            fm = np.vdot(oracle.pool_forward(oracle.POOL_MAX, xm, cid, n_out)[0].astype(np.float64), g)
            fd = (fp - fm) / (2 * eps)
            # away from ties the two-sided difference is g at the argmax, or half of it when the bump crosses a tie
            assert abs(fd - gx[v, k]) < 1e-2 or abs(2 * fd - g[cid[v], k]) < 1e-2 or abs(fd) < 1e-2


def test_pooling_on_a_decimated_mesh(oracle):
    """cluster_id straight from the decimation: average pooling of the vertex positions of a
    single round reproduces the contracted positions (mean placement), max pooling bounds them."""
    from paper_2103_15076_amd import meshgen
    V, F = meshgen.noisy_grid(20, 15, seed=4)
    r = oracle.decimate(V, F, 1, max_rounds=1)
    avg = oracle.pool_forward(oracle.POOL_AVG, V, r["cluster_id"], r["verts"].shape[0])
    np.testing.assert_allclose(avg, r["verts"], atol=1e-6)
    mx, _ = oracle.pool_forward(oracle.POOL_MAX, V, r["cluster_id"], r["verts"].shape[0])
    assert np.all(mx >= r["verts"] - 1e-6)


def test_bad_inputs(oracle):
    x = np.zeros((4, 2), np.float32)
    with pytest.raises(ValueError):
        oracle.pool_forward(oracle.POOL_AVG, x, np.array([0, 1, 2, 3], np.int32), 3)
    with pytest.raises(ValueError):
        oracle.pool_forward(oracle.POOL_AVG, x, np.array([0, -1, 0, 0], np.int32), 3)
