"""Pins for the oracle of the two mesh convolutions (Sec. 4 "Mesh Convolution";
supplementary, "Backward propagations of different convolutions"): hand-sized
closed forms of the interpolation lattice, numpy re-derivations through a
different algebraic route (the 3x3 moment matrix of the lattice; scatter-adds),
finite differences and the adjoint identity for every backward pass.  CPU only.
"""
import itertools

import numpy as np
import pytest
from scipy.special import softmax

from paper_2103_15076_amd import meshgen


def _lattice(k):
    if k == 1:
        return np.array([[1 / 3, 1 / 3, 1 / 3]])
    pts = [(i, j, k - 1 - i - j) for i in range(k) for j in range(k - i)]
    return np.array(pts, float) / (k - 1)


def test_v2f_small_levels_closed_forms(oracle):
    """k = 1: the centroid alone, J = (w1+w2+w3)(I1+I2+I3)/9.  k = 2: the three
    vertices, J = (w1 I1 + w2 I2 + w3 I3)/3.  k = 3: vertices and edge midpoints,
    J = [sum_s w_s I_s + sum_{s<r} (w_s+w_r)(I_s+I_r)/4] / 6."""
    rng = np.random.default_rng(0)
    x = rng.normal(size=(3, 5)).astype(np.float32)
    w = rng.normal(size=(3, 5)).astype(np.float32)
    F = np.array([[0, 1, 2]], np.int32)
    X, W = x.astype(float), w.astype(float)
    j1 = W.sum(0) * X.sum(0) / 9
    j2 = (W * X).sum(0) / 3
    j3 = ((W * X).sum(0) + sum((W[s] + W[r]) * (X[s] + X[r]) / 4 for s, r in ((0, 1), (0, 2), (1, 2)))) / 6
    for k, want in ((1, j1), (2, j2), (3, j3)):
        got = oracle.v2f_forward(x, F, [k], w)[0]
        np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("k", [1, 2, 3, 4, 7])
def test_v2f_is_the_moment_matrix_of_the_lattice(oracle, k):
    """J = w^T M I with M = (1/K) sum_k xi xi^T: K = k(k+1)/2 lattice points that sum
    to 1 each; by symmetry M has one diagonal and one off-diagonal value."""
    xi = _lattice(k)
    assert xi.shape[0] == k * (k + 1) // 2 and np.allclose(xi.sum(1), 1) and xi.min() >= 0
    M = xi.T @ xi / xi.shape[0]
    assert np.allclose(np.diag(M), M[0, 0]) and np.allclose(M[~np.eye(3, dtype=bool)], M[0, 1])
    rng = np.random.default_rng(k)
    V, F = meshgen.icosphere(1, seed=None)
    x = rng.normal(size=(V.shape[0], 4)).astype(np.float32)
    w = rng.normal(size=(3, 4)).astype(np.float32)
    y = oracle.v2f_forward(x, F, np.full(F.shape[0], k), w)
    want = np.einsum("sc,sr,frc->fc", w.astype(float), M, x.astype(float)[F])
    np.testing.assert_allclose(y, want, rtol=1e-12, atol=1e-12)
    # relabelling a facet's corners together with the filter rows changes nothing
    for perm in itertools.permutations(range(3)):
        yp = oracle.v2f_forward(x, F[:, perm], np.full(F.shape[0], k), w[list(perm)])
        np.testing.assert_allclose(yp, y, rtol=1e-12, atol=1e-12)


def _fd(fn, a, eps=1e-3):
    """Central finite differences of the scalar fn with respect to the float32 array a."""
    g = np.zeros(a.shape)
    it = np.nditer(a, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        ap, am = a.copy(), a.copy()
        ap[i] += eps
        am[i] -= eps
        g[i] = (fn(ap) - fn(am)) / (float(ap[i]) - float(am[i]))
    return g


def test_v2f_backward_is_the_gradient_and_the_adjoint(oracle):
    rng = np.random.default_rng(2)
    V, F = meshgen.icosphere(1, seed=None)
    N, C = V.shape[0], 3
    level = rng.integers(1, 5, F.shape[0]).astype(np.int32)
    x = rng.normal(size=(N, C)).astype(np.float32)
    w = rng.normal(size=(3, C)).astype(np.float32)
    gy = rng.normal(size=(F.shape[0], C)).astype(np.float32)
    gx, gw = oracle.v2f_backward(gy, x, F, level, w)
    loss = lambda xx, ww: float((oracle.v2f_forward(xx, F, level, ww) * gy).sum())
    np.testing.assert_allclose(gx, _fd(lambda a: loss(a, w), x), rtol=2e-4, atol=2e-4)
    np.testing.assert_allclose(gw, _fd(lambda a: loss(x, a), w), rtol=2e-4, atol=2e-4)
    # the forward pass is linear in x for fixed w and vice versa
    assert loss(x, w) == pytest.approx(float((gx * x).sum()), rel=1e-6)
    assert loss(x, w) == pytest.approx(float((gw * w).sum()), rel=1e-6)


def test_f2v_reduces_to_the_mean_of_adjacent_facets(oracle):
    """T = 1, pi = 1, w = 1: I_v is the plain average of the features of the facets
    around v (numpy scatter-add), zero for a vertex without facets."""
    rng = np.random.default_rng(3)
    V, F = meshgen.noisy_grid(9, 7, seed=1)
    N = V.shape[0] + 2  # two vertices no facet refers to
    y = rng.normal(size=(F.shape[0], 6)).astype(np.float32)
    x = oracle.f2v_forward(y, np.ones((F.shape[0], 1)), np.ones((1, 6)), F, N)
    acc, deg = np.zeros((N, 6)), np.zeros(N)
    for s in range(3):
        np.add.at(acc, F[:, s], y.astype(float))
        np.add.at(deg, F[:, s], 1)
    want = np.where(deg[:, None] > 0, acc / np.maximum(deg, 1)[:, None], 0.0)
    np.testing.assert_allclose(x, want, rtol=1e-12, atol=1e-12)
    assert np.all(x[-2:] == 0)


def test_f2v_general_case_by_another_route(oracle):
    rng = np.random.default_rng(4)
    V, F = meshgen.icosphere(2, seed=None)
    N, C, T = V.shape[0], 5, 4
    y = rng.normal(size=(F.shape[0], C)).astype(np.float32)
    pi = softmax(rng.normal(size=(F.shape[0], T)), axis=1).astype(np.float32)
    w = rng.normal(size=(T, C)).astype(np.float32)
    x = oracle.f2v_forward(y, pi, w, F, N)
    contrib = (pi.astype(float) @ w.astype(float)) * y.astype(float)   # per facet
    acc, deg = np.zeros((N, C)), np.zeros(N)
    for s in range(3):
        np.add.at(acc, F[:, s], contrib)
        np.add.at(deg, F[:, s], 1)
    np.testing.assert_allclose(x, acc / deg[:, None], rtol=1e-12, atol=1e-12)


def test_f2v_backward_is_the_gradient_and_the_adjoint(oracle):
    rng = np.random.default_rng(5)
    V, F = meshgen.icosphere(1, seed=None)
    N, C, T = V.shape[0], 3, 3
    y = rng.normal(size=(F.shape[0], C)).astype(np.float32)
    pi = softmax(rng.normal(size=(F.shape[0], T)), axis=1).astype(np.float32)
    w = rng.normal(size=(T, C)).astype(np.float32)
    gx = rng.normal(size=(N, C)).astype(np.float32)
    gy, gw, gpi = oracle.f2v_backward(gx, y, pi, w, F)
    loss = lambda yy, pp, ww: float((oracle.f2v_forward(yy, pp, ww, F, N) * gx).sum())
    np.testing.assert_allclose(gy, _fd(lambda a: loss(a, pi, w), y), rtol=2e-4, atol=2e-4)
    np.testing.assert_allclose(gw, _fd(lambda a: loss(y, pi, a), w), rtol=2e-4, atol=2e-4)
    np.testing.assert_allclose(gpi, _fd(lambda a: loss(y, a, w), pi, eps=1e-4), rtol=2e-3, atol=2e-3)
    assert loss(y, pi, w) == pytest.approx(float((gy * y).sum()), rel=1e-6)
    assert loss(y, pi, w) == pytest.approx(float((gw * w).sum()), rel=1e-6)


def test_facet_geometry_levels_and_fuzzy_coefficients(oracle):
    V = np.array([[0, 0, 0], [2, 0, 0], [0, 1, 0], [0, 0, 3], [5, 5, 5]], np.float32)
    F = np.array([[0, 1, 2], [0, 3, 1], [0, 2, 3], [4, 4, 1]], np.int32)
    n, a = oracle.facet_geometry(V, F)
    assert a.tolist() == [1.0, 3.0, 1.5, 0.0]
    assert n.tolist() == [[0, 0, 1], [0, 1, 0], [1, 0, 0], [0, 0, 0]]
    # Eq. "interpolate_num" with alpha = beta = 1: floor(ratio) is 1 only for the largest facet
    assert oracle.facet_levels(a).tolist() == [1, 2, 1, 1]
    assert oracle.facet_levels(a, alpha=3, beta=2).tolist() == [2, 5, 2, 2]
    assert oracle.facet_levels(np.array([2.0, 2.0, 2.0])).tolist() == [1, 1, 1]            # all equal: ratio 0
    assert oracle.facet_levels(a, foff=[0, 2, 4]).tolist() == [1, 2, 2, 1]                 # per mesh of a batch
    # fuzzy coefficients against scipy's softmax of -z
    rng = np.random.default_rng(6)
    mu = np.array([[1, 0, 0], [-1, 0, 0], [0, 1, 0], [0, -1, 0], [0, 0, 1], [0, 0, -1]], np.float32)
    inv_var = rng.uniform(0.5, 4.0, 6).astype(np.float32)
    Vs, Fs = meshgen.icosphere(2, seed=3)
    ns, _ = oracle.facet_geometry(Vs, Fs)
    pi = oracle.fuzzy(ns, mu, inv_var)
    z = ((ns.astype(float)[:, None, :] - mu[None].astype(float)) ** 2).sum(-1) * inv_var[None].astype(float)
    np.testing.assert_allclose(pi, softmax(-z, axis=1), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(pi.sum(1), 1.0, rtol=1e-12)
    # a normal on a mean with a narrow component is claimed by it
    p = oracle.fuzzy(np.array([[0.0, 0.0, 1.0]], np.float32), mu, np.full(6, 50.0, np.float32))
    assert p[0, 4] > 0.999999


def test_vertex_corner_csr(oracle):
    F = np.array([[0, 1, 2], [2, 1, 3], [3, 3, 0]], np.int32)
    off, cor = oracle.vertex_corner_csr(F, 5)
    assert off.tolist() == [0, 2, 4, 6, 9, 9]
    assert cor.tolist() == [0, 8, 1, 4, 2, 3, 5, 6, 7]
    V, Fm = meshgen.icosphere(2, seed=None)
    off, cor = oracle.vertex_corner_csr(Fm, V.shape[0])
    flat = Fm.reshape(-1)
    for v in range(0, V.shape[0], 11):
        mine = cor[off[v]:off[v + 1]]
        assert np.all(flat[mine] == v) and np.all(np.diff(mine) > 0) and len(mine) == (flat == v).sum()


def test_facet_geometry_against_numpy_fp64(oracle):
    V, F = meshgen.icosphere(3, seed=5, jitter=0.05)
    n, a = oracle.facet_geometry(V, F)
    P = V.astype(float)[F]
    cr = np.cross(P[:, 1] - P[:, 0], P[:, 2] - P[:, 0])
    ln = np.linalg.norm(cr, axis=1)
    np.testing.assert_allclose(a, 0.5 * ln, rtol=1e-5)
    np.testing.assert_allclose(n, cr / ln[:, None], atol=1e-5)
    lev = oracle.facet_levels(a)
    assert (lev == 2).sum() == (a == a.max()).sum() and set(lev.tolist()) == {1, 2}


def _textured(rng, F, x, max_level=4):
    """Texture points of every facet = the lattice of a random level, their features = the
    barycentric interpolation of the vertex features (what vertex2facet interpolates itself)."""
    level = rng.integers(1, max_level + 1, F.shape[0]).astype(np.int32)
    bary = [_lattice(int(k)) for k in level]
    poff = np.concatenate([[0], np.cumsum([b.shape[0] for b in bary])]).astype(np.int32)
    tex = np.concatenate([b @ x.astype(float)[F[f]] for f, b in enumerate(bary)])
    return level, np.concatenate(bary).astype(np.float32), poff, tex.astype(np.float32)


def test_f2f_on_interpolated_textures_is_vertex2facet(oracle):
    """Facet2facet differs from vertex2facet only in that the points' features are given: fed with
    the features vertex2facet would interpolate, at the same points, it must give the same facet
    features (up to the fp32 rounding of the stored textures)."""
    rng = np.random.default_rng(7)
    V, F = meshgen.icosphere(2, seed=None)
    x = rng.normal(size=(V.shape[0], 5)).astype(np.float32)
    w = rng.normal(size=(3, 5)).astype(np.float32)
    level, bary, poff, tex = _textured(rng, F, x)
    got = oracle.f2f_forward(tex, bary, poff, w)
    want = oracle.v2f_forward(x, F, level, w)
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-6)
    # a facet without points gets 0; one point with weight w gives w . xi times its feature
    y = oracle.f2f_forward(np.array([[2.0, 3.0]], np.float32), np.array([[0.5, 0.25, 0.25]], np.float32), [0, 0, 1],
                           np.array([[1, 1], [2, 4], [4, 8]], np.float32))
    assert y.tolist() == [[0.0, 0.0], [2.0 * 2.0, 3.0 * 3.5]]


def test_f2f_backward_is_the_gradient_and_the_adjoint(oracle):
    rng = np.random.default_rng(8)
    V, F = meshgen.icosphere(1, seed=None)
    C = 3
    x = rng.normal(size=(V.shape[0], C)).astype(np.float32)
    w = rng.normal(size=(3, C)).astype(np.float32)
    _, bary, poff, tex = _textured(rng, F, x, max_level=3)
    tex = (tex + rng.normal(size=tex.shape)).astype(np.float32)   # textures of their own
    gy = rng.normal(size=(F.shape[0], C)).astype(np.float32)
    gtex, gw = oracle.f2f_backward(gy, tex, bary, poff, w)
    loss = lambda tt, ww: float((oracle.f2f_forward(tt, bary, poff, ww) * gy).sum())
    np.testing.assert_allclose(gtex, _fd(lambda a: loss(a, w), tex), rtol=2e-4, atol=2e-4)
    np.testing.assert_allclose(gw, _fd(lambda a: loss(tex, a), w), rtol=2e-4, atol=2e-4)
    assert loss(tex, w) == pytest.approx(float((gtex * tex).sum()), rel=1e-6)
    assert loss(tex, w) == pytest.approx(float((gw * w).sum()), rel=1e-6)
