"""Pins for the oracle's inverse-placement variant (supplementary section
"Quadric error computation", Eq. "inverse_optimal": target = -A^-1 b where A
has full rank by the reciprocal of its condition number, else the mean of Eq.
"average_optimal"; the oracle estimates that number by the pivot ratio d3 / d1
of a diagonally pivoted L D L^T factorisation).  Every check compares the oracle with something that is
not the oracle: exact small cases, fp64 linear algebra from numpy, the
minimum property of the quadratic form, a recomputation of a whole round from
the input mesh.  (CPU only.)
"""
import numpy as np
import pytest

from paper_2103_15076_amd import meshgen

MEAN, INVERSE = 0, 1


def _mat(q):
    q = np.asarray(q, np.float64)
    A = np.array([[q[0], q[1], q[2]], [q[1], q[3], q[4]], [q[2], q[4], q[5]]])
    return A, q[6:9].copy(), float(q[9])


def _plane_quadric64(n, p):
    n = np.asarray(n, np.float64)
    n = n / np.linalg.norm(n)
    d = -float(n @ np.asarray(p, np.float64))
    A = np.outer(n, n)
    return np.array([A[0, 0], A[0, 1], A[0, 2], A[1, 1], A[1, 2], A[2, 2], d * n[0], d * n[1], d * n[2], d * d])


def test_three_orthogonal_planes_give_their_corner_exactly(oracle):
    """Planes x = a, y = b, z = c: A = I, b = -(a, b, c), so -A^-1 b is the corner
    itself, rcond is 1 and the quadric error there is exactly zero."""
    a, b, c = 0.75, -1.5, 2.25
    V = np.array([[a, 0, 0], [a, 1, 0], [a, 0, 1],
                  [0, b, 0], [0, b, 1], [1, b, 0],
                  [0, 0, c], [1, 0, c], [0, 1, c]], np.float32)
    F = np.array([[0, 1, 2], [3, 4, 5], [6, 7, 8]], np.int32)
    q = oracle.facet_quadrics(V, F).sum(axis=0, dtype=np.float32)
    pu, pv = np.array([5, 6, 7], np.float32), np.array([-1, 0, 3], np.float32)
    t, rcond, used = oracle.pair_target(q, pu, pv, INVERSE, 1e-3)
    assert used and rcond == 1.0
    assert np.array_equal(t, np.array([a, b, c], np.float32))
    # the cost of the pair is the error at that target: split q over two "vertices"
    Q = np.stack([q * np.float32(0.5), q * np.float32(0.5)])
    cost, _ = oracle.edge_costs(np.stack([pu, pv]), Q, np.array([[0, 1]], np.int32), INVERSE, 1e-3)
    assert cost[0] == 0.0
    # with the mean placement the same pair costs the squared distances of the mean to the planes
    cost_m, _ = oracle.edge_costs(np.stack([pu, pv]), Q, np.array([[0, 1]], np.int32))
    m = (pu.astype(np.float64) + pv) / 2
    assert cost_m[0] == pytest.approx(float(((m - [a, b, c]) ** 2).sum()), rel=1e-6)
    # placement = mean ignores the quadric
    t0, _, used0 = oracle.pair_target(q, pu, pv, MEAN, 0.0)
    assert not used0 and np.array_equal(t0, (pu + pv) * np.float32(0.5))


@pytest.mark.parametrize("normal", [(0, 0, 1), (1, 2, 3), (-0.3, 0.9, 0.1)])
def test_planar_patch_falls_back_to_the_mean(oracle, normal):
    """All facets in one plane: A = k n n^T has rank 1 (up to rounding), so the
    target must be the mean of the pair for any threshold above rounding noise."""
    rng = np.random.default_rng(3)
    n = np.asarray(normal, np.float64)
    n /= np.linalg.norm(n)
    # an orthonormal basis of the plane through p0
    u = np.cross(n, [1.0, 0.0, 0.0] if abs(n[0]) < 0.9 else [0.0, 1.0, 0.0])
    u /= np.linalg.norm(u)
    w = np.cross(n, u)
    p0 = np.array([0.3, -0.2, 0.5])
    uv = rng.uniform(-1, 1, size=(12, 2))
    V = (p0 + uv[:, :1] * u + uv[:, 1:] * w).astype(np.float32)
    F = np.array([[0, 1, 2], [3, 4, 5], [6, 7, 8], [9, 10, 11]], np.int32)
    q = oracle.facet_quadrics(V, F).sum(axis=0, dtype=np.float32)
    pu, pv = V[0], V[5]
    t, rcond, used = oracle.pair_target(q, pu, pv, INVERSE, 1e-5)
    assert not used and rcond < 1e-5
    assert np.array_equal(t, (pu + pv) * np.float32(0.5))


def test_target_solves_the_linear_system_and_rcond_brackets_the_true_one(oracle):
    """Random well-conditioned sums of plane quadrics: the target agrees with
    numpy's fp64 solve of A x = -b within the fp32 error bound eps * cond, and the
    reported pivot ratio lies between lambda_min / lambda_max (numpy, fp64) and
    27 times that, the bracket that holds for a diagonally pivoted 3x3 positive
    definite matrix (a wrong pivot, sign, or swapped component fails this)."""
    rng = np.random.default_rng(11)
    eps = 2.0 ** -24
    checked = 0
    for _ in range(300):
        k = int(rng.integers(3, 7))
        q64 = sum(_plane_quadric64(rng.normal(size=3), rng.uniform(-2, 2, size=3)) for _ in range(k))
        A, b, _ = _mat(q64)
        rc64 = 1.0 / (np.linalg.norm(A, 1) * np.linalg.norm(np.linalg.inv(A), 1))
        if rc64 < 1e-2:
            continue
        q = q64.astype(np.float32)
        A32, b32, _ = _mat(q)  # the system the oracle actually sees
        x64 = np.linalg.solve(A32, -b32)
        t, rcond, used = oracle.pair_target(q, np.zeros(3, np.float32), np.ones(3, np.float32), INVERSE, 1e-3)
        assert used
        lam = np.linalg.eigvalsh(A32)
        rc_seen = lam[0] / lam[2]
        assert rc_seen * (1 - 1e-4) <= rcond <= 27 * rc_seen * (1 + 1e-4)
        assert np.abs(t - x64).max() <= 64 * eps / rc_seen * max(1.0, np.abs(x64).max())
        checked += 1
    assert checked > 100


def test_threshold_is_strict_and_applies_to_rcond(oracle):
    """A = diag(1, 1, e): the pivots are 1, 1, e, so the ratio is e exactly; the
    minimiser is used iff e > threshold."""
    e = np.float32(2.0 ** -10)
    q = np.array([1, 0, 0, 1, 0, e, 0.5, -0.25, 2.0 ** -12, 0.0], np.float32)
    pu, pv = np.zeros(3, np.float32), np.array([2, 4, 6], np.float32)
    t, rcond, used = oracle.pair_target(q, pu, pv, INVERSE, float(e))
    assert rcond == float(e) and not used and np.array_equal(t, np.array([1, 2, 3], np.float32))
    t, rcond, used = oracle.pair_target(q, pu, pv, INVERSE, float(e) / 2)
    assert used and np.array_equal(t, np.array([-0.5, 0.25, -0.25], np.float32))


def test_target_minimises_the_quadric(oracle):
    """Wherever the minimiser is used, no nearby point has a smaller error and the
    gradient 2 (A x + b) vanishes to rounding (fp64 evaluation)."""
    rng = np.random.default_rng(5)
    for _ in range(100):
        q64 = sum(_plane_quadric64(rng.normal(size=3), rng.uniform(-1, 1, size=3)) for _ in range(5))
        q = q64.astype(np.float32)
        A, b, c = _mat(q)
        t, rcond, used = oracle.pair_target(q, np.zeros(3, np.float32), np.ones(3, np.float32), INVERSE, 1e-2)
        if not used:
            continue
        x = t.astype(np.float64)
        val = x @ A @ x + 2 * b @ x + c
        assert np.abs(A @ x + b).max() < 1e-4 / rcond * 1e-2 + 1e-5
        for _ in range(8):
            y = x + rng.normal(scale=0.05, size=3)
            assert y @ A @ y + 2 * b @ y + c >= val - 1e-6


def test_an_unreachable_threshold_reproduces_the_mean_placement_path(oracle):
    """rcond never exceeds 1, so with threshold 1 the variant must give the default
    path's result bit for bit, over several rounds."""
    cfg = meshgen.config("grid64")
    a = oracle.decimate(cfg["verts"], cfg["facets"], 1024)
    b = oracle.decimate(cfg["verts"], cfg["facets"], 1024, placement=INVERSE, rcond_min=1.0)
    assert a["status"] == b["status"] == 0 and a["rounds"] == b["rounds"]
    for k in ("verts", "facets", "cluster_id"):
        assert np.array_equal(a[k], b[k]), k


def _vertex_quadrics64(V, F):
    """Vertex quadrics from the definition, in fp64, with numpy only."""
    V = V.astype(np.float64)
    Q = np.zeros((V.shape[0], 10))
    for f in F:
        p0, p1, p2 = V[f[0]], V[f[1]], V[f[2]]
        n = np.cross(p1 - p0, p2 - p0)
        ln = np.linalg.norm(n)
        if ln == 0 or len(set(f.tolist())) < 3:
            continue
        qf = _plane_quadric64(n, p0)
        for v in f:
            Q[v] += qf
    return Q


def test_one_round_recomputed_from_the_input_mesh(oracle):
    """One run of the core algorithm on a bumpy closed surface: every output vertex
    whose cluster is a pair sits at numpy's fp64 minimiser of the pair's summed
    quadric where that system is well conditioned, at the pair's mean where it is
    far below the threshold, and un-paired vertices stay where they were."""
    rng = np.random.default_rng(21)
    V, F = meshgen.icosphere(3, seed=None)
    V = (V * (1.0 + 0.08 * rng.normal(size=(V.shape[0], 1)))).astype(np.float32)
    thr = 1e-3
    res = oracle.decimate(V, F, V.shape[0] // 2, max_rounds=1, placement=INVERSE, rcond_min=thr)
    assert res["status"] in (0, 1) and res["rounds"] == 1
    cid = res["cluster_id"]
    Q = _vertex_quadrics64(V, F)
    n_inv = n_mean = 0
    for c in range(res["verts"].shape[0]):
        members = np.nonzero(cid == c)[0]
        assert 1 <= len(members) <= 2
        if len(members) == 1:
            assert np.array_equal(res["verts"][c], V[members[0]])
            continue
        A, b, _ = _mat(Q[members].sum(axis=0))
        lam = np.linalg.eigvalsh(A)
        rc = max(lam[0], 0.0) / lam[2]  # the oracle's pivot ratio lies in [rc, 27 rc]
        mean = (V[members[0]].astype(np.float64) + V[members[1]]) / 2
        if rc > 10 * thr:
            x = np.linalg.solve(A, -b)
            assert np.abs(res["verts"][c] - x).max() < 2e-5 / rc
            n_inv += 1
        elif rc < thr / 100:
            assert np.abs(res["verts"][c] - mean).max() < 1e-6
            n_mean += 1
    assert n_inv > 50


def test_a_planted_mistake_in_the_solve_would_be_caught(oracle):
    """The solve pin above is sharp: numpy's solution of a system with one
    off-diagonal sign flipped differs from the oracle's target by far more than the
    tolerance used there."""
    rng = np.random.default_rng(2)
    q64 = sum(_plane_quadric64(rng.normal(size=3), rng.uniform(-2, 2, size=3)) for _ in range(4))
    q = q64.astype(np.float32)
    A, b, _ = _mat(q)
    t, rcond, used = oracle.pair_target(q, np.zeros(3, np.float32), np.ones(3, np.float32), INVERSE, 1e-4)
    assert used
    A_bad = A.copy()
    A_bad[0, 1] = A_bad[1, 0] = -A[0, 1]
    x_bad = np.linalg.solve(A_bad, -b)
    assert np.abs(t - x_bad).max() > 1e-3


def test_target_is_equivariant_under_relabelling_the_axes(oracle):
    """Pivoting eliminates the largest diagonal entry first whatever axis carries
    it, so relabelling the axes of the quadric relabels the target bit for bit
    (all three pivot choices and the exchange in the 2x2 block are exercised)."""
    import itertools
    rng = np.random.default_rng(8)
    idx = {(0, 0): 0, (0, 1): 1, (0, 2): 2, (1, 1): 3, (1, 2): 4, (2, 2): 5}
    for _ in range(20):
        q64 = sum(_plane_quadric64(rng.normal(size=3), rng.uniform(-1, 1, size=3)) for _ in range(4))
        q = q64.astype(np.float32)
        t, _, used = oracle.pair_target(q, np.zeros(3, np.float32), np.ones(3, np.float32), INVERSE, 1e-4)
        if not used:
            continue
        for perm in itertools.permutations(range(3)):
            qp = q.copy()
            for i in range(3):
                for j in range(i, 3):
                    a, b = sorted((perm[i], perm[j]))
                    qp[idx[(i, j)]] = q[idx[(a, b)]]
                qp[6 + i] = q[6 + perm[i]]
            tp, _, usedp = oracle.pair_target(qp, np.zeros(3, np.float32), np.ones(3, np.float32), INVERSE, 1e-4)
            assert usedp and np.array_equal(tp, t[list(perm)]), perm
