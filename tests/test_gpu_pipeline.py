"""One hierarchy level the way a network would use the library, through the C-ABI
only: facet geometry -> fuzzy coefficients -> vertex2facet -> facet2vertex
(a vertex2vertex convolution, Sec. 4) -> decimation with its cluster map (Sec.
3, Alg. 2) -> max pooling over the clusters -> the same convolution on the
coarse mesh -> unpooling back.  Every stage is compared with the oracle's stage
fed with the GPU's own inputs to that stage (integer work bit-exact, feature
sums within the bounds stated in the stage tests).
"""
import numpy as np
import pytest

from paper_2103_15076_amd import meshgen

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

EPS = 2.0 ** -24


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _v2v(ctx, oracle, V, F, x, w3, wt, mu, inv_var):
    """GPU vertex2vertex convolution with each stage checked; returns the GPU result (host)."""
    N, C, T = V.shape[0], x.shape[1], wt.shape[0]
    dV, dF = dev(V), dev(F)
    off, cor = ctx.picasso_vertex_corner_csr(dF, N)
    off_r, cor_r = oracle.vertex_corner_csr(F, N)
    assert np.array_equal(off.cpu().numpy(), off_r) and np.array_equal(cor.cpu().numpy(), cor_r)
    nrm, area, lev = ctx.picasso_facet_geometry(dV, dF)
    n_r, a_r = oracle.facet_geometry(V, F)
    lev_r = oracle.facet_levels(a_r)
    assert np.array_equal(nrm.cpu().numpy().view(np.uint32), n_r.view(np.uint32))
    assert np.array_equal(lev.cpu().numpy(), lev_r)
    pi = ctx.picasso_fuzzy_coefficients(nrm, dev(mu), dev(inv_var))
    pih = pi.cpu().numpy()
    assert np.abs(pih - oracle.fuzzy(n_r, mu, inv_var)).max() <= 16 * EPS
    y = ctx.picasso_v2f_forward(dev(x), dF, lev, dev(w3))
    yh = y.cpu().numpy()
    bound = 25 * EPS * oracle.v2f_forward(np.abs(x), F, lev_r, np.abs(w3)) + 1e-30
    assert np.all(np.abs(yh - oracle.v2f_forward(x, F, lev_r, w3)) <= bound)
    x2 = ctx.picasso_f2v_forward(y, pi, dev(wt), off, cor, N).cpu().numpy()
    deg = int(np.diff(off_r).max())
    bound = ((T + 2) * deg + 16) * EPS * oracle.f2v_forward(np.abs(yh), pih, np.abs(wt), F, N) + 1e-30
    assert np.all(np.abs(x2 - oracle.f2v_forward(yh, pih, wt, F, N)) <= bound)
    return x2


@pytest.mark.parametrize("absorb", [0, 1])
def test_one_level_of_a_mesh_network(oracle, absorb):
    import paper_2103_15076_amd as pk
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    V, F = meshgen.room_scene(21, room=(4.0, 3.0, 2.0), n_boxes=6, spacing=0.07)
    N, C, T = V.shape[0], 16, 6
    rng = np.random.default_rng(absorb)
    x = rng.normal(size=(N, C)).astype(np.float32)
    w3 = rng.normal(size=(3, C)).astype(np.float32)
    wt = rng.normal(size=(T, C)).astype(np.float32)
    mu = np.array([[1, 0, 0], [-1, 0, 0], [0, 1, 0], [0, -1, 0], [0, 0, 1], [0, 0, -1]], np.float32)
    inv_var = np.full(T, 3.0, np.float32)
    ctx = pk.Context(N, F.shape[0], 1, device=0)
    try:
        ctx.set_option(pk.PICASSO_OPT_ABSORB, absorb)
        print(f"pipeline N={N} F={F.shape[0]} absorb={absorb}", flush=True)
        h = _v2v(ctx, oracle, V, F, x, w3, wt, mu, inv_var)
        # decimation to a quarter, with the maps that pooling needs
        target = N // 4
        st, vo, fo, cid = ctx.picasso_decimate(dev(V), dev(F), target)
        ref = oracle.decimate(V, F, target, absorb=bool(absorb))
        assert st == ref["status"] == 0 and vo.shape[0] == target
        assert np.array_equal(cid.cpu().numpy(), ref["cluster_id"]) and np.array_equal(fo.cpu().numpy(), ref["facets"])
        assert np.array_equal(vo.cpu().numpy().view(np.uint32), ref["verts"].view(np.uint32))
        rep, mp = ctx.picasso_replace_mapping(cid, target)
        rep_r, mp_r = oracle.replace_mapping(ref["cluster_id"], target)
        assert np.array_equal(rep.cpu().numpy(), rep_r) and np.array_equal(mp.cpu().numpy(), mp_r)
        offc, mem = ctx.picasso_cluster_csr(cid, target)
        pooled, arg = ctx.picasso_pool_forward(pk.PICASSO_POOL_MAX, dev(h), offc, mem)
        p_ref, a_ref = oracle.pool_forward(oracle.POOL_MAX, h, ref["cluster_id"], target)
        assert np.array_equal(pooled.cpu().numpy(), p_ref) and np.array_equal(arg.cpu().numpy(), a_ref)
        # the same convolution on the coarse mesh, then back up
        h2 = _v2v(ctx, oracle, ref["verts"], ref["facets"], p_ref, w3, wt, mu, inv_var)
        up = ctx.picasso_unpool_forward(dev(h2), cid).cpu().numpy()
        assert np.array_equal(up, oracle.unpool_forward(h2, ref["cluster_id"]))
        assert np.array_equal(up[rep_r], up)  # every vertex carries its representative's feature
    finally:
        ctx.close()
