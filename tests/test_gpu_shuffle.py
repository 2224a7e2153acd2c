"""GPU parity of the seeded shuffle of equal-cost pairs (Sec. 3, footnote to the
sorting step; Sec. 5, augmentation) against the CPU oracle's same variant,
through the C-ABI: flat regions, where every cost ties, are where it acts.
Integer outputs bit-exact, positions bit-identical.
"""
import numpy as np
import pytest

from paper_2103_15076_amd import meshgen

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

SEEDS = [1, 0xDEADBEEF, 0x1234_5678_9ABC_DEF0]


@pytest.fixture(scope="module")
def pk():
    import paper_2103_15076_amd as p
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    p.load_library()
    return p


@pytest.fixture(scope="module")
def ctx(pk):
    c = pk.Context(1_300_000, 2_500_000, 8, device=0)
    yield c
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _meshes():
    yield "flat", meshgen.flat_grid(33, 18, spacing=0.5)
    yield "room", meshgen.room_scene(11, room=(3.0, 2.0, 1.5), n_boxes=5, spacing=0.05, jitter=0.0)
    yield "grid", meshgen.noisy_grid(40, 33, seed=5, noise=0.02)


def _same(st, vo, fo, cid, ref):
    assert st == ref["status"]
    vo, fo, cid = vo.cpu().numpy(), fo.cpu().numpy(), cid.cpu().numpy()
    assert vo.shape[0] == ref["verts"].shape[0], (vo.shape, ref["verts"].shape)
    assert fo.shape[0] == ref["facets"].shape[0], (fo.shape, ref["facets"].shape)
    assert np.array_equal(cid, ref["cluster_id"])
    assert np.array_equal(fo, ref["facets"])
    assert np.array_equal(vo.view(np.uint32), ref["verts"].view(np.uint32))


def _run(pk, ctx, seed, fn, absorb=0):
    ctx.set_option(pk.PICASSO_OPT_SHUFFLE_SEED, seed)
    ctx.set_option(pk.PICASSO_OPT_ABSORB, absorb)
    try:
        return fn()
    finally:
        ctx.set_option(pk.PICASSO_OPT_SHUFFLE_SEED, 0)
        ctx.set_option(pk.PICASSO_OPT_ABSORB, 0)


@pytest.mark.parametrize("name,mesh", list(_meshes()), ids=lambda x: x if isinstance(x, str) else "")
@pytest.mark.parametrize("seed", SEEDS)
@pytest.mark.parametrize("frac", [0.8, 0.5, 0.2])
def test_decimate_with_shuffle_matches_oracle(pk, ctx, oracle, name, mesh, seed, frac):
    V, F = mesh
    target = max(1, int(V.shape[0] * frac))
    print(f"shuffle {name} N={V.shape[0]} target={target} seed={seed:#x}", flush=True)
    st, vo, fo, cid = _run(pk, ctx, seed, lambda: ctx.picasso_decimate(dev(V), dev(F), target))
    ref = oracle.decimate(V, F, target, shuffle_seed=seed)
    _same(st, vo, fo, cid, ref)
    if name == "flat":
        assert not np.array_equal(ref["cluster_id"], oracle.decimate(V, F, target)["cluster_id"])


@pytest.mark.parametrize("block_max", [0, 1 << 15], ids=["sorted", "per_mesh_select"])
@pytest.mark.parametrize("absorb", [0, 1])
def test_budget_steps_under_the_shuffle_both_ways(pk, ctx, oracle, block_max, absorb):
    """Where the budget ends inside a run of equal costs the tie-break decides who stays: by the
    per-mesh selection and by the sort, for the pairs and for the vertices of line 11."""
    ctx.set_option(pk.PICASSO_OPT_TRUNC_BLOCK_MAX, block_max)
    try:
        for name, (V, F) in _meshes():
            for frac in (0.9, 0.62, 0.48):
                target = int(V.shape[0] * frac)
                print(f"shuffle budget {name} target={target} block_max={block_max} absorb={absorb}", flush=True)
                st, vo, fo, cid = _run(pk, ctx, 77, lambda: ctx.picasso_decimate(dev(V), dev(F), target), absorb)
                _same(st, vo, fo, cid, oracle.decimate(V, F, target, shuffle_seed=77, absorb=bool(absorb)))
    finally:
        ctx.set_option(pk.PICASSO_OPT_TRUNC_BLOCK_MAX, 1 << 15)


def test_batch_with_shuffle_equals_the_meshes_one_by_one_with_their_own_numbering(pk, ctx, oracle):
    """In a batch the tie-break sees the batch's edge numbering, so the reference is the oracle on
    the concatenated mesh as ONE mesh per budget share: here every mesh is given a budget it meets
    in the same number of runs, and the comparison is made on a batch of one mesh per call."""
    for i, (V, F) in enumerate([meshgen.flat_grid(21, 17, spacing=0.25), meshgen.noisy_grid(30, 22, seed=1)]):
        tg = V.shape[0] // 3
        st, vo, fo, cid, nvo, nfo = _run(
            pk, ctx, 5 + i, lambda: ctx.picasso_decimate_batch(dev(V), dev(F), [V.shape[0]], [F.shape[0]], [tg]))
        ref = oracle.decimate(V, F, tg, shuffle_seed=5 + i)
        _same(st, vo, fo, cid, ref)


@pytest.mark.parametrize("name", ["room115k", "scene1p2m"])
@pytest.mark.parametrize("absorb", [0, 1])
def test_config_full_size_with_shuffle(pk, ctx, oracle, name, absorb):
    c = meshgen.config(name)
    V, F, target = c["verts"], c["facets"], int(c["target"][0])
    print(f"shuffle config {name}: N={V.shape[0]} absorb={absorb}", flush=True)
    st, vo, fo, cid = _run(pk, ctx, 0xC0FFEE, lambda: ctx.picasso_decimate(dev(V), dev(F), target), absorb)
    print("  gpu done; oracle...", flush=True)
    _same(st, vo, fo, cid, oracle.decimate(V, F, target, shuffle_seed=0xC0FFEE, absorb=bool(absorb)))


def test_seed_zero_is_the_default_path(pk, ctx, oracle):
    V, F = meshgen.flat_grid(33, 18, spacing=0.5)
    st, vo, fo, cid = _run(pk, ctx, 0, lambda: ctx.picasso_decimate(dev(V), dev(F), V.shape[0] // 4))
    _same(st, vo, fo, cid, oracle.decimate(V, F, V.shape[0] // 4))


def test_batch_with_shuffle_meets_every_budget_and_is_reproducible(pk, ctx):
    """With several meshes in a batch the tie-break runs over the batch's edge numbering, so there is
    no per-mesh reference; what must hold: every mesh meets its budget exactly, the clusters of a
    mesh stay inside it, the same seed gives the same bytes, another seed other clusters."""
    parts = [meshgen.flat_grid(21, 17, spacing=0.25), meshgen.noisy_grid(30, 22, seed=1),
             meshgen.flat_grid(15, 15, spacing=0.5), meshgen.icosphere(3, seed=2)]
    nv = [p[0].shape[0] for p in parts]
    nf = [p[1].shape[0] for p in parts]
    off = np.cumsum([0] + nv)
    V = np.concatenate([p[0] for p in parts])
    F = np.concatenate([p[1] + off[i] for i, p in enumerate(parts)]).astype(np.int32)
    tg = [nv[0] // 3, nv[1] // 2, nv[2] // 4, nv[3] // 5]
    runs = {}
    for seed in (11, 11, 12):
        for absorb in (0, 1):
            st, vo, fo, cid, nvo, nfo = _run(pk, ctx, seed, lambda: ctx.picasso_decimate_batch(dev(V), dev(F), nv, nf, tg), absorb)
            assert st == 0 and nvo.tolist() == tg
            cid = cid.cpu().numpy()
            oo = np.cumsum([0] + tg)
            for i in range(4):
                part = cid[off[i]:off[i + 1]]
                assert part.min() == oo[i] and part.max() == oo[i + 1] - 1 and np.unique(part).size == tg[i]
            key = (seed, absorb)
            if key in runs:
                assert np.array_equal(runs[key][0], cid) and np.array_equal(runs[key][1], vo.cpu().numpy())
            runs[key] = (cid, vo.cpu().numpy())
    assert not np.array_equal(runs[(11, 0)][0], runs[(12, 0)][0])


@pytest.mark.parametrize("seed", [0, 77])
@pytest.mark.parametrize("absorb", [0, 1])
def test_budget_ends_inside_thousands_of_equal_costs(pk, ctx, oracle, seed, absorb):
    """A flat lattice (every cost is exactly zero) beside a jittered one: the budget step has to pick
    1,500 and then 5,000 of many thousands of pairs with one and the same cost key, more than the
    search hands to a single wave, by edge order (seed 0) or by the seeded tie-break."""
    Va, Fa = meshgen.flat_grid(150, 120, spacing=0.1)
    Vb, Fb = meshgen.noisy_grid(60, 50, seed=3, noise=0.02)
    V = np.concatenate([Va, Vb + np.float32(40.0)])
    F = np.concatenate([Fa, Fb + Va.shape[0]]).astype(np.int32)
    for drop in (1500, 5000, 9000):
        target = V.shape[0] - drop
        print(f"equal costs: N={V.shape[0]} target={target} seed={seed} absorb={absorb}", flush=True)
        st, vo, fo, cid = _run(pk, ctx, seed, lambda: ctx.picasso_decimate(dev(V), dev(F), target), absorb)
        _same(st, vo, fo, cid, oracle.decimate(V, F, target, shuffle_seed=seed, absorb=bool(absorb)))
