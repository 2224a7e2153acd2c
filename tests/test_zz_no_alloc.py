"""The entry point for callers that cannot allocate (picasso_replace_mapping_static: no context, its one
scratch table in a static device array of the library) against picasso_replace_mapping, through the
C-ABI, bit for bit: two calls in a row, the second on a smaller input (the static array keeps the
first call's contents), then a bad index, the size limit, a side stream and a call recorded into a HIP
graph and replayed.  The caller passes every tensor, outputs included."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def pk():
    import paper_2103_15076_amd as p
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    p.load_library()
    return p


def _cluster_ids(n_in, n_out, seed):
    rng = np.random.default_rng(seed)
    cid = rng.integers(0, n_out, size=n_in).astype(np.int32)
    cid[rng.permutation(n_in)[:n_out]] = np.arange(n_out, dtype=np.int32)   # every cluster has a member
    return cid


def _static(pk, cid_dev, n_out, stream=None):
    n_in = cid_dev.shape[0]
    rep = torch.full((n_in,), -7, dtype=torch.int32, device="cuda:0")
    mp = torch.full((n_in,), -7, dtype=torch.int32, device="cuda:0")
    status = torch.full((1,), 99, dtype=torch.int32, device="cuda:0")
    st = pk.picasso_replace_mapping_static(cid_dev, n_out, rep, mp, status, device=0, stream=stream)
    return st, rep, mp, status


def test_static_entry_point_matches_the_context_one_twice_in_a_row(pk):
    with pk.Context(700_000, 10, 1, device=0) as ctx:
        for n_in, n_out, seed in ((600_001, 211_003, 1), (5_000, 1_234, 2), (1, 1, 3), (70_000, 69_999, 4)):
            print(f"static replace/mapping n_in={n_in} n_out={n_out}", flush=True)
            cid = _cluster_ids(n_in, n_out, seed)
            d = torch.from_numpy(cid).to("cuda:0")
            st, rep, mp, status = _static(pk, d, n_out)
            assert st == pk.PICASSO_OK
            rep_ref, mp_ref = ctx.picasso_replace_mapping(d, n_out)
            torch.cuda.synchronize()
            assert int(status.item()) == pk.PICASSO_OK
            assert torch.equal(rep, rep_ref) and torch.equal(mp, mp_ref)
            # and what the tensors mean (first member represents; cluster_id = mapping o replace)
            r, m = rep.cpu().numpy(), mp.cpu().numpy()
            first = np.full(n_out, n_in, np.int64)
            np.minimum.at(first, cid, np.arange(n_in))
            assert np.array_equal(r, first[cid]) and np.array_equal(m[r], cid)


def test_static_entry_point_reports_a_bad_index_on_the_device_and_recovers(pk):
    cid = _cluster_ids(4_000, 900, 5)
    bad = cid.copy()
    bad[1234] = 900
    st, _, _, status = _static(pk, torch.from_numpy(bad).to("cuda:0"), 900)
    torch.cuda.synchronize()
    assert st == pk.PICASSO_OK and int(status.item()) == pk.PICASSO_ERR_BAD_INDEX
    bad[1234] = -2            # (-1 alone is legal: a vertex whose cluster was dropped)
    st, _, _, status = _static(pk, torch.from_numpy(bad).to("cuda:0"), 900)
    torch.cuda.synchronize()
    assert st == pk.PICASSO_OK and int(status.item()) == pk.PICASSO_ERR_BAD_INDEX
    # the flag does not stick
    st, rep, mp, status = _static(pk, torch.from_numpy(cid).to("cuda:0"), 900)
    torch.cuda.synchronize()
    assert st == pk.PICASSO_OK and int(status.item()) == pk.PICASSO_OK
    assert np.array_equal(mp.cpu().numpy()[rep.cpu().numpy()], cid)


def test_static_entry_point_rejects_what_it_cannot_hold(pk):
    d = torch.zeros(8, dtype=torch.int32, device="cuda:0")
    out = torch.zeros(8, dtype=torch.int32, device="cuda:0")
    status = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    f = pk.picasso_replace_mapping_static
    assert f(d, pk.PICASSO_STATIC_MAX_CLUSTERS + 1, out, out.clone(), status) == pk.PICASSO_ERR_WORKSPACE
    assert f(d, -1, out, out.clone(), status) == pk.PICASSO_ERR_INVALID_ARG
    assert f(d, 4, out, out.clone(), status, device=64) == pk.PICASSO_ERR_INVALID_ARG
    assert f(d, 4, out, out.clone(), status, device=-1) == pk.PICASSO_ERR_INVALID_ARG
    # the largest table it holds
    n_out = pk.PICASSO_STATIC_MAX_CLUSTERS
    cid = torch.arange(n_out, dtype=torch.int32, device="cuda:0")
    st, rep, mp, status = _static(pk, cid, n_out)
    torch.cuda.synchronize()
    assert st == pk.PICASSO_OK and int(status.item()) == 0
    assert torch.equal(rep, cid) and torch.equal(mp, cid)


def test_static_entry_point_on_a_side_stream_and_in_a_graph(pk):
    cid = _cluster_ids(50_000, 12_345, 6)
    d = torch.from_numpy(cid).to("cuda:0")
    st, rep0, mp0, _ = _static(pk, d, 12_345)          # eager result; also the address look-up, outside capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        st, rep, mp, status = _static(pk, d, 12_345, stream=side)
    side.synchronize()
    assert st == pk.PICASSO_OK and int(status.item()) == 0 and torch.equal(rep, rep0) and torch.equal(mp, mp0)
    # recorded once, replayed three times with eager calls on other inputs in between
    rep_g = torch.zeros_like(rep0)
    mp_g = torch.zeros_like(mp0)
    status_g = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        st = pk.picasso_replace_mapping_static(d, 12_345, rep_g, mp_g, status_g, device=0,
                                               stream=torch.cuda.current_stream())
    assert st == pk.PICASSO_OK
    other = torch.from_numpy(_cluster_ids(3_000, 77, 7)).to("cuda:0")
    for i in range(3):
        rep_g.fill_(-5)
        mp_g.fill_(-5)
        status_g.fill_(55)
        g.replay()
        torch.cuda.synchronize()
        assert int(status_g.item()) == 0 and torch.equal(rep_g, rep0) and torch.equal(mp_g, mp0), f"replay {i}"
        st, r2, m2, s2 = _static(pk, other, 77)        # eager work between the replays
        torch.cuda.synchronize()
        assert st == pk.PICASSO_OK and int(s2.item()) == 0
