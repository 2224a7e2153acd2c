"""CPU oracle for the Picasso decimation path -- TEST INFRASTRUCTURE ONLY.

ctypes front end of ``picasso_oracle.cpp`` (host pointers, numpy arrays).
Nothing in the product package imports this; only tests, the smoke check and
the benchmark's cpu_baseline leg do.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "picasso_oracle.cpp"), os.path.join(_HERE, "picasso_pool_oracle.cpp"),
         os.path.join(_HERE, "picasso_conv_oracle.cpp")]
_LIB = os.path.join(_HERE, "libpicasso_oracle.so")
_lib = None

OK = 0
WARN_BUDGET_UNMET = 1
ERR_INVALID_ARG = -1
ERR_BAD_INDEX = -2
ERR_NONFINITE = -3

PLACE_MEAN, PLACE_INVERSE = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with strict IEEE fp32 semantics (no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(p) for p in _SRCS):
        cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
               "-o", _LIB] + _SRCS
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.picasso_oracle_cost_key.restype = ctypes.c_uint32
        _lib.picasso_oracle_cost_key.argtypes = [ctypes.c_float]
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def facet_quadrics(verts, facets):
    verts, facets = _f32(verts), _i32(facets)
    out = np.empty((facets.shape[0], 10), np.float32)
    lib().picasso_oracle_facet_quadrics(_p(verts), verts.shape[0], _p(facets), facets.shape[0], _p(out))
    return out


def vertex_quadrics(verts, facets):
    verts, facets = _f32(verts), _i32(facets)
    out = np.empty((verts.shape[0], 10), np.float32)
    lib().picasso_oracle_vertex_quadrics(_p(verts), verts.shape[0], _p(facets), facets.shape[0], _p(out))
    return out


def edges(facets):
    facets = _i32(facets)
    out = np.empty((max(1, 3 * facets.shape[0]), 2), np.int32)
    n = ctypes.c_int32(0)
    lib().picasso_oracle_edges(_p(facets), facets.shape[0], _p(out), ctypes.byref(n))
    return out[: n.value].copy()


def edge_costs(pos, Q, edge_list, placement=PLACE_MEAN, rcond_min=0.0):
    pos, Q, edge_list = _f32(pos), _f32(Q), _i32(edge_list)
    E = edge_list.shape[0]
    cost = np.empty(E, np.float32)
    key = np.empty(E, np.uint32)
    if placement == PLACE_MEAN:
        lib().picasso_oracle_edge_costs(_p(pos), _p(Q), _p(edge_list), E, _p(cost), _p(key))
    else:
        lib().picasso_oracle_edge_costs_opts(_p(pos), _p(Q), _p(edge_list), E, int(placement),
                                             ctypes.c_float(rcond_min), _p(cost), _p(key))
    return cost, key


def pair_target(quadric_sum, pu, pv, placement, rcond_min):
    """Contraction target of one pair: returns (target[3], rcond, used_inverse)."""
    q, pu, pv = _f32(quadric_sum), _f32(pu), _f32(pv)
    t = np.zeros(3, np.float32)
    rc = ctypes.c_float(0.0)
    used = ctypes.c_int32(0)
    lib().picasso_oracle_pair_target(_p(q), _p(pu), _p(pv), int(placement), ctypes.c_float(rcond_min), _p(t),
                                     ctypes.byref(rc), ctypes.byref(used))
    return t, float(rc.value), bool(used.value)


def cost_key(c: float) -> int:
    return int(lib().picasso_oracle_cost_key(ctypes.c_float(c)))


def select(edge_list, key, n_verts, n_remove):
    edge_list = _i32(edge_list)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    sel = np.zeros(edge_list.shape[0], np.uint8)
    n = lib().picasso_oracle_select(_p(edge_list), _p(key), edge_list.shape[0], int(n_verts), int(n_remove), _p(sel))
    return sel.astype(bool), n


def select_absorb(edge_list, key, n_verts, n_remove):
    """Alg. 2 lines 3-11 (line 11 under the budget): (selected[E], via[N], vertices removed)."""
    edge_list = _i32(edge_list)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    sel = np.zeros(edge_list.shape[0], np.uint8)
    via = np.full(int(n_verts), -1, np.int32)
    n = lib().picasso_oracle_select_absorb(_p(edge_list), _p(key), edge_list.shape[0], int(n_verts), int(n_remove),
                                           _p(sel), _p(via))
    return sel.astype(bool), via, n


def tie_break(seed, i):
    f = lib().picasso_oracle_tie_break
    f.restype = ctypes.c_uint32
    f.argtypes = [ctypes.c_uint64, ctypes.c_uint32]
    return int(f(int(seed), int(i)))


def select_shuffled(edge_list, key, n_verts, n_remove, seed, absorb=False):
    """Alg. 2 lines 3-10 (and 11 with absorb) with equal keys visited in the order of tie_break(seed, index)."""
    edge_list = _i32(edge_list)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    sel = np.zeros(edge_list.shape[0], np.uint8)
    via = np.full(int(n_verts), -1, np.int32)
    f = lib().picasso_oracle_select_shuffled
    f.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_uint64,
                  ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
    n = f(_p(edge_list), _p(key), edge_list.shape[0], int(n_verts), int(n_remove), int(seed), int(bool(absorb)),
          _p(sel), _p(via))
    return sel.astype(bool), via, n


def drop_unreferenced(res, nv=None):
    """Removes the output vertices that no output facet refers to from a decimate / decimate_batch result
    (in a copy): cluster ids of dropped clusters become -1; nv = per-mesh vertex counts of a batch."""
    verts, facets, cid = _f32(res["verts"]).copy(), _i32(res["facets"]).reshape(-1, 3).copy(), _i32(res["cluster_id"]).copy()
    nvo = _i32([verts.shape[0]] if nv is None else nv).copy()
    st = lib().picasso_oracle_drop_unreferenced(_p(verts), _p(facets), facets.shape[0], _p(cid), cid.shape[0],
                                                nvo.shape[0], _p(nvo))
    if st != 0:
        raise ValueError(f"oracle status {st}")
    out = dict(res)
    out.update(verts=verts[: int(nvo.sum())].copy(), facets=facets, cluster_id=cid)
    if nv is not None:
        out["nv"] = nvo
    return out


def decimate(verts, facets, target_nv, max_rounds=-1, return_quadrics=False, placement=PLACE_MEAN, rcond_min=0.0,
             absorb=False, shuffle_seed=0):
    """Returns dict(status, verts, facets, cluster_id, rounds[, quadrics])."""
    verts, facets = _f32(verts), _i32(facets).reshape(-1, 3)
    N, F = verts.shape[0], facets.shape[0]
    vo = np.zeros((max(N, 1), 3), np.float32)
    fo = np.zeros((max(F, 1), 3), np.int32)
    cid = np.zeros(max(N, 1), np.int32)
    qo = np.zeros((max(N, 1), 10), np.float32)
    nv, nf, rounds = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int32(0)
    if placement != PLACE_MEAN or absorb or shuffle_seed:
        st = lib().picasso_oracle_decimate_opts(
            _p(verts), N, _p(facets), F, int(target_nv), int(max_rounds), int(placement), ctypes.c_float(rcond_min),
            int(bool(absorb)), ctypes.c_uint64(int(shuffle_seed)), _p(vo), _p(fo), _p(cid), ctypes.byref(nv),
            ctypes.byref(nf), ctypes.byref(rounds), _p(qo))
    else:
        st = lib().picasso_oracle_decimate_rounds(
            _p(verts), N, _p(facets), F, int(target_nv), int(max_rounds), _p(vo), _p(fo), _p(cid),
            ctypes.byref(nv), ctypes.byref(nf), ctypes.byref(rounds), _p(qo))
    if st < 0:
        return dict(status=st)
    res = dict(status=st, verts=vo[: nv.value].copy(), facets=fo[: nf.value].copy(), cluster_id=cid[:N].copy(),
               rounds=rounds.value)
    if return_quadrics:
        res["quadrics"] = qo[: nv.value].copy()
    return res


def replace_mapping(cluster_id, n_out):
    """(replace[n_in], mapping[n_in]) of Alg. 2's output list, from cluster_id."""
    cluster_id = _i32(cluster_id)
    n_in = cluster_id.shape[0]
    rep = np.zeros(n_in, np.int32)
    mp = np.zeros(n_in, np.int32)
    st = lib().picasso_oracle_replace_mapping(_p(cluster_id), n_in, int(n_out), _p(rep), _p(mp))
    if st != 0:
        raise ValueError(f"oracle status {st}")
    return rep, mp


def decimate_batch(verts, facets, nv_in, nf_in, target_nv):
    verts, facets = _f32(verts), _i32(facets).reshape(-1, 3)
    nv_in, nf_in, target_nv = _i32(nv_in), _i32(nf_in), _i32(target_nv)
    B = nv_in.shape[0]
    N, F = verts.shape[0], facets.shape[0]
    vo = np.zeros((max(N, 1), 3), np.float32)
    fo = np.zeros((max(F, 1), 3), np.int32)
    cid = np.zeros(max(N, 1), np.int32)
    nvo = np.zeros(B, np.int32)
    nfo = np.zeros(B, np.int32)
    st = lib().picasso_oracle_decimate_batch(B, _p(verts), _p(facets), _p(nv_in), _p(nf_in), _p(target_nv),
                                             _p(vo), _p(fo), _p(cid), _p(nvo), _p(nfo))
    if st < 0:
        return dict(status=st)
    return dict(status=st, verts=vo[: int(nvo.sum())].copy(), facets=fo[: int(nfo.sum())].copy(),
                cluster_id=cid[:N].copy(), nv=nvo, nf=nfo)


# ---- pooling / unpooling over the recorded clusters (Sec. 3, "Pooling and unpooling")

POOL_AVG, POOL_MAX, POOL_WEIGHTED, POOL_SUM = 0, 1, 2, 3


def pool_forward(mode, x, cluster_id, n_out, weight=None):
    """Returns y[n_out, C] (and argmax[n_out, C] for max pooling)."""
    x, cluster_id = _f32(x), _i32(cluster_id)
    n_in, C = x.shape
    y = np.zeros((n_out, C), np.float32)
    arg = np.full((n_out, C), -1, np.int32)
    w = _f32(weight) if weight is not None else None
    st = lib().picasso_oracle_pool_forward(int(mode), _p(x), n_in, C, _p(cluster_id), int(n_out),
                                           _p(w) if w is not None else None, _p(y), _p(arg))
    if st != 0:
        raise ValueError(f"oracle status {st}")
    return (y, arg) if mode == POOL_MAX else y


def pool_backward(mode, gy, cluster_id, n_in, weight=None, argmax=None):
    gy, cluster_id = _f32(gy), _i32(cluster_id)
    n_out, C = gy.shape
    gx = np.zeros((n_in, C), np.float32)
    w = _f32(weight) if weight is not None else None
    a = _i32(argmax) if argmax is not None else None
    st = lib().picasso_oracle_pool_backward(int(mode), _p(gy), int(n_in), C, _p(cluster_id), n_out,
                                            _p(w) if w is not None else None, _p(a) if a is not None else None, _p(gx))
    if st != 0:
        raise ValueError(f"oracle status {st}")
    return gx


def unpool_forward(y, cluster_id):
    y, cluster_id = _f32(y), _i32(cluster_id)
    n_out, C = y.shape
    x = np.zeros((cluster_id.shape[0], C), np.float32)
    st = lib().picasso_oracle_unpool_forward(_p(y), cluster_id.shape[0], C, _p(cluster_id), n_out, _p(x))
    if st != 0:
        raise ValueError(f"oracle status {st}")
    return x


def unpool_backward(gx, cluster_id, n_out):
    gx, cluster_id = _f32(gx), _i32(cluster_id)
    n_in, C = gx.shape
    gy = np.zeros((n_out, C), np.float32)
    st = lib().picasso_oracle_unpool_backward(_p(gx), n_in, C, _p(cluster_id), int(n_out), _p(gy))
    if st != 0:
        raise ValueError(f"oracle status {st}")
    return gy


# ---- mesh convolutions, depth-wise (Sec. 4 "Mesh Convolution"; supplementary, backward propagations); fp64 results


def _check(st):
    if st != 0:
        raise ValueError(f"oracle status {st}")


def facet_geometry(verts, facets):
    """(normals float32[F,3], areas float32[F])."""
    verts, facets = _f32(verts), _i32(facets).reshape(-1, 3)
    F = facets.shape[0]
    n, a = np.zeros((F, 3), np.float32), np.zeros(F, np.float32)
    _check(lib().picasso_oracle_facet_geometry(_p(verts), verts.shape[0], _p(facets), F, _p(n), _p(a)))
    return n, a


def facet_levels(areas, foff=None, alpha=1, beta=1):
    areas = _f32(areas)
    foff = _i32([0, areas.shape[0]] if foff is None else foff)
    lev = np.zeros(areas.shape[0], np.int32)
    _check(lib().picasso_oracle_facet_levels(_p(areas), foff.shape[0] - 1, _p(foff), int(alpha), int(beta), _p(lev)))
    return lev


def fuzzy(normals, mu, inv_var):
    normals = _f32(normals)
    mu, inv_var = _f32(mu), _f32(inv_var)
    T = mu.shape[0]
    pi = np.zeros((normals.shape[0], T))
    _check(lib().picasso_oracle_fuzzy(_p(normals), normals.shape[0], _p(mu), _p(inv_var), T, _p(pi)))
    return pi


def v2f_forward(x, facets, level, w):
    x, facets, level, w = _f32(x), _i32(facets).reshape(-1, 3), _i32(level), _f32(w)
    N, C = x.shape
    y = np.zeros((facets.shape[0], C))
    _check(lib().picasso_oracle_v2f_forward(_p(x), N, C, _p(facets), facets.shape[0], _p(level), _p(w), _p(y)))
    return y


def v2f_backward(gy, x, facets, level, w):
    gy, x, facets, level, w = _f32(gy), _f32(x), _i32(facets).reshape(-1, 3), _i32(level), _f32(w)
    N, C = x.shape
    gx, gw = np.zeros((N, C)), np.zeros((3, C))
    _check(lib().picasso_oracle_v2f_backward(_p(gy), _p(x), N, C, _p(facets), facets.shape[0], _p(level), _p(w),
                                             _p(gx), _p(gw)))
    return gx, gw


def f2v_forward(y, pi, w, facets, n_verts):
    y, pi, w, facets = _f32(y), _f32(pi), _f32(w), _i32(facets).reshape(-1, 3)
    F, C = y.shape
    T = pi.shape[1]
    x = np.zeros((int(n_verts), C))
    _check(lib().picasso_oracle_f2v_forward(_p(y), F, C, _p(pi), T, _p(w), _p(facets), int(n_verts), _p(x)))
    return x


def f2v_backward(gx, y, pi, w, facets):
    gx, y, pi, w, facets = _f32(gx), _f32(y), _f32(pi), _f32(w), _i32(facets).reshape(-1, 3)
    F, C = y.shape
    T = pi.shape[1]
    gy, gw, gpi = np.zeros((F, C)), np.zeros((T, C)), np.zeros((F, T))
    _check(lib().picasso_oracle_f2v_backward(_p(gx), _p(y), F, C, _p(pi), T, _p(w), _p(facets), gx.shape[0], _p(gy),
                                             _p(gw), _p(gpi)))
    return gy, gw, gpi


def vertex_corner_csr(facets, n_verts):
    facets = _i32(facets).reshape(-1, 3)
    off = np.zeros(int(n_verts) + 1, np.int32)
    cor = np.zeros(max(1, 3 * facets.shape[0]), np.int32)
    _check(lib().picasso_oracle_vertex_corner_csr(_p(facets), facets.shape[0], int(n_verts), _p(off), _p(cor)))
    return off, cor[: 3 * facets.shape[0]]


def f2f_forward(tex, bary, poff, w):
    tex, bary, poff, w = _f32(tex), _f32(bary), _i32(poff), _f32(w)
    F, C = poff.shape[0] - 1, tex.shape[1]
    y = np.zeros((F, C))
    _check(lib().picasso_oracle_f2f_forward(_p(tex), _p(bary), _p(poff), F, C, _p(w), _p(y)))
    return y


def f2f_backward(gy, tex, bary, poff, w):
    gy, tex, bary, poff, w = _f32(gy), _f32(tex), _f32(bary), _i32(poff), _f32(w)
    F, C = poff.shape[0] - 1, tex.shape[1]
    gtex, gw = np.zeros(tex.shape), np.zeros((3, C))
    _check(lib().picasso_oracle_f2f_backward(_p(gy), _p(tex), _p(bary), _p(poff), F, C, _p(w), _p(gtex), _p(gw)))
    return gtex, gw
