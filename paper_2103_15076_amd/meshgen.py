"""Seeded synthetic triangle-mesh generators (inputs only; none of the method's arithmetic).

These stand in for the room-scale scan meshes the paper measures on (Sec. 5.2,
"Mesh Simplification Efficiency": 10K..1157K vertices, facets ~= 2x vertices).
Both the CPU oracle's tests and the HIP path's tests/bench take their inputs
from here, so that the two sides see identical bytes.

Every generator returns ``(verts float32[N,3], facets int32[F,3])`` as
C-contiguous numpy arrays and is a pure function of its arguments.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "grid_patch",
    "noisy_grid",
    "flat_grid",
    "icosphere",
    "room_scene",
    "room_scene_sized",
    "room_batch",
    "config",
    "CONFIG_NAMES",
]


def grid_patch(nu: int, nv: int):
    """Index pattern of an ``nu`` x ``nv`` vertex lattice: vertex id = j*nu + i.

    Each cell (i,j) is split along the v00-v11 diagonal into
    (v00, v10, v11) and (v00, v11, v01).
    """
    i, j = np.meshgrid(np.arange(nu - 1), np.arange(nv - 1), indexing="xy")
    v00 = (j * nu + i).ravel()
    v10 = v00 + 1
    v01 = v00 + nu
    v11 = v01 + 1
    f = np.empty((v00.size, 2, 3), dtype=np.int64)
    f[:, 0, 0] = v00
    f[:, 0, 1] = v10
    f[:, 0, 2] = v11
    f[:, 1, 0] = v00
    f[:, 1, 1] = v11
    f[:, 1, 2] = v01
    return f.reshape(-1, 3)


def noisy_grid(w: int = 64, h: int = 64, seed: int = 1001, noise: float = 0.002):
    """Height field on [0,1]^2: z = 0.05 sin(6x) cos(6y) + N(0, noise)."""
    rng = np.random.default_rng(seed)
    x = np.linspace(0.0, 1.0, w)
    y = np.linspace(0.0, 1.0, h)
    X, Y = np.meshgrid(x, y, indexing="xy")
    Z = 0.05 * np.sin(6.0 * X) * np.cos(6.0 * Y) + rng.normal(0.0, noise, size=X.shape)
    verts = np.stack([X.ravel(), Y.ravel(), Z.ravel()], axis=1).astype(np.float32)
    facets = grid_patch(w, h).astype(np.int32)
    return np.ascontiguousarray(verts), np.ascontiguousarray(facets)


def flat_grid(w: int, h: int, spacing: float = 1.0):
    """Exactly planar lattice in z = 0 with integer-multiple coordinates."""
    X, Y = np.meshgrid(np.arange(w) * spacing, np.arange(h) * spacing, indexing="xy")
    verts = np.stack([X.ravel(), Y.ravel(), np.zeros(X.size)], axis=1).astype(np.float32)
    return np.ascontiguousarray(verts), np.ascontiguousarray(grid_patch(w, h).astype(np.int32))


def icosphere(level: int = 6, seed: int | None = 1002, jitter: float = 0.01):
    """Icosahedron with ``level`` 1->4 midpoint splits, projected to the unit
    sphere, radius scaled by 1 + U(-jitter, jitter).  Midpoints are numbered in
    ascending order of their (lo, hi) parent edge, after all existing vertices.
    """
    t = (1.0 + 5.0 ** 0.5) / 2.0
    v = np.array(
        [[-1, t, 0], [1, t, 0], [-1, -t, 0], [1, -t, 0],
         [0, -1, t], [0, 1, t], [0, -1, -t], [0, 1, -t],
         [t, 0, -1], [t, 0, 1], [-t, 0, -1], [-t, 0, 1]], dtype=np.float64)
    f = np.array(
        [[0, 11, 5], [0, 5, 1], [0, 1, 7], [0, 7, 10], [0, 10, 11],
         [1, 5, 9], [5, 11, 4], [11, 10, 2], [10, 7, 6], [7, 1, 8],
         [3, 9, 4], [3, 4, 2], [3, 2, 6], [3, 6, 8], [3, 8, 9],
         [4, 9, 5], [2, 4, 11], [6, 2, 10], [8, 6, 7], [9, 8, 1]], dtype=np.int64)
    v /= np.linalg.norm(v, axis=1, keepdims=True)
    for _ in range(level):
        n = v.shape[0]
        a = f[:, [0, 1, 2]].ravel()
        b = f[:, [1, 2, 0]].ravel()
        lo = np.minimum(a, b)
        hi = np.maximum(a, b)
        key = lo * n + hi
        uniq, inv = np.unique(key, return_inverse=True)
        mid = 0.5 * (v[uniq // n] + v[uniq % n])
        mid /= np.linalg.norm(mid, axis=1, keepdims=True)
        v = np.concatenate([v, mid], axis=0)
        m = (n + inv).reshape(-1, 3)  # m[:,0]=mid(01), m[:,1]=mid(12), m[:,2]=mid(20)
        a0, a1, a2 = f[:, 0], f[:, 1], f[:, 2]
        f = np.concatenate(
            [np.stack([a0, m[:, 0], m[:, 2]], 1),
             np.stack([a1, m[:, 1], m[:, 0]], 1),
             np.stack([a2, m[:, 2], m[:, 1]], 1),
             np.stack([m[:, 0], m[:, 1], m[:, 2]], 1)], axis=0)
    if seed is not None and jitter > 0:
        rng = np.random.default_rng(seed)
        v = v * (1.0 + rng.uniform(-jitter, jitter, size=(v.shape[0], 1)))
    return np.ascontiguousarray(v.astype(np.float32)), np.ascontiguousarray(f.astype(np.int32))


def _cells(length, h):
    """Lattice cells along an edge of this length at spacing about h."""
    return max(1, int(np.ceil(length / h)))


def _box_surface(lo, size, h, with_bottom):
    """Lattice over the faces of an axis-aligned box, welded along the box's edges: every face is a
    regular patch (cells split like ``grid_patch``), and lattice points shared by two or three faces
    are one vertex.  Faces: top, y = y0, y = y1, x = x0, x = x1 and, with ``with_bottom``, the bottom.
    Vertices are numbered in the order in which the faces first reach them.
    Returns (points float64[n,3], facets int64[m,3])."""
    n = [_cells(size[d], h) for d in range(3)]
    ax = [np.linspace(0.0, size[d], n[d] + 1) + lo[d] for d in range(3)]
    specs = [(2, n[2]), (1, 0), (1, n[1]), (0, 0), (0, n[0])] + ([(2, 0)] if with_bottom else [])
    ijk, tris, base = [], [], 0
    for d, val in specs:
        u, v = [a for a in range(3) if a != d]
        nu, nv = n[u] + 1, n[v] + 1
        I, J = np.meshgrid(np.arange(nu), np.arange(nv), indexing="xy")
        idx = np.zeros((I.size, 3), np.int64)
        idx[:, u] = I.ravel()
        idx[:, v] = J.ravel()
        idx[:, d] = val
        ijk.append(idx)
        tris.append(grid_patch(nu, nv) + base)
        base += I.size
    ijk = np.concatenate(ijk, axis=0)
    tris = np.concatenate(tris, axis=0)
    key = (ijk[:, 0] * (n[1] + 1) + ijk[:, 1]) * (n[2] + 1) + ijk[:, 2]
    _, first, inv = np.unique(key, return_index=True, return_inverse=True)
    order = np.argsort(first, kind="stable")      # distinct points in order of first appearance
    rank = np.empty_like(order)
    rank[order] = np.arange(order.size)
    pick = ijk[first[order]]
    pts = np.stack([ax[0][pick[:, 0]], ax[1][pick[:, 1]], ax[2][pick[:, 2]]], axis=1)
    return pts, rank[inv.reshape(-1)][tris]


def _box_surface_counts(size, h, with_bottom):
    """(vertices, facets) of ``_box_surface`` without building it."""
    a, b, c = (_cells(size[d], h) + 1 for d in range(3))
    nv = 2 * (a * b + a * c + b * c) - 4 * (a + b + c) + 8
    nf = 4 * ((a - 1) * (b - 1) + (a - 1) * (c - 1) + (b - 1) * (c - 1))
    if not with_bottom:
        nv -= (a - 2) * (b - 2)
        nf -= 2 * (a - 1) * (b - 1)
    return nv, nf


def _scene_boxes(seed, room, n_boxes):
    """The room and its furniture: (rng, [(lo, size, with_bottom)]); the rng goes on to the jitter."""
    rng = np.random.default_rng(seed)
    rx, ry, rz = room
    boxes = [((0.0, 0.0, 0.0), (rx, ry, rz), True)]
    sizes = rng.uniform(0.3, 2.0, size=(n_boxes, 3))
    sizes[:, 2] = np.minimum(sizes[:, 2], rz)
    px = rng.uniform(0.0, 1.0, size=n_boxes) * (rx - sizes[:, 0])
    py = rng.uniform(0.0, 1.0, size=n_boxes) * (ry - sizes[:, 1])
    for k in range(n_boxes):
        boxes.append(((px[k], py[k], 0.0), tuple(sizes[k]), False))
    return rng, boxes


def room_scene(seed: int, room=(10.0, 8.0, 3.0), n_boxes: int = 40, spacing: float = 0.07,
               jitter: float = 0.003):
    """Box room (floor, ceiling, 4 walls: a closed surface) plus ``n_boxes`` axis-aligned furniture
    boxes (sizes U(0.3, 2.0) m per axis, standing on the floor, five faces each, open towards the
    floor).  The faces of one box are welded along its edges; boxes are not joined to the floor or to
    each other (separate components, intersecting surfaces, open boundaries: as in scanned rooms).
    Facets come to about twice the vertices, as in the paper's room meshes.  Per-coordinate vertex
    jitter N(0, jitter).
    """
    rng, boxes = _scene_boxes(seed, room, n_boxes)
    vs, fs, base = [], [], 0
    for lo, size, with_bottom in boxes:
        p, f = _box_surface(lo, size, spacing, with_bottom)
        vs.append(p)
        fs.append(f + base)
        base += p.shape[0]
    v = np.concatenate(vs, axis=0)
    f = np.concatenate(fs, axis=0)
    v = v + rng.normal(0.0, jitter, size=v.shape)
    return np.ascontiguousarray(v.astype(np.float32)), np.ascontiguousarray(f.astype(np.int32))


def _count_verts(seed, room, n_boxes, h):
    _, boxes = _scene_boxes(seed, room, n_boxes)
    return sum(_box_surface_counts(size, h, with_bottom)[0] for _, size, with_bottom in boxes)


def room_scene_sized(seed: int, n_target: int, room=(10.0, 8.0, 3.0), n_boxes: int = 40,
                     jitter: float = 0.003):
    """``room_scene`` with the lattice spacing solved (bisection) so that the
    vertex count lands within about 1 % of ``n_target``.  Returns
    (verts, facets, spacing)."""
    lo, hi = 1e-3, 2.0
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        if _count_verts(seed, room, n_boxes, mid) > n_target:
            lo = mid
        else:
            hi = mid
    v, f = room_scene(seed, room, n_boxes, hi, jitter)
    return v, f, hi


def room_batch(n_meshes: int = 16, n_target_each: int = 60000, seed0: int = 5000):
    """Concatenation of ``n_meshes`` room scenes (seeds seed0, seed0+1, ...) with
    global facet indices.  Returns (verts, facets, nv[B], nf[B])."""
    vs, fs, nvs, nfs, base = [], [], [], [], 0
    for k in range(n_meshes):
        v, f, _ = room_scene_sized(seed0 + k, n_target_each)
        vs.append(v)
        fs.append(f + base)
        nvs.append(v.shape[0])
        nfs.append(f.shape[0])
        base += v.shape[0]
    return (np.ascontiguousarray(np.concatenate(vs, 0)),
            np.ascontiguousarray(np.concatenate(fs, 0).astype(np.int32)),
            np.asarray(nvs, dtype=np.int32), np.asarray(nfs, dtype=np.int32))


CONFIG_NAMES = ("grid64", "icosphere6", "room115k", "scene1p2m", "batch16x60k")


def config(name: str):
    """The five benchmark workloads.  Returns a dict with verts, facets,
    nv[B], nf[B], target[B] (per mesh) and, for the batch, ``levels``."""
    if name == "grid64":
        v, f = noisy_grid(64, 64, seed=1001)
        tgt = [1024]
    elif name == "icosphere6":
        v, f = icosphere(6, seed=1002)
        tgt = [10240]
    elif name == "room115k":
        v, f, _ = room_scene_sized(1003, 115000)
        tgt = [41500]
    elif name == "scene1p2m":
        v, f, _ = room_scene_sized(1004, 1200000, room=(30.0, 20.0, 3.0), n_boxes=300)
        tgt = [v.shape[0] // 4]
    elif name == "batch16x60k":
        v, f, nv, nf = room_batch(16, 60000, 5000)
        return dict(name=name, verts=v, facets=f, nv=nv, nf=nf,
                    target=(nv.astype(np.int64) * 4 // 10).astype(np.int32), levels=4)
    else:
        raise KeyError(name)
    return dict(name=name, verts=v, facets=f,
                nv=np.asarray([v.shape[0]], np.int32), nf=np.asarray([f.shape[0]], np.int32),
                target=np.asarray(tgt, np.int32), levels=1)
