"""Thin ctypes binding of include/picasso.h: argument marshalling only.

torch supplies device memory and the stream; every step of the path runs in
libpicasso_hip.so.  There is no fallback: if the library is missing or cannot
be loaded, ``load_library`` raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpicasso_hip.so")

PICASSO_OK = 0
PICASSO_WARN_BUDGET_UNMET = 1
PICASSO_ERR_INVALID_ARG = -1
PICASSO_ERR_BAD_INDEX = -2
PICASSO_ERR_NONFINITE = -3
PICASSO_ERR_WORKSPACE = -4
PICASSO_ERR_HIP = -5
PICASSO_ERR_INTERNAL = -6

PICASSO_OPT_MAX_ROUNDS = 0
PICASSO_OPT_STAGE_TIMING = 1
PICASSO_OPT_SUBROUND_BATCH = 2
PICASSO_OPT_KERNEL_TIMING = 3
PICASSO_OPT_OVERLAP = 4
PICASSO_OPT_TRUNC_BLOCK_MAX = 5
PICASSO_OPT_PLACEMENT = 6
PICASSO_OPT_RCOND_MIN_BITS = 7
PICASSO_OPT_ABSORB = 8
PICASSO_OPT_SHUFFLE_SEED = 9
PICASSO_OPT_HOST_POLL = 10
PICASSO_OPT_LAUNCH_AHEAD = 11
PICASSO_OPT_TRUNC_WIDTH = 12
PICASSO_OPT_DROP_DEGENERATED = 13
PICASSO_OPT_TRUNC_SELECT = 14
PICASSO_PLACE_MEAN, PICASSO_PLACE_INVERSE = 0, 1

(PICASSO_KERNEL_SORT, PICASSO_KERNEL_UNIQUE_COST, PICASSO_KERNEL_SUBROUND0, PICASSO_KERNEL_FACET_INSERT,
 PICASSO_KERNEL_QUADRIC_ROWS, PICASSO_KERNEL_SORT_INCIDENCE, PICASSO_KERNEL_COUNT) = range(7)
TIMED_KERNEL_NAMES = (
    "bucket_keys_kernel<u64> (edge-key sort, per-bucket LDS sort)",
    "tile_scatter_kernel<UniquePred, UniqueOut> (distinct edges, costs, first bids)",
    "select_subround_kernel (first sub-round of the selection)",
    "facet_insert_kernel (facet hash set, label compose)",
    "quadric_rows_kernel (vertex quadrics from facet planes)",
    "bucket_keys_kernel<u64> (incidence-key sort of the vertex quadrics, per-bucket LDS sort)",
)

PICASSO_STATS_ROUNDS = 32
PICASSO_ST_COUNT = 8
STAGE_NAMES = ("quadrics", "edges", "select", "contract", "facets")

EXPORTED_SYMBOLS = (
    "picasso_workspace_bytes", "picasso_create", "picasso_destroy", "picasso_set_option", "picasso_strerror",
    "picasso_last_hip_error", "picasso_decimate", "picasso_decimate_batch", "picasso_vertex_quadrics",
    "picasso_edge_costs", "picasso_radix_sort", "picasso_kernel_timing",
    "picasso_device_copy", "picasso_bucket_sort", "picasso_cluster_csr", "picasso_replace_mapping",
    "picasso_replace_mapping_static",
    "picasso_vertex_corner_csr", "picasso_facet_geometry", "picasso_fuzzy_coefficients", "picasso_v2f_forward",
    "picasso_v2f_backward", "picasso_f2f_forward", "picasso_f2f_backward", "picasso_f2v_forward",
    "picasso_f2v_backward", "picasso_pool_forward",
    "picasso_pool_backward", "picasso_unpool_forward", "picasso_unpool_backward",
)

PICASSO_POOL_AVG, PICASSO_POOL_MAX, PICASSO_POOL_WEIGHTED, PICASSO_POOL_SUM = 0, 1, 2, 3


class picasso_stats(ctypes.Structure):
    _fields_ = [
        ("rounds", ctypes.c_int32),
        ("nv_out", ctypes.c_int32),
        ("nf_out", ctypes.c_int32),
        ("nv", ctypes.c_int32 * PICASSO_STATS_ROUNDS),
        ("nf", ctypes.c_int32 * PICASSO_STATS_ROUNDS),
        ("ne", ctypes.c_int32 * PICASSO_STATS_ROUNDS),
        ("nsel", ctypes.c_int32 * PICASSO_STATS_ROUNDS),
        ("subrounds", ctypes.c_int32 * PICASSO_STATS_ROUNDS),
        ("ms_stage", (ctypes.c_float * PICASSO_ST_COUNT) * PICASSO_STATS_ROUNDS),
        ("ms_total", ctypes.c_float),
    ]

    def as_dict(self):
        r = min(self.rounds, PICASSO_STATS_ROUNDS)
        return dict(
            rounds=self.rounds, nv_out=self.nv_out, nf_out=self.nf_out, ms_total=self.ms_total,
            nv=list(self.nv[:r]), nf=list(self.nf[:r]), ne=list(self.ne[:r]), nsel=list(self.nsel[:r]),
            subrounds=list(self.subrounds[:r]),
            ms_stage=[{n: self.ms_stage[i][j] for j, n in enumerate(STAGE_NAMES)} for i in range(max(r, 1))],
        )


_lib = None


class PicassoError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"picasso status {status}: {msg}")
        self.status = status


def load_library():
    """Loads libpicasso_hip.so; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2103_15076_amd.build` "
            "(hipcc, gfx950).  There is no CPU fallback.")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.picasso_workspace_bytes.restype = ctypes.c_size_t
    lib.picasso_workspace_bytes.argtypes = [i64, i64, i32]
    lib.picasso_create.restype = ctypes.c_int
    lib.picasso_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64, i64, i32]
    lib.picasso_destroy.restype = None
    lib.picasso_destroy.argtypes = [vp]
    lib.picasso_set_option.restype = ctypes.c_int
    lib.picasso_set_option.argtypes = [vp, ctypes.c_int, i64]
    lib.picasso_strerror.restype = ctypes.c_char_p
    lib.picasso_strerror.argtypes = [ctypes.c_int]
    lib.picasso_last_hip_error.restype = ctypes.c_char_p
    lib.picasso_last_hip_error.argtypes = [vp]
    lib.picasso_decimate.restype = ctypes.c_int
    lib.picasso_decimate.argtypes = [vp, vp, vp, i32, vp, i32, i32, vp, vp, vp, ctypes.POINTER(i32),
                                     ctypes.POINTER(i32), ctypes.POINTER(picasso_stats)]
    lib.picasso_decimate_batch.restype = ctypes.c_int
    lib.picasso_decimate_batch.argtypes = [vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                           ctypes.POINTER(picasso_stats)]
    lib.picasso_vertex_quadrics.restype = ctypes.c_int
    lib.picasso_vertex_quadrics.argtypes = [vp, vp, vp, i32, vp, i32, vp]
    lib.picasso_edge_costs.restype = ctypes.c_int
    lib.picasso_edge_costs.argtypes = [vp, vp, vp, i32, vp, i32, vp, vp, ctypes.POINTER(i32)]
    lib.picasso_kernel_timing.restype = ctypes.c_int
    lib.picasso_kernel_timing.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.POINTER(i64),
                                          ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.picasso_device_copy.restype = ctypes.c_int
    lib.picasso_device_copy.argtypes = [vp, vp, vp, ctypes.c_size_t]
    lib.picasso_radix_sort.restype = ctypes.c_int
    lib.picasso_radix_sort.argtypes = [vp, vp, ctypes.c_int, vp, vp, i64, ctypes.c_int]
    lib.picasso_cluster_csr.restype = ctypes.c_int
    lib.picasso_cluster_csr.argtypes = [vp, vp, vp, i32, i32, vp, vp]
    lib.picasso_replace_mapping.restype = ctypes.c_int
    lib.picasso_replace_mapping.argtypes = [vp, vp, vp, i32, i32, vp, vp]
    lib.picasso_replace_mapping_static.restype = ctypes.c_int
    lib.picasso_replace_mapping_static.argtypes = [ctypes.c_int, vp, vp, i32, i32, vp, vp, vp]
    lib.picasso_vertex_corner_csr.restype = ctypes.c_int
    lib.picasso_vertex_corner_csr.argtypes = [vp, vp, vp, i32, i32, vp, vp]
    lib.picasso_facet_geometry.restype = ctypes.c_int
    lib.picasso_facet_geometry.argtypes = [vp, vp, vp, i32, vp, i32, i32, vp, i32, i32, vp, vp, vp]
    lib.picasso_fuzzy_coefficients.restype = ctypes.c_int
    lib.picasso_fuzzy_coefficients.argtypes = [vp, vp, vp, i32, vp, vp, i32, vp]
    lib.picasso_v2f_forward.restype = ctypes.c_int
    lib.picasso_v2f_forward.argtypes = [vp, vp, vp, i32, i32, vp, i32, vp, vp, vp]
    lib.picasso_v2f_backward.restype = ctypes.c_int
    lib.picasso_v2f_backward.argtypes = [vp, vp, vp, vp, i32, i32, vp, i32, vp, vp, vp, vp, vp, vp]
    lib.picasso_f2f_forward.restype = ctypes.c_int
    lib.picasso_f2f_forward.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, vp, vp]
    lib.picasso_f2f_backward.restype = ctypes.c_int
    lib.picasso_f2f_backward.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp]
    lib.picasso_f2v_forward.restype = ctypes.c_int
    lib.picasso_f2v_forward.argtypes = [vp, vp, vp, i32, i32, vp, i32, vp, vp, vp, i32, vp]
    lib.picasso_f2v_backward.restype = ctypes.c_int
    lib.picasso_f2v_backward.argtypes = [vp, vp, vp, vp, i32, i32, vp, i32, vp, vp, vp, i32, vp, vp, vp]
    lib.picasso_pool_forward.restype = ctypes.c_int
    lib.picasso_pool_forward.argtypes = [vp, vp, ctypes.c_int, vp, i32, i32, vp, vp, i32, vp, vp, vp]
    lib.picasso_pool_backward.restype = ctypes.c_int
    lib.picasso_pool_backward.argtypes = [vp, vp, ctypes.c_int, vp, i32, i32, vp, vp, vp, i32, vp, vp, vp]
    lib.picasso_unpool_forward.restype = ctypes.c_int
    lib.picasso_unpool_forward.argtypes = [vp, vp, vp, i32, i32, vp, vp]
    lib.picasso_unpool_backward.restype = ctypes.c_int
    lib.picasso_unpool_backward.argtypes = [vp, vp, vp, i32, i32, vp, vp, i32, vp]
    lib.picasso_bucket_sort.restype = ctypes.c_int
    lib.picasso_bucket_sort.argtypes = [vp, vp, ctypes.c_int, vp, vp, i64, ctypes.c_int]
    _lib = lib
    return lib


def picasso_strerror(status: int) -> str:
    return load_library().picasso_strerror(int(status)).decode()


def picasso_workspace_bytes(max_verts: int, max_facets: int, max_meshes: int = 1) -> int:
    return int(load_library().picasso_workspace_bytes(int(max_verts), int(max_facets), int(max_meshes)))


def _stream_ptr(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _dev_ptr(t, dtype, what):
    import torch
    if t is None:
        return ctypes.c_void_p(0)
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{what}: expected a contiguous CUDA tensor of dtype {dtype}")
    return ctypes.c_void_p(t.data_ptr())


def picasso_device_copy(dst, src, stream=None):
    """dst[:] = src with the library's plain copy kernel (both contiguous CUDA tensors of equal byte size)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes and dst.is_cuda and src.is_cuda
    st = load_library().picasso_device_copy(_stream_ptr(stream), ctypes.c_void_p(dst.data_ptr()),
                                            ctypes.c_void_p(src.data_ptr()), nbytes)
    if st != PICASSO_OK:
        raise PicassoError(st, picasso_strerror(st))


PICASSO_STATIC_MAX_CLUSTERS = 1 << 22


def picasso_replace_mapping_static(cluster_id, n_out, replace, mapping, status, device=0, stream=None):
    """picasso_replace_mapping for callers that cannot allocate: no context; every tensor, outputs
    (replace, mapping int32[n_in], status int32[1]) included, comes from the caller; asynchronous.
    Returns the call's own status (argument checks and launch errors); the bad-index verdict is left
    in ``status`` on the device."""
    import torch
    return int(load_library().picasso_replace_mapping_static(
        int(device), _stream_ptr(stream), _dev_ptr(cluster_id, torch.int32, "cluster_id"), int(cluster_id.shape[0]),
        int(n_out), _dev_ptr(replace, torch.int32, "replace"), _dev_ptr(mapping, torch.int32, "mapping"),
        _dev_ptr(status, torch.int32, "status")))


class Context:
    """Owns a picasso_ctx (device workspace sized at creation)."""

    def __init__(self, max_verts: int, max_facets: int, max_meshes: int = 1, device: int = 0):
        self._lib = load_library()
        self._h = ctypes.c_void_p(0)
        st = self._lib.picasso_create(ctypes.byref(self._h), int(device), int(max_verts), int(max_facets),
                                      int(max_meshes))
        if st != PICASSO_OK:
            raise PicassoError(st, picasso_strerror(st))
        self.max_verts, self.max_facets, self.max_meshes, self.device = max_verts, max_facets, max_meshes, device

    def close(self):
        if getattr(self, "_h", None) and self._h.value:
            self._lib.picasso_destroy(self._h)
            self._h = ctypes.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def set_option(self, option: int, value: int):
        st = self._lib.picasso_set_option(self._h, int(option), int(value))
        if st != PICASSO_OK:
            raise PicassoError(st, picasso_strerror(st))

    def set_placement(self, placement: int, rcond_min: float = 1e-3):
        """PICASSO_OPT_PLACEMENT and its binary32 threshold (passed on as a bit pattern)."""
        import struct
        self.set_option(PICASSO_OPT_RCOND_MIN_BITS, struct.unpack("<I", struct.pack("<f", float(rcond_min)))[0])
        self.set_option(PICASSO_OPT_PLACEMENT, placement)

    def picasso_kernel_timing(self, kernel, reset=False):
        """Totals for one of the bracketed kernels (PICASSO_KERNEL_*) while PICASSO_OPT_KERNEL_TIMING is on."""
        n, ms, by = ctypes.c_int64(0), ctypes.c_double(0.0), ctypes.c_double(0.0)
        st = self._lib.picasso_kernel_timing(self._h, int(kernel), int(bool(reset)), ctypes.byref(n), ctypes.byref(ms),
                                             ctypes.byref(by))
        if st != PICASSO_OK:
            self._raise(st)
        return dict(kernel=TIMED_KERNEL_NAMES[int(kernel)], launches=n.value, ms_total=ms.value, bytes_total=by.value)

    def last_hip_error(self) -> str:
        return self._lib.picasso_last_hip_error(self._h).decode()

    def _raise(self, st):
        msg = picasso_strerror(st)
        if st == PICASSO_ERR_HIP:
            msg += ": " + self.last_hip_error()
        raise PicassoError(st, msg)

    # -- the calls of include/picasso.h, same names ---------------------------------------------

    def picasso_decimate(self, verts, facets, target_nv, verts_out=None, facets_out=None, cluster_id=None,
                         stats=None, stream=None, check=True):
        """Returns (status, verts_out[:nv], facets_out[:nf], cluster_id).  Output
        tensors are allocated with torch when not supplied (capacity = input sizes)."""
        import torch
        N, F = int(verts.shape[0]), int(facets.shape[0])
        dev = verts.device
        if verts_out is None:
            verts_out = torch.empty((max(N, 1), 3), dtype=torch.float32, device=dev)
        if facets_out is None:
            facets_out = torch.empty((max(F, 1), 3), dtype=torch.int32, device=dev)
        if cluster_id is None:
            cluster_id = torch.empty((max(N, 1),), dtype=torch.int32, device=dev)
        nv, nf = ctypes.c_int32(0), ctypes.c_int32(0)
        st = self._lib.picasso_decimate(
            self._h, _stream_ptr(stream), _dev_ptr(verts, torch.float32, "verts"), N,
            _dev_ptr(facets, torch.int32, "facets"), F, int(target_nv),
            _dev_ptr(verts_out, torch.float32, "verts_out"), _dev_ptr(facets_out, torch.int32, "facets_out"),
            _dev_ptr(cluster_id, torch.int32, "cluster_id"), ctypes.byref(nv), ctypes.byref(nf),
            ctypes.byref(stats) if stats is not None else None)
        if st < 0:
            if check:
                self._raise(st)
            return st, None, None, None
        return st, verts_out[: nv.value], facets_out[: nf.value], cluster_id[:N]

    def picasso_decimate_batch(self, verts, facets, nv_in, nf_in, target_nv, verts_out=None, facets_out=None,
                               cluster_id=None, stats=None, stream=None, check=True):
        """nv_in / nf_in / target_nv: host int sequences [B].  Returns
        (status, verts_out[:sum nv], facets_out[:sum nf], cluster_id, nv_out[B], nf_out[B])."""
        import numpy as np
        import torch
        nv_in = np.ascontiguousarray(nv_in, dtype=np.int32)
        nf_in = np.ascontiguousarray(nf_in, dtype=np.int32)
        target_nv = np.ascontiguousarray(target_nv, dtype=np.int32)
        B = int(nv_in.shape[0])
        N, F = int(verts.shape[0]), int(facets.shape[0])
        dev = verts.device
        if verts_out is None:
            verts_out = torch.empty((max(N, 1), 3), dtype=torch.float32, device=dev)
        if facets_out is None:
            facets_out = torch.empty((max(F, 1), 3), dtype=torch.int32, device=dev)
        if cluster_id is None:
            cluster_id = torch.empty((max(N, 1),), dtype=torch.int32, device=dev)
        nvo = np.zeros(B, np.int32)
        nfo = np.zeros(B, np.int32)
        hp = lambda a: a.ctypes.data_as(ctypes.c_void_p)
        st = self._lib.picasso_decimate_batch(
            self._h, _stream_ptr(stream), B, _dev_ptr(verts, torch.float32, "verts"),
            _dev_ptr(facets, torch.int32, "facets"), hp(nv_in), hp(nf_in), hp(target_nv),
            _dev_ptr(verts_out, torch.float32, "verts_out"), _dev_ptr(facets_out, torch.int32, "facets_out"),
            _dev_ptr(cluster_id, torch.int32, "cluster_id"), hp(nvo), hp(nfo),
            ctypes.byref(stats) if stats is not None else None)
        if st < 0:
            if check:
                self._raise(st)
            return st, None, None, None, None, None
        return st, verts_out[: int(nvo.sum())], facets_out[: int(nfo.sum())], cluster_id[:N], nvo, nfo

    def picasso_vertex_quadrics(self, verts, facets, stream=None):
        import torch
        N, F = int(verts.shape[0]), int(facets.shape[0])
        out = torch.empty((N, 10), dtype=torch.float32, device=verts.device)
        st = self._lib.picasso_vertex_quadrics(self._h, _stream_ptr(stream), _dev_ptr(verts, torch.float32, "verts"),
                                               N, _dev_ptr(facets, torch.int32, "facets"), F,
                                               _dev_ptr(out, torch.float32, "out"))
        if st != PICASSO_OK:
            self._raise(st)
        return out

    def picasso_edge_costs(self, verts, facets, stream=None):
        import torch
        N, F = int(verts.shape[0]), int(facets.shape[0])
        edges = torch.empty((max(3 * F, 1), 2), dtype=torch.int32, device=verts.device)
        cost = torch.empty((max(3 * F, 1),), dtype=torch.float32, device=verts.device)
        ne = ctypes.c_int32(0)
        st = self._lib.picasso_edge_costs(self._h, _stream_ptr(stream), _dev_ptr(verts, torch.float32, "verts"), N,
                                          _dev_ptr(facets, torch.int32, "facets"), F,
                                          _dev_ptr(edges, torch.int32, "edges"), _dev_ptr(cost, torch.float32, "cost"),
                                          ctypes.byref(ne))
        if st != PICASSO_OK:
            self._raise(st)
        return edges[: ne.value], cost[: ne.value]

    # -- pooling / unpooling over cluster_id ------------------------------------------------------

    def picasso_replace_mapping(self, cluster_id, n_out, stream=None):
        """Returns (replace int32[n_in], mapping int32[n_in]) device tensors."""
        import torch
        n_in = int(cluster_id.shape[0])
        rep = torch.empty((n_in,), dtype=torch.int32, device=cluster_id.device)
        mp = torch.empty((n_in,), dtype=torch.int32, device=cluster_id.device)
        st = self._lib.picasso_replace_mapping(self._h, _stream_ptr(stream),
                                               _dev_ptr(cluster_id, torch.int32, "cluster_id"), n_in, int(n_out),
                                               _dev_ptr(rep, torch.int32, "replace"), _dev_ptr(mp, torch.int32, "mapping"))
        if st != PICASSO_OK:
            self._raise(st)
        return rep, mp

    def picasso_cluster_csr(self, cluster_id, n_out, stream=None):
        """Returns (offsets int32[n_out+1], members int32[n_in]) device tensors."""
        import torch
        n_in = int(cluster_id.shape[0])
        off = torch.empty((n_out + 1,), dtype=torch.int32, device=cluster_id.device)
        mem = torch.empty((n_in,), dtype=torch.int32, device=cluster_id.device)
        st = self._lib.picasso_cluster_csr(self._h, _stream_ptr(stream), _dev_ptr(cluster_id, torch.int32, "cluster_id"),
                                           n_in, int(n_out), _dev_ptr(off, torch.int32, "off"),
                                           _dev_ptr(mem, torch.int32, "mem"))
        if st != PICASSO_OK:
            self._raise(st)
        return off, mem

    def picasso_pool_forward(self, mode, x, offsets, members, weight=None, want_argmax=None, stream=None):
        """Returns y[n_out, C]; for PICASSO_POOL_MAX returns (y, argmax)."""
        import torch
        n_in, C = int(x.shape[0]), int(x.shape[1])
        n_out = int(offsets.shape[0]) - 1
        y = torch.empty((n_out, C), dtype=torch.float32, device=x.device)
        if want_argmax is None:
            want_argmax = mode == PICASSO_POOL_MAX
        arg = torch.empty((n_out, C), dtype=torch.int32, device=x.device) if want_argmax else None
        st = self._lib.picasso_pool_forward(self._h, _stream_ptr(stream), int(mode), _dev_ptr(x, torch.float32, "x"),
                                            n_in, C, _dev_ptr(offsets, torch.int32, "offsets"),
                                            _dev_ptr(members, torch.int32, "members"), n_out,
                                            _dev_ptr(weight, torch.float32, "weight"), _dev_ptr(y, torch.float32, "y"),
                                            _dev_ptr(arg, torch.int32, "argmax"))
        if st != PICASSO_OK:
            self._raise(st)
        return (y, arg) if want_argmax else y

    def picasso_pool_backward(self, mode, gy, cluster_id, offsets, members, weight=None, argmax=None, stream=None):
        import torch
        n_in, C = int(cluster_id.shape[0]), int(gy.shape[1])
        n_out = int(offsets.shape[0]) - 1
        gx = torch.empty((n_in, C), dtype=torch.float32, device=gy.device)
        st = self._lib.picasso_pool_backward(self._h, _stream_ptr(stream), int(mode), _dev_ptr(gy, torch.float32, "gy"),
                                             n_in, C, _dev_ptr(cluster_id, torch.int32, "cluster_id"),
                                             _dev_ptr(offsets, torch.int32, "offsets"),
                                             _dev_ptr(members, torch.int32, "members"), n_out,
                                             _dev_ptr(weight, torch.float32, "weight"),
                                             _dev_ptr(argmax, torch.int32, "argmax"), _dev_ptr(gx, torch.float32, "gx"))
        if st != PICASSO_OK:
            self._raise(st)
        return gx

    def picasso_unpool_forward(self, y, cluster_id, stream=None):
        import torch
        n_in, C = int(cluster_id.shape[0]), int(y.shape[1])
        x = torch.empty((n_in, C), dtype=torch.float32, device=y.device)
        st = self._lib.picasso_unpool_forward(self._h, _stream_ptr(stream), _dev_ptr(y, torch.float32, "y"), n_in, C,
                                              _dev_ptr(cluster_id, torch.int32, "cluster_id"),
                                              _dev_ptr(x, torch.float32, "x"))
        if st != PICASSO_OK:
            self._raise(st)
        return x

    def picasso_unpool_backward(self, gx, offsets, members, stream=None):
        import torch
        n_in, C = int(gx.shape[0]), int(gx.shape[1])
        n_out = int(offsets.shape[0]) - 1
        gy = torch.empty((n_out, C), dtype=torch.float32, device=gx.device)
        st = self._lib.picasso_unpool_backward(self._h, _stream_ptr(stream), _dev_ptr(gx, torch.float32, "gx"), n_in, C,
                                               _dev_ptr(offsets, torch.int32, "offsets"),
                                               _dev_ptr(members, torch.int32, "members"), n_out,
                                               _dev_ptr(gy, torch.float32, "gy"))
        if st != PICASSO_OK:
            self._raise(st)
        return gy

    # ---- mesh convolutions, depth-wise (Sec. 4; supplementary, backward propagations)

    def picasso_vertex_corner_csr(self, facets, n_verts, stream=None):
        """Returns (offsets int32[N+1], corners int32[3F]) device tensors."""
        import torch
        F = int(facets.shape[0])
        off = torch.empty((int(n_verts) + 1,), dtype=torch.int32, device=facets.device)
        cor = torch.empty((3 * F,), dtype=torch.int32, device=facets.device)
        st = self._lib.picasso_vertex_corner_csr(self._h, _stream_ptr(stream), _dev_ptr(facets, torch.int32, "facets"),
                                                 F, int(n_verts), _dev_ptr(off, torch.int32, "off"),
                                                 _dev_ptr(cor, torch.int32, "cor"))
        if st != PICASSO_OK:
            self._raise(st)
        return off, cor

    def picasso_facet_geometry(self, verts, facets, nf=None, alpha=1, beta=1, stream=None):
        """Returns (normals f32[F,3], areas f32[F], level int32[F]); nf = facets per mesh of a batch."""
        import torch
        N, F = int(verts.shape[0]), int(facets.shape[0])
        nrm = torch.empty((F, 3), dtype=torch.float32, device=verts.device)
        area = torch.empty((F,), dtype=torch.float32, device=verts.device)
        lev = torch.empty((F,), dtype=torch.int32, device=verts.device)
        B = 1 if nf is None else len(nf)
        h_nf = None if nf is None else (ctypes.c_int32 * B)(*[int(v) for v in nf])
        st = self._lib.picasso_facet_geometry(self._h, _stream_ptr(stream), _dev_ptr(verts, torch.float32, "verts"), N,
                                              _dev_ptr(facets, torch.int32, "facets"), F, B, h_nf, int(alpha), int(beta),
                                              _dev_ptr(nrm, torch.float32, "normals"),
                                              _dev_ptr(area, torch.float32, "areas"), _dev_ptr(lev, torch.int32, "level"))
        if st != PICASSO_OK:
            self._raise(st)
        return nrm, area, lev

    def picasso_fuzzy_coefficients(self, normals, mu, inv_var, stream=None):
        import torch
        F, T = int(normals.shape[0]), int(mu.shape[0])
        pi = torch.empty((F, T), dtype=torch.float32, device=normals.device)
        st = self._lib.picasso_fuzzy_coefficients(self._h, _stream_ptr(stream),
                                                  _dev_ptr(normals, torch.float32, "normals"), F,
                                                  _dev_ptr(mu, torch.float32, "mu"),
                                                  _dev_ptr(inv_var, torch.float32, "inv_var"), T,
                                                  _dev_ptr(pi, torch.float32, "pi"))
        if st != PICASSO_OK:
            self._raise(st)
        return pi

    def picasso_v2f_forward(self, x, facets, level, w, out=None, stream=None):
        import torch
        N, C, F = int(x.shape[0]), int(x.shape[1]), int(facets.shape[0])
        y = out if out is not None else torch.empty((F, C), dtype=torch.float32, device=x.device)
        st = self._lib.picasso_v2f_forward(self._h, _stream_ptr(stream), _dev_ptr(x, torch.float32, "x"), N, C,
                                           _dev_ptr(facets, torch.int32, "facets"), F,
                                           _dev_ptr(level, torch.int32, "level") if level is not None else None,
                                           _dev_ptr(w, torch.float32, "w"), _dev_ptr(y, torch.float32, "y"))
        if st != PICASSO_OK:
            self._raise(st)
        return y

    def picasso_v2f_backward(self, gy, x, facets, level, w, offsets, corners, stream=None):
        """Returns (gx[N,C], gw[3,C])."""
        import torch
        N, C, F = int(x.shape[0]), int(x.shape[1]), int(facets.shape[0])
        gx = torch.empty((N, C), dtype=torch.float32, device=x.device)
        gw = torch.empty((3, C), dtype=torch.float32, device=x.device)
        st = self._lib.picasso_v2f_backward(self._h, _stream_ptr(stream), _dev_ptr(gy, torch.float32, "gy"),
                                            _dev_ptr(x, torch.float32, "x"), N, C,
                                            _dev_ptr(facets, torch.int32, "facets"), F,
                                            _dev_ptr(level, torch.int32, "level") if level is not None else None,
                                            _dev_ptr(w, torch.float32, "w"), _dev_ptr(offsets, torch.int32, "offsets"),
                                            _dev_ptr(corners, torch.int32, "corners"),
                                            _dev_ptr(gx, torch.float32, "gx"), _dev_ptr(gw, torch.float32, "gw"))
        if st != PICASSO_OK:
            self._raise(st)
        return gx, gw

    def picasso_f2f_forward(self, tex, bary, poff, w, stream=None):
        import torch
        P, C, F = int(tex.shape[0]), int(tex.shape[1]), int(poff.shape[0]) - 1
        y = torch.empty((F, C), dtype=torch.float32, device=tex.device)
        st = self._lib.picasso_f2f_forward(self._h, _stream_ptr(stream), _dev_ptr(tex, torch.float32, "tex"),
                                           _dev_ptr(bary, torch.float32, "bary"), _dev_ptr(poff, torch.int32, "poff"),
                                           F, P, C, _dev_ptr(w, torch.float32, "w"), _dev_ptr(y, torch.float32, "y"))
        if st != PICASSO_OK:
            self._raise(st)
        return y

    def picasso_f2f_backward(self, gy, tex, bary, poff, w, stream=None):
        """Returns (gtex[P,C], gw[3,C])."""
        import torch
        P, C, F = int(tex.shape[0]), int(tex.shape[1]), int(poff.shape[0]) - 1
        gtex = torch.zeros((P, C), dtype=torch.float32, device=tex.device)
        gw = torch.empty((3, C), dtype=torch.float32, device=tex.device)
        st = self._lib.picasso_f2f_backward(self._h, _stream_ptr(stream), _dev_ptr(gy, torch.float32, "gy"),
                                            _dev_ptr(tex, torch.float32, "tex"), _dev_ptr(bary, torch.float32, "bary"),
                                            _dev_ptr(poff, torch.int32, "poff"), F, P, C,
                                            _dev_ptr(w, torch.float32, "w"), _dev_ptr(gtex, torch.float32, "gtex"),
                                            _dev_ptr(gw, torch.float32, "gw"))
        if st != PICASSO_OK:
            self._raise(st)
        return gtex, gw

    def picasso_f2v_forward(self, y, pi, w, offsets, corners, n_verts, out=None, stream=None):
        import torch
        F, C, T = int(y.shape[0]), int(y.shape[1]), int(pi.shape[1])
        x = out if out is not None else torch.empty((int(n_verts), C), dtype=torch.float32, device=y.device)
        st = self._lib.picasso_f2v_forward(self._h, _stream_ptr(stream), _dev_ptr(y, torch.float32, "y"), F, C,
                                           _dev_ptr(pi, torch.float32, "pi"), T, _dev_ptr(w, torch.float32, "w"),
                                           _dev_ptr(offsets, torch.int32, "offsets"),
                                           _dev_ptr(corners, torch.int32, "corners"), int(n_verts),
                                           _dev_ptr(x, torch.float32, "x"))
        if st != PICASSO_OK:
            self._raise(st)
        return x

    def picasso_f2v_backward(self, gx, y, pi, w, facets, offsets, want_gpi=True, stream=None):
        """Returns (gy[F,C], gw[T,C], gpi[F,T] or None)."""
        import torch
        F, C, T, N = int(y.shape[0]), int(y.shape[1]), int(pi.shape[1]), int(gx.shape[0])
        gy = torch.empty((F, C), dtype=torch.float32, device=y.device)
        gw = torch.empty((T, C), dtype=torch.float32, device=y.device)
        gpi = torch.empty((F, T), dtype=torch.float32, device=y.device) if want_gpi else None
        st = self._lib.picasso_f2v_backward(self._h, _stream_ptr(stream), _dev_ptr(gx, torch.float32, "gx"),
                                            _dev_ptr(y, torch.float32, "y"), F, C, _dev_ptr(pi, torch.float32, "pi"), T,
                                            _dev_ptr(w, torch.float32, "w"), _dev_ptr(facets, torch.int32, "facets"),
                                            _dev_ptr(offsets, torch.int32, "offsets"), N,
                                            _dev_ptr(gy, torch.float32, "gy"), _dev_ptr(gw, torch.float32, "gw"),
                                            _dev_ptr(gpi, torch.float32, "gpi") if want_gpi else None)
        if st != PICASSO_OK:
            self._raise(st)
        return gy, gw, gpi

    def picasso_bucket_sort(self, keys, vals=None, key_bits=None, stream=None):
        """Same as picasso_radix_sort, by top-digit partition + per-bucket LDS sort (n <= 2^20)."""
        return self.picasso_radix_sort(keys, vals, key_bits, stream, _fn="picasso_bucket_sort")

    def picasso_radix_sort(self, keys, vals=None, key_bits=None, stream=None, _fn="picasso_radix_sort"):
        """In-place stable sort of a uint32-as-int32 / uint64-as-int64 tensor on its low key_bits bits."""
        import torch
        if keys.dtype == torch.int64:
            kb = 8
        elif keys.dtype == torch.int32:
            kb = 4
        else:
            raise TypeError("keys must be int32 or int64 (bit patterns of unsigned keys)")
        if key_bits is None:
            key_bits = 8 * kb
        st = getattr(self._lib, _fn)(self._h, _stream_ptr(stream), kb, _dev_ptr(keys, keys.dtype, "keys"),
                                          _dev_ptr(vals, torch.int32, "vals") if vals is not None else None,
                                          int(keys.shape[0]), int(key_bits))
        if st != PICASSO_OK:
            self._raise(st)
        return keys, vals
