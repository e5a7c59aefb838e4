"""ctypes binding of libcapgnn.so: same names as the C entry points, argument marshalling only.

Every step of the path runs inside the HIP library.  torch is used here for device memory,
pinned host memory and streams, nothing else.  There is no CPU fallback: if the shared library is
missing, ``lib()`` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
SO_PATH = os.path.join(_HERE, "libcapgnn.so")

OK, EINVAL, ENOMEM, EHIP, ENOTFOUND, EUNSUPPORTED = 0, -1, -2, -3, -4, -5
F32, BF16 = 0, 1
GCN, SAGE_MEAN = 0, 1
ACT_NONE, ACT_RELU = 0, 1
ORDER_AUTO, AGG_FIRST, XFORM_FIRST = 0, 1, 2
MAP_DIRECT, MAP_HASH = 0, 1
NORM_SYM, NORM_MEAN = 0, 1
GRAPH_SYMMETRIC = 1
MISS_ZEROCOPY, MISS_STAGED, MISS_PIPELINED = 0, 1, 2
MAX_RECORDS = 96
KIND_NAMES = {1: "gather_hit", 2: "gather_miss", 3: "spmm_fwd", 4: "spmm_bwd", 5: "gemm", 6: "loss", 7: "elementwise",
              8: "gather_staged"}


class CapgnnError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"capgnn error {code}: {msg}")
        self.code = code


class Layer(C.Structure):
    _fields_ = [("kind", C.c_int), ("f_in", C.c_int), ("f_out", C.c_int), ("act", C.c_int), ("dtype", C.c_int),
                ("order", C.c_int), ("out_f32", C.c_int), ("f32_product", C.c_int), ("W", C.c_void_p), ("W_self", C.c_void_p),
                ("bias", C.c_void_p)]


class RapaDevice(C.Structure):
    _fields_ = [("t_spmm", C.c_double), ("t_mm", C.c_double), ("f_h2d", C.c_double), ("f_d2h", C.c_double),
                ("f_idt", C.c_double), ("mem_bytes", C.c_double)]


class RapaParams(C.Structure):
    _fields_ = [("alpha", C.c_double), ("epsilon", C.c_double), ("m_vertex", C.c_double), ("m_edge", C.c_double),
                ("m_feat", C.c_double), ("f_dim", C.c_int64), ("beta", C.c_double), ("max_sweeps", C.c_int)]


class GatherStats(C.Structure):
    _fields_ = [("hits", C.c_int64), ("misses", C.c_int64), ("absent", C.c_int64)]


class _Record(C.Structure):
    _fields_ = [("kind", C.c_int), ("layer", C.c_int), ("backward", C.c_int), ("ms", C.c_float)]


class EpochTimes(C.Structure):
    _fields_ = [("total_ms", C.c_float), ("check_cache_ms", C.c_float), ("pick_cache_ms", C.c_float),
                ("communication_ms", C.c_float), ("aggregation_ms", C.c_float), ("combine_ms", C.c_float),
                ("loss_ms", C.c_float), ("other_ms", C.c_float), ("n_records", C.c_int),
                ("records", _Record * MAX_RECORDS)]

    def as_dict(self):
        d = {k: float(getattr(self, k)) for k, _ in self._fields_[:8]}
        d["records"] = [dict(kind=KIND_NAMES.get(r.kind, str(r.kind)), layer=r.layer, backward=r.backward, ms=float(r.ms))
                        for r in list(self.records)[: self.n_records]]
        return d


# name -> (restype, argtypes); this table is also what the symbol-export test walks
_vp, _i64, _i32, _sz = C.c_void_p, C.c_int64, C.c_int, C.c_size_t
SIGNATURES = {
    "capgnn_last_error": (C.c_char_p, []),
    "capgnn_version": (_i32, []),
    "capgnn_norm_scales": (_i32, [_i32, _i64, _i64, _vp, _vp, _vp, _vp]),
    "capgnn_gin_operator": (_i32, [_i64, _i64, _vp, _vp, C.c_float, _vp, _vp, _vp]),
    "capgnn_graph_create": (_i32, [C.POINTER(_vp), _i64, _i64, _vp, _vp, _vp, _vp, _vp, C.c_uint32, _vp]),
    "capgnn_graph_destroy": (_i32, [_vp]),
    "capgnn_spmm_workspace_bytes": (_sz, [_vp, _i32, _i32]),
    "capgnn_spmm_fwd": (_i32, [_vp, _vp, _i64, _vp, _i64, _i32, _i32, _vp, _sz, _vp]),
    "capgnn_spmm_bwd": (_i32, [_vp, _vp, _i64, _vp, _i64, _i32, _i32, _vp, _sz, _vp]),
    "capgnn_cal_capacity": (_i32, [C.c_double, C.c_double, _vp, _i32, _i32, _i64, C.POINTER(_i64)]),
    "capgnn_cache_sizes": (_i32, [_i64, _i64, _vp, _i32, _i32, C.POINTER(_sz), C.POINTER(_sz), C.POINTER(_sz)]),
    "capgnn_cache_build": (_i32, [C.POINTER(_vp), _i64, _vp, _vp, _i64, _vp, _i32, _i32, _vp, _vp, _i32, _vp]),
    "capgnn_cache_destroy": (_i32, [_vp]),
    "capgnn_cache_set_miss_mode": (_i32, [_vp, _i32]),
    "capgnn_overlap_ratio": (_i32, [_vp, _i64, _i64, _vp, _vp]),
    "capgnn_influence_score": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp]),
    "capgnn_policy_simulate": (_i32, [_i32, _vp, _vp, _i32, _i64, _i64, _i32, _i32, _vp]),
    "capgnn_halo_edge_counts": (_i32, [_i64, _i64, _vp, _vp, C.POINTER(_i64), _vp]),
    "capgnn_rapa_adjust": (_i32, [_i32, _vp, _vp, _vp, _vp, _vp, C.POINTER(RapaDevice), C.POINTER(RapaParams), _vp, _vp, _vp,
                                  C.POINTER(_i32), C.POINTER(C.c_double)]),
    "capgnn_prune_halo": (_i32, [_i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp]),
    "capgnn_locality_order": (_i32, [_i32, _i64, _i64, _vp, _vp, _vp]),
    "capgnn_relabel_csr": (_i32, [_i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "capgnn_epoch_graph_create": (_i32, [C.POINTER(_vp), _vp, _vp, _vp, _i32, _vp, _i64, _vp, _vp, C.c_double, _vp, _vp, _vp, _vp,
                                         C.c_float, _vp, _vp, _sz, _vp, _vp]),
    "capgnn_epoch_graph_launch": (_i32, [_vp, _vp]),
    "capgnn_epoch_graph_destroy": (_i32, [_vp]),
    "capgnn_cache_update": (_i32, [_vp, _i32, _vp, _i64, _i32, _vp, _i64, _i64, _vp, _vp]),
    "capgnn_cache_stale": (_i32, [_vp, _i32, _i64, _i64, _vp, _vp, _vp, _vp]),
    "capgnn_cache_fill": (_i32, [_vp, _i32, _vp, _i64, _vp]),
    "capgnn_cache_query": (_i32, [_vp, _vp, _i64, _i32, _vp, _vp]),
    "capgnn_cache_lookup": (_i32, [_vp, _vp, _i64, _i32, _vp, _vp, _vp]),
    "capgnn_halo_gather": (_i32, [_vp, _i32, _vp, _i64, _i32, _vp, _i64, _vp, _vp, _vp, C.POINTER(GatherStats)]),
    "capgnn_gemm_workspace_bytes": (_sz, [_i32, _i64, _i64, _i64]),
    "capgnn_mfma_peak": (_i32, [_i32, _i32, _i32, _vp, C.POINTER(C.c_double), _vp]),
    "capgnn_gather_peak": (_i32, [_vp, _i64, _i32, _i32, _i32, _vp, C.POINTER(C.c_double), _vp]),
    "capgnn_gemm": (_i32, [_i32, _i32, _i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _i32, _i32, _i32, _vp, _i32,
                           _vp, _i64, _i32, _vp, _sz, _vp]),
    "capgnn_layer_order": (_i32, [_vp, C.POINTER(Layer), _i32]),
    "capgnn_layer_saved_bytes": (_sz, [_vp, C.POINTER(Layer)]),
    "capgnn_layer_workspace_bytes": (_sz, [_vp, C.POINTER(Layer)]),
    "capgnn_layer_fwd": (_i32, [_vp, C.POINTER(Layer), _vp, _i64, _vp, _i64, _vp, _vp, _sz, _vp]),
    "capgnn_layer_bwd": (_i32, [_vp, C.POINTER(Layer), _vp, _i64, _vp, _i64, _vp, _vp, _i64, _vp, _vp, _vp, _vp, _i64,
                                _i32, _vp, _sz, _vp]),
    "capgnn_loss_workspace_bytes": (_sz, [_i64]),
    "capgnn_softmax_ce": (_i32, [_i64, _i32, _vp, _i64, _vp, _vp, C.c_double, _vp, _vp, _i64, _i32, _vp, _sz, _vp]),
    "capgnn_softmax_ce_static": (_i32, [_i64, _i32, _vp, _i64, _vp, _vp, C.c_double, _vp, _vp, _i64, _i32, _vp]),
    "capgnn_sigmoid_bce": (_i32, [_i64, _i32, _vp, _i64, _vp, _i64, _vp, C.c_double, _vp, _vp, _i64, _i32, _vp, _sz, _vp]),
    "capgnn_epoch_multilabel": (_i32, [_vp, _vp, C.POINTER(Layer), _i32, _vp, _i64, _vp, _i64, _vp, C.c_double, _vp,
                                       C.POINTER(_vp), C.POINTER(_vp), C.POINTER(_vp), C.c_float, C.POINTER(C.c_float),
                                       C.POINTER(EpochTimes), _vp, _sz, _vp, _vp]),
    "capgnn_epoch_workspace_bytes": (_sz, [_vp, _vp, C.POINTER(Layer), _i32]),
    "capgnn_epoch_activation": (_i32, [_vp, _vp, C.POINTER(Layer), _i32, _i32, _vp, C.POINTER(_vp), C.POINTER(_i64)]),
    "capgnn_epoch": (_i32, [_vp, _vp, C.POINTER(Layer), _i32, _vp, _i64, _vp, _vp, C.c_double, _vp, C.POINTER(_vp),
                            C.POINTER(_vp), C.POINTER(_vp), C.c_float, C.POINTER(C.c_float), C.POINTER(EpochTimes),
                            _vp, _sz, _vp, _vp]),
}

_lib = None


def lib():
    """The loaded shared library.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(SO_PATH):
            raise RuntimeError(f"{SO_PATH} is missing: build it with `python -m paper_2508_13716_amd.build`")
        # torch first: the library must bind to the HIP runtime torch has loaded (its own copy), else a second
        # runtime would be pulled in from the system path and the device memory torch hands over would be foreign
        import torch  # noqa: F401
        L = C.CDLL(SO_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _check(rc: int) -> int:
    if rc != OK:
        raise CapgnnError(rc, lib().capgnn_last_error().decode("utf-8", "replace"))
    return rc


def _p(x):
    """Raw address of a torch tensor / numpy array / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    return x.data_ptr()          # torch.Tensor


def _stream(s):
    if s is None:
        return None
    return s.cuda_stream if hasattr(s, "cuda_stream") else int(s)


def last_error() -> str:
    return lib().capgnn_last_error().decode("utf-8", "replace")


def version() -> int:
    return int(lib().capgnn_version())


# --------------------------------------------------------------------------- graph
def norm_scales(kind: int, n_loc: int, n_halo: int, rowptr: np.ndarray, halo_degree: Optional[np.ndarray]):
    rowptr = np.ascontiguousarray(rowptr, np.int64)
    hd = None if halo_degree is None else np.ascontiguousarray(halo_degree, np.int64)
    r = np.empty(n_loc, np.float32)
    c = np.empty(n_loc + n_halo, np.float32)
    _check(lib().capgnn_norm_scales(kind, n_loc, n_halo, _p(rowptr), _p(hd), _p(r), _p(c)))
    return r, c


class Graph:
    def __init__(self, n_loc: int, n_halo: int, rowptr, col, row_scale=None, col_scale=None, edge_val=None,
                 flags: int = 0, stream=None):
        rowptr = np.ascontiguousarray(rowptr, np.int64)
        col = np.ascontiguousarray(col, np.int32)
        rs = None if row_scale is None else np.ascontiguousarray(row_scale, np.float32)
        cs = None if col_scale is None else np.ascontiguousarray(col_scale, np.float32)
        ev = None if edge_val is None else np.ascontiguousarray(edge_val, np.float32)
        h = C.c_void_p()
        _check(lib().capgnn_graph_create(C.byref(h), n_loc, n_halo, _p(rowptr), _p(col), _p(rs), _p(cs), _p(ev),
                                         flags, _stream(stream)))
        self.h = h
        self.n_loc, self.n_halo, self.n_cols, self.nnz = n_loc, n_halo, n_loc + n_halo, int(rowptr[-1])

    def close(self):
        if self.h:
            lib().capgnn_graph_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def graph_create(*a, **k) -> Graph:
    return Graph(*a, **k)


def spmm_workspace_bytes(g: Graph, F: int, dtype: int) -> int:
    return int(lib().capgnn_spmm_workspace_bytes(g.h, F, dtype))


def spmm_fwd(g: Graph, X, ldx: int, Y, ldy: int, F: int, dtype: int, stream=None, ws=None, ws_bytes: int = 0):
    _check(lib().capgnn_spmm_fwd(g.h, _p(X), ldx, _p(Y), ldy, F, dtype, _p(ws), ws_bytes, _stream(stream)))


def spmm_bwd(g: Graph, dY, lddy: int, dX, lddx: int, F: int, dtype: int, stream=None, ws=None, ws_bytes: int = 0):
    _check(lib().capgnn_spmm_bwd(g.h, _p(dY), lddy, _p(dX), lddx, F, dtype, _p(ws), ws_bytes, _stream(stream)))


# --------------------------------------------------------------------------- cache
def cal_capacity(mem_gb: float, reserved_mb: float, dims: Sequence[int], n_candidates: int, elem_bytes: int = 4) -> int:
    d = np.ascontiguousarray(dims, np.int32)
    out = C.c_int64()
    _check(lib().capgnn_cal_capacity(mem_gb, reserved_mb, _p(d), len(d), elem_bytes, n_candidates, C.byref(out)))
    return int(out.value)


def cache_sizes(n_halo: int, cap_gpu: int, dims: Sequence[int], dtype: int):
    d = np.ascontiguousarray(dims, np.int32)
    a, b, s = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(lib().capgnn_cache_sizes(n_halo, cap_gpu, _p(d), len(d), dtype, C.byref(a), C.byref(b), C.byref(s)))
    return int(a.value), int(b.value), int(s.value)


class Cache:
    """Owns the two tier buffers (torch: device memory and pinned host memory) and the library handle."""

    def __init__(self, gid, prio, cap_gpu: int, dims: Sequence[int], dtype: int, map_kind: int = MAP_DIRECT,
                 stream=None):
        import torch
        gid = np.ascontiguousarray(gid, np.int64)
        prio = np.ascontiguousarray(prio, np.int64)
        self.n_halo = len(gid)
        self.dims = [int(d) for d in dims]
        self.dtype = dtype
        gb, hb, sb = cache_sizes(self.n_halo, cap_gpu, self.dims, dtype)
        self.gpu_bytes, self.host_bytes, self.staging_bytes = gb, hb, sb
        self.gpu_tier = torch.empty(max(gb, 256), dtype=torch.uint8, device="cuda")
        self.host_tier = torch.empty(max(hb, 256), dtype=torch.uint8, pin_memory=True)
        d = np.ascontiguousarray(self.dims, np.int32)
        h = C.c_void_p()
        _check(lib().capgnn_cache_build(C.byref(h), self.n_halo, _p(gid), _p(prio), cap_gpu, _p(d), len(d), dtype,
                                        _p(self.gpu_tier), _p(self.host_tier), map_kind, _stream(stream)))
        self.h = h
        self.cap_gpu = min(cap_gpu, self.n_halo)

    def set_miss_mode(self, mode: int):
        _check(lib().capgnn_cache_set_miss_mode(self.h, mode))

    def fill(self, layer: int, rows: np.ndarray, stream=None):
        rows = np.ascontiguousarray(rows)
        _check(lib().capgnn_cache_fill(self.h, layer, _p(rows), rows.shape[1], _stream(stream)))

    def query(self, ids, by_gid: bool = False, check: bool = True):
        ids = np.ascontiguousarray(ids, np.int64)
        tier = np.empty(len(ids), np.int8)
        slot = np.empty(len(ids), np.int64)
        rc = lib().capgnn_cache_query(self.h, _p(ids), len(ids), int(by_gid), _p(tier), _p(slot))
        if rc != OK and (check or rc != ENOTFOUND):
            _check(rc)
        return tier, slot

    def lookup(self, ids, tier, slot, by_gid: bool = False, stream=None):
        _check(lib().capgnn_cache_lookup(self.h, _p(ids), ids.numel(), int(by_gid), _p(tier), _p(slot), _stream(stream)))

    def close(self):
        if self.h:
            lib().capgnn_cache_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def cache_build(*a, **k) -> Cache:
    return Cache(*a, **k)


def halo_gather(c: Cache, layer: int, ids, n: int, out, ld: int, by_gid: bool = False, stream=None,
                side_stream=None, staging=None, want_stats: bool = False, check: bool = True):
    st = GatherStats() if want_stats else None
    rc = lib().capgnn_halo_gather(c.h, layer, _p(ids), n, int(by_gid), _p(out), ld, _stream(stream),
                                  _stream(side_stream), _p(staging), C.byref(st) if st is not None else None)
    if rc != OK and (check or rc != ENOTFOUND):
        _check(rc)
    return (rc, st) if want_stats else rc


def cache_update(c: Cache, layer: int, ids, n: int, rows, ld: int, epoch: int, by_gid: bool = False, stream=None,
                 want_stats: bool = False):
    st = GatherStats() if want_stats else None
    _check(lib().capgnn_cache_update(c.h, layer, _p(ids), n, int(by_gid), _p(rows), ld, epoch, _stream(stream),
                                     C.byref(st) if st is not None else None))
    return st


def cache_stale(c: Cache, layer: int, epoch_now: int, max_age: int, ids_out, stream=None):
    """Returns (number of stale rows, oldest stamp); ids_out (device int64[n_halo]) receives their indices."""
    n, lo = C.c_int64(0), C.c_int64(0)
    _check(lib().capgnn_cache_stale(c.h, layer, epoch_now, max_age, _p(ids_out), C.byref(n), C.byref(lo), _stream(stream)))
    return int(n.value), int(lo.value)


POLICY_JACA, POLICY_JACA_LOW, POLICY_FIFO, POLICY_LRU = 0, 1, 2, 3


def overlap_ratio(halo_ids, n_ids: int, n_vertices: int, R, stream=None):
    _check(lib().capgnn_overlap_ratio(_p(halo_ids), n_ids, n_vertices, _p(R), _stream(stream)))


def influence_score(g: Graph, inv_sqrt_din, inv_sqrt_dout, count, S, stream=None):
    _check(lib().capgnn_influence_score(g.h, _p(inv_sqrt_din), _p(inv_sqrt_dout), _p(count), _p(S), _stream(stream)))


def policy_simulate(halo_sets, policy: int, cap_local: int, cap_global: int, epochs: int, warmup: int = 1):
    """halo_sets: list of ascending, duplicate-free int64 arrays.  Returns (local hits, global hits, misses)."""
    ptr = np.zeros(len(halo_sets) + 1, np.int64)
    np.cumsum([len(h) for h in halo_sets], out=ptr[1:])
    ids = np.ascontiguousarray(np.concatenate(halo_sets) if len(halo_sets) else np.zeros(0, np.int64), np.int64)
    out = np.zeros(3, np.int64)
    _check(lib().capgnn_policy_simulate(len(halo_sets), _p(ptr), _p(ids), policy, cap_local, cap_global, epochs, warmup, _p(out)))
    return int(out[0]), int(out[1]), int(out[2])


def halo_edge_counts(n_loc: int, n_halo: int, rowptr, col):
    """(edges between inner vertices, int64 array of edges per halo vertex) of a partition graph."""
    rowptr = np.ascontiguousarray(rowptr, np.int64)
    col = np.ascontiguousarray(col, np.int32)
    e_inner = C.c_int64(0)
    cnt = np.zeros(n_halo, np.int64)
    _check(lib().capgnn_halo_edge_counts(n_loc, n_halo, _p(rowptr), _p(col), C.byref(e_inner), _p(cnt)))
    return int(e_inner.value), cnt


def rapa_adjust(n_inner, e_inner, halo_edges: Sequence[np.ndarray], scores: Sequence[np.ndarray], devices: Sequence[RapaDevice],
                params: RapaParams):
    """Alg. 2 / Alg. 3 on P subgraphs.  Returns dict(keep: per-subgraph uint8 arrays, lam, r, sweeps, sigma)."""
    P = len(devices)
    ni = np.ascontiguousarray(n_inner, np.int64)
    ei = np.ascontiguousarray(e_inner, np.int64)
    ptr = np.zeros(P + 1, np.int64)
    np.cumsum([len(h) for h in halo_edges], out=ptr[1:])
    he = np.ascontiguousarray(np.concatenate([np.asarray(h, np.int64) for h in halo_edges]) if ptr[-1] else np.zeros(0, np.int64))
    sc = np.ascontiguousarray(np.concatenate([np.asarray(x, np.float32) for x in scores]) if ptr[-1] else np.zeros(0, np.float32))
    keep = np.zeros(int(ptr[-1]), np.uint8)
    lam = np.zeros(P, np.float64)
    r = np.zeros(P, np.int32)
    sweeps, sigma = C.c_int(0), C.c_double(0.0)
    devs = (RapaDevice * P)(*devices)
    _check(lib().capgnn_rapa_adjust(P, _p(ni), _p(ei), _p(ptr), _p(he), _p(sc), devs, C.byref(params), _p(keep), _p(lam), _p(r),
                                    C.byref(sweeps), C.byref(sigma)))
    return {"keep": [keep[ptr[i]:ptr[i + 1]].copy() for i in range(P)], "lam": lam, "r": r.tolist(), "sweeps": int(sweeps.value),
            "sigma": float(sigma.value)}


def prune_halo(n_loc: int, n_halo: int, rowptr, col, keep):
    """(rowptr, col, new_index) of the subgraph without the halo vertices keep[] drops."""
    rowptr = np.ascontiguousarray(rowptr, np.int64)
    col = np.ascontiguousarray(col, np.int32)
    keep = np.ascontiguousarray(keep, np.uint8)
    rp, cl, ni = np.zeros_like(rowptr), np.zeros_like(col), np.zeros(n_halo, np.int64)
    _check(lib().capgnn_prune_halo(n_loc, n_halo, _p(rowptr), _p(col), _p(keep), _p(rp), _p(cl), _p(ni)))
    return rp, cl[: int(rp[-1])].copy(), ni


RELABEL_POPULARITY, RELABEL_BFS = 0, 1


def locality_order(method: int, n_loc: int, n_halo: int, rowptr, col) -> np.ndarray:
    """new2old (int32 [n_loc + n_halo]): the vertex to store at each place."""
    rowptr = np.ascontiguousarray(rowptr, np.int64)
    col = np.ascontiguousarray(col, np.int32)
    out = np.zeros(n_loc + n_halo, np.int32)
    _check(lib().capgnn_locality_order(method, n_loc, n_halo, _p(rowptr), _p(col), _p(out)))
    return out


def relabel_csr(n_loc: int, n_halo: int, rowptr, col, new2old, edge_val=None):
    """(rowptr, col, edge_val) of the partition with its vertices moved to the places new2old names."""
    rowptr = np.ascontiguousarray(rowptr, np.int64)
    col = np.ascontiguousarray(col, np.int32)
    new2old = np.ascontiguousarray(new2old, np.int32)
    val = None if edge_val is None else np.ascontiguousarray(edge_val, np.float32)
    rp, cl = np.zeros_like(rowptr), np.zeros_like(col)
    vl = None if val is None else np.zeros_like(val)
    _check(lib().capgnn_relabel_csr(n_loc, n_halo, _p(rowptr), _p(col), _p(val), _p(new2old), _p(rp), _p(cl), _p(vl)))
    return rp, cl, vl


# --------------------------------------------------------------------------- dense, layer, loss, epoch
F32_PRODUCT_AUTO, F32_PRODUCT_NATIVE, F32_PRODUCT_SPLIT = 0, 1, 2     # how a product of fp32 operands is formed


def mfma_peak(dtype: int, workgroups: int, iters: int, out, stream=None) -> float:
    """Launches the register-resident matrix-instruction loop; returns the FLOPs it performs (the caller times it)."""
    flop = C.c_double(0.0)
    _check(lib().capgnn_mfma_peak(dtype, workgroups, iters, _p(out), C.byref(flop), _stream(stream)))
    return float(flop.value)


def gather_peak(table, table_lines: int, workgroups: int, iters: int, out, stream=None, line_stride: int = 1) -> float:
    """Launches the pure 128-byte-line gather loop over `table`; returns the bytes it requests (the caller times it)."""
    nbytes = C.c_double(0.0)
    _check(lib().capgnn_gather_peak(_p(table), table_lines, line_stride, workgroups, iters, _p(out), C.byref(nbytes), _stream(stream)))
    return float(nbytes.value)


def gemm_workspace_bytes(trans_a: int, M: int, N: int, K: int) -> int:
    return int(lib().capgnn_gemm_workspace_bytes(trans_a, M, N, K))


def gemm(trans_a: int, trans_b: int, M: int, N: int, K: int, A, lda: int, B, ldb: int, Cm, ldc: int, dtype: int,
         out_f32: int = 0, accumulate: int = 0, bias=None, relu: int = 0, relu_mask=None, ldm: int = 0, ws=None,
         ws_bytes: int = 0, stream=None, f32_product: int = F32_PRODUCT_AUTO):
    _check(lib().capgnn_gemm(trans_a, trans_b, M, N, K, _p(A), lda, _p(B), ldb, _p(Cm), ldc, dtype, out_f32, accumulate,
                             _p(bias), relu, _p(relu_mask), ldm, f32_product, _p(ws), ws_bytes, _stream(stream)))


def make_layer(kind: int, f_in: int, f_out: int, act: int, dtype: int, W, W_self=None, bias=None,
               order: int = ORDER_AUTO, out_f32: int = 0, f32_product: int = F32_PRODUCT_AUTO) -> Layer:
    return Layer(kind, f_in, f_out, act, dtype, order, out_f32, f32_product, _p(W), _p(W_self), _p(bias))


def layer_order(g: Graph, l: Layer, need_dx: bool) -> int:
    rc = lib().capgnn_layer_order(g.h, C.byref(l), int(need_dx))
    if rc < 0:
        _check(rc)
    return rc


def layer_saved_bytes(g: Graph, l: Layer) -> int:
    return int(lib().capgnn_layer_saved_bytes(g.h, C.byref(l)))


def layer_workspace_bytes(g: Graph, l: Layer) -> int:
    return int(lib().capgnn_layer_workspace_bytes(g.h, C.byref(l)))


def layer_fwd(g: Graph, l: Layer, X, ldx: int, H, ldh: int, saved, ws, ws_bytes: int, stream=None):
    _check(lib().capgnn_layer_fwd(g.h, C.byref(l), _p(X), ldx, _p(H), ldh, _p(saved), _p(ws), ws_bytes, _stream(stream)))


def layer_bwd(g: Graph, l: Layer, X, ldx: int, H, ldh: int, saved, dH, lddh: int, dW, dW_self, dbias, dX, lddx: int,
              need_halo_grad: bool, ws, ws_bytes: int, stream=None):
    _check(lib().capgnn_layer_bwd(g.h, C.byref(l), _p(X), ldx, _p(H), ldh, _p(saved), _p(dH), lddh, _p(dW), _p(dW_self),
                                  _p(dbias), _p(dX), lddx, int(need_halo_grad), _p(ws), ws_bytes, _stream(stream)))


def loss_workspace_bytes(n: int) -> int:
    return int(lib().capgnn_loss_workspace_bytes(n))


def softmax_ce(n: int, n_classes: int, Z, ldz: int, labels, mask, loss_norm: float, loss_dev, dZ, lddz: int,
               dz_dtype: int, ws, ws_bytes: int, stream=None):
    _check(lib().capgnn_softmax_ce(n, n_classes, _p(Z), ldz, _p(labels), _p(mask), loss_norm, _p(loss_dev), _p(dZ), lddz,
                                   dz_dtype, _p(ws), ws_bytes, _stream(stream)))


LOSS_STATIC_MAX_ROWS = 1 << 20


def softmax_ce_static(n: int, n_classes: int, Z, ldz: int, labels, mask, loss_norm: float, loss_dev, dZ, lddz: int,
                      dz_dtype: int, stream=None):
    """capgnn_softmax_ce on the library's built-in scratch: no workspace, no allocation (n <= LOSS_STATIC_MAX_ROWS)."""
    _check(lib().capgnn_softmax_ce_static(n, n_classes, _p(Z), ldz, _p(labels), _p(mask), loss_norm, _p(loss_dev), _p(dZ),
                                          lddz, dz_dtype, _stream(stream)))


def sigmoid_bce(n: int, n_classes: int, Z, ldz: int, targets, ldt: int, mask, loss_norm: float, loss_dev, dZ, lddz: int,
                dz_dtype: int, ws, ws_bytes: int, stream=None):
    _check(lib().capgnn_sigmoid_bce(n, n_classes, _p(Z), ldz, _p(targets), ldt, _p(mask), loss_norm, _p(loss_dev), _p(dZ),
                                    lddz, dz_dtype, _p(ws), ws_bytes, _stream(stream)))


def gin_operator(n_loc: int, n_halo: int, rowptr, col, eps: float):
    """(rowptr, col, edge_val) of the GIN aggregation operator: unit entries plus a diagonal of 1 + eps."""
    rowptr = np.ascontiguousarray(rowptr, np.int64)
    col = np.ascontiguousarray(col, np.int32)
    nnz = int(rowptr[n_loc]) + n_loc
    rp, cl, vl = np.zeros(n_loc + 1, np.int64), np.zeros(nnz, np.int32), np.zeros(nnz, np.float32)
    _check(lib().capgnn_gin_operator(n_loc, n_halo, _p(rowptr), _p(col), eps, _p(rp), _p(cl), _p(vl)))
    return rp, cl, vl


def epoch_workspace_bytes(g: Graph, c: Optional[Cache], layers: List[Layer]) -> int:
    arr = (Layer * len(layers))(*layers)
    return int(lib().capgnn_epoch_workspace_bytes(g.h, c.h if c is not None else None, arr, len(layers)))


def epoch_activation(g: Graph, c: Optional[Cache], layers: List[Layer], l: int, ws):
    """(device address, leading dimension) of hidden layer l's output inside the epoch workspace."""
    arr = (Layer * len(layers))(*layers)
    ptr, ld = C.c_void_p(), C.c_int64()
    _check(lib().capgnn_epoch_activation(g.h, c.h if c is not None else None, arr, len(layers), l, _p(ws),
                                         C.byref(ptr), C.byref(ld)))
    return int(ptr.value), int(ld.value)


class EpochGraph:
    """capgnn_epoch recorded as a HIP graph (capgnn_epoch_graph_create); launch() replays it.  Keeps references to every
    tensor it was given: the graph holds their addresses."""

    def __init__(self, g: Graph, c: Optional[Cache], layers: List[Layer], X0, ld0: int, labels, mask, loss_norm: float,
                 logits, dW: Sequence, dW_self: Optional[Sequence], dbias: Sequence, lr: float, loss_dev, ws, ws_bytes: int,
                 stream, side_stream=None):
        L = len(layers)
        arr = (Layer * L)(*layers)
        pw = (C.c_void_p * L)(*[_p(t) for t in dW])
        ps = (C.c_void_p * L)(*[_p(t) for t in dW_self]) if dW_self is not None else None
        pb = (C.c_void_p * L)(*[_p(t) for t in dbias])
        self._keep = (g, c, layers, X0, labels, mask, logits, dW, dW_self, dbias, loss_dev, ws)
        h = C.c_void_p()
        _check(lib().capgnn_epoch_graph_create(C.byref(h), g.h, c.h if c is not None else None, arr, L, _p(X0), ld0, _p(labels),
                                               _p(mask), loss_norm, _p(logits), pw, ps, pb, lr, _p(loss_dev), _p(ws), ws_bytes,
                                               _stream(stream), _stream(side_stream)))
        self.h = h

    def launch(self, stream):
        _check(lib().capgnn_epoch_graph_launch(self.h, _stream(stream)))

    def close(self):
        if self.h:
            lib().capgnn_epoch_graph_destroy(self.h)
            self.h = None
            self._keep = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def epoch(g: Graph, c: Optional[Cache], layers: List[Layer], X0, ld0: int, labels, mask, loss_norm: float, logits,
          dW: Sequence, dW_self: Optional[Sequence], dbias: Sequence, lr: float, ws, ws_bytes: int, stream=None,
          side_stream=None, want_loss: bool = True, want_times: bool = False, targets=None, ldt: int = 0):
    """One epoch; with `targets` (device uint8 [n_loc x ldt]) the multi-label entry point runs and `labels` is unused."""
    L = len(layers)
    arr = (Layer * L)(*layers)
    pw = (C.c_void_p * L)(*[_p(t) for t in dW])
    ps = (C.c_void_p * L)(*[_p(t) for t in dW_self]) if dW_self is not None else None
    pb = (C.c_void_p * L)(*[_p(t) for t in dbias])
    loss = C.c_float(float("nan"))
    times = EpochTimes() if want_times else None
    tail = (_p(mask), loss_norm, _p(logits), pw, ps, pb, lr, C.byref(loss) if want_loss else None,
            C.byref(times) if times is not None else None, _p(ws), ws_bytes, _stream(stream), _stream(side_stream))
    if targets is not None:
        _check(lib().capgnn_epoch_multilabel(g.h, c.h if c is not None else None, arr, L, _p(X0), ld0, _p(targets), ldt, *tail))
    else:
        _check(lib().capgnn_epoch(g.h, c.h if c is not None else None, arr, L, _p(X0), ld0, _p(labels), *tail))
    return (float(loss.value) if want_loss else None), (times.as_dict() if times is not None else None)
