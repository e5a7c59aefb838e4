"""CPU oracle: the plain fp64 definition of the partition-local layer step.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module; only
``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` do.
It imports nothing from the HIP package and shares no code with it.

The numeric steps live in ``capgnn_oracle.c`` (plain loops, double precision, each output
summed sequentially); this file marshals numpy arrays into it and writes the layer and
epoch out in the paper's order:

* GCN layer (forward rule in the proof of Lemma 2):   Z = A_hat H W (+ bias),  H' = sigma(Z)
* GraphSAGE-mean layer (Eq. 1 with AGGREGATE = mean, COMBINE = two linear maps + sigma)
* backward: the chain rule of those two rules (Lemma 3's recursion, made conformable)
* loss: cross-entropy (evaluation setup), averaged over the masked local rows
* epoch: for each layer, halo rows are first taken from the cache tables (JACA workflow),
  then the layer runs on [local rows; halo rows]; backward visits the layers in reverse;
  the optional parameter step is W <- W - tau * grad (update rule in the theorem's proof).

Readings where the paper is silent (self loops, halo degrees, sigma = ReLU with
sigma'(0) = 0, mean aggregator, ties by global id, ...) are listed in the design notes
at the repository root.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from fractions import Fraction
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "capgnn_oracle.c")
_SO = os.path.join(_HERE, "libcapgnn_oracle.so")
_lib_handle = None
_blas_limit = None


def build(force: bool = False) -> str:
    """Compile the C part with gcc (-O2, OpenMP).  Returns the path of the shared object."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
                               "-o", _SO, _SRC, "-lm"])
    return _SO


def _lib():
    global _lib_handle
    if _lib_handle is None:
        build()
        L = C.CDLL(_SO)
        i64, p = C.c_int64, C.c_void_p
        L.orc_max_threads.restype = C.c_int
        L.orc_set_threads.argtypes = [C.c_int]
        L.orc_placement.argtypes = [i64, p, p, i64, p, p]
        L.orc_locality_order.argtypes = [C.c_int, i64, i64, p, p, p]
        L.orc_locality_order.restype = C.c_int
        L.orc_gather.argtypes = [p, i64, i64, p, i64, p]
        L.orc_gather.restype = i64
        L.orc_cache_update.argtypes = [p, p, i64, i64, p, i64, p, i64]
        L.orc_cache_update.restype = i64
        L.orc_stale_ids.argtypes = [p, i64, i64, i64, p, p]
        L.orc_stale_ids.restype = i64
        L.orc_influence.argtypes = [i64, i64, p, p, p, p, p, p]
        L.orc_gcn_scales.argtypes = [i64, i64, p, p, p, p]
        L.orc_mean_scales.argtypes = [i64, i64, p, p, p]
        L.orc_spmm_fwd.argtypes = [i64, p, p, p, p, p, p, i64, p]
        L.orc_spmm_bwd.argtypes = [i64, i64, p, p, p, p, p, p, i64, p]
        L.orc_softmax_ce.argtypes = [i64, i64, p, p, p, C.c_double, p]
        L.orc_softmax_ce.restype = C.c_double
        _lib_handle = L
    return _lib_handle


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def max_threads() -> int:
    return int(_lib().orc_max_threads())


def set_threads(n: int) -> None:
    """Threads of the C loops (OpenMP) and of numpy's matrix product (its BLAS thread pool)."""
    global _blas_limit
    _lib().orc_set_threads(int(n))
    from threadpoolctl import threadpool_limits
    _blas_limit = threadpool_limits(limits=int(n), user_api="blas")


# ------------------------------------------------------------------ cache side
def placement(gid: np.ndarray, prio: np.ndarray, cap_gpu: int):
    """Rank halo vertices by (priority descending, global id ascending); the first
    min(cap_gpu, n_halo) go to the GPU tier (0), the rest to the host tier (1)."""
    gid = np.ascontiguousarray(gid, np.int64)
    prio = np.ascontiguousarray(prio, np.int64)
    n = len(gid)
    order = np.zeros(n, np.int64)
    tier = np.zeros(n, np.int8)
    _lib().orc_placement(n, _ptr(gid), _ptr(prio), int(cap_gpu), _ptr(order), _ptr(tier))
    return order, tier


def cal_capacity(mem_gb, reserved_mb, dims: Sequence[int], n_candidates: int, elem_bytes: int = 4) -> int:
    """Adaptive cache capacity (Alg. 1): rows = min(floor(((mem_gb*1024 - reserved_mb) * 1024^2)
    / sum_k(dims[k] * elem_bytes)), n_candidates), exact rational arithmetic, never negative."""
    num = (Fraction(mem_gb) * 1024 - Fraction(reserved_mb)) * 1024 * 1024
    den = sum(int(d) for d in dims) * int(elem_bytes)
    rows = int(num // den) if num > 0 else 0
    return min(rows, int(n_candidates))


def gather(table: np.ndarray, ids: np.ndarray):
    """out[r,:] = table[ids[r],:] as a bit copy; ids outside the table give zero rows.  Returns (out, absent)."""
    table = np.ascontiguousarray(table)
    ids = np.ascontiguousarray(ids, np.int64)
    row_bytes = table.strides[0] if table.shape[0] > 0 else table.shape[1] * table.itemsize
    out = np.zeros((len(ids), table.shape[1]), dtype=table.dtype)
    absent = _lib().orc_gather(_ptr(table), table.shape[0], row_bytes, _ptr(ids), len(ids), _ptr(out))
    return out, int(absent)


def cache_update(table: np.ndarray, stamp: np.ndarray, ids, rows: np.ndarray, epoch: int) -> int:
    """Vertex update: table[ids[r], :] = rows[r, :] and stamp[ids[r]] = epoch, r ascending (the last of several
    updates of one row stays); ids outside the table are skipped.  In place; returns the number skipped."""
    assert table.flags.c_contiguous and stamp.dtype == np.int64 and stamp.flags.c_contiguous
    ids = np.ascontiguousarray(ids, np.int64)
    rows = np.ascontiguousarray(rows, dtype=table.dtype)
    assert rows.shape == (len(ids), table.shape[1])
    row_bytes = table.shape[1] * table.itemsize
    return int(_lib().orc_cache_update(_ptr(table), _ptr(stamp), table.shape[0], row_bytes, _ptr(ids), len(ids),
                                       _ptr(rows), int(epoch)))


def stale_ids(stamp: np.ndarray, epoch_now: int, max_age: int):
    """Bounded staleness: ascending ids of the rows not refreshed for more than max_age iterations, and the
    oldest stamp."""
    stamp = np.ascontiguousarray(stamp, np.int64)
    out = np.zeros(len(stamp), np.int64)
    oldest = np.zeros(1, np.int64)
    n = _lib().orc_stale_ids(_ptr(stamp), len(stamp), int(epoch_now), int(max_age), _ptr(out), _ptr(oldest))
    return out[:n].copy(), int(oldest[0])


def overlap_ratio(halo_sets: Sequence[np.ndarray]):
    """Vertex overlap ratio (Eq. 2): for every vertex in the union of the partitions' halo sets, the
    number of partitions whose halo set contains it.  Returns (vertex ids ascending, counts)."""
    allv = np.concatenate([np.unique(np.asarray(h, np.int64)) for h in halo_sets]) if len(halo_sets) else np.zeros(0, np.int64)
    ids, cnt = np.unique(allv, return_counts=True)
    return ids, cnt.astype(np.int64)


def policy_hit_counts(halo_sets: Sequence[np.ndarray], policy: str, cap_local: int, cap_global: int,
                      epochs: int, warmup: int = 1):
    """Two-level cache policy comparison (evaluation sections on the vertex overlap ratio and on cache
    capacity: JACA against FIFO and LRU, all on the same local + global structure).

    Model (the paper gives no listing; this is the reading the design notes record): in every epoch the
    partitions i = 0..P-1 take turns, and partition i asks for every vertex of its halo set in ascending id
    order.  A request is served by the partition's local cache, else by the shared global cache, else it is a
    miss (the vertex has to be communicated).
      'jaca' / 'jaca_low': static contents chosen by the vertex overlap ratio R (Eq. 2) - local cache i holds the
          cap_local vertices of H_i with the highest (lowest) R, the global cache the cap_global vertices of the
          union with the highest (lowest) R, ties by ascending vertex id.
      'fifo' / 'lru': both levels start empty; a global hit or a miss inserts the vertex into the local cache, a
          miss also into the global cache, evicting the first-inserted / least-recently-used entry of a full
          cache (an LRU hit refreshes the entry; capacity 0 holds nothing).
    Requests of the first `warmup` epochs fill the caches and are not counted.  Returns (local hits, global
    hits, misses) over the remaining epochs."""
    from collections import OrderedDict
    sets = [np.unique(np.asarray(h, np.int64)) for h in halo_sets]
    P = len(sets)
    hits_l = hits_g = misses = 0
    if policy in ("jaca", "jaca_low"):
        ids, cnt = overlap_ratio(sets)
        R = dict(zip(ids.tolist(), cnt.tolist()))
        sign = -1 if policy == "jaca" else 1
        key = lambda v: (sign * R[v], v)
        glob = set(sorted(ids.tolist(), key=key)[:max(cap_global, 0)])
        loc = [set(sorted(h.tolist(), key=key)[:max(cap_local, 0)]) for h in sets]
        for e in range(epochs):
            for i in range(P):
                for v in sets[i].tolist():
                    if e < warmup:
                        continue
                    if v in loc[i]:
                        hits_l += 1
                    elif v in glob:
                        hits_g += 1
                    else:
                        misses += 1
        return hits_l, hits_g, misses
    assert policy in ("fifo", "lru")
    lru = policy == "lru"

    def insert(cache: "OrderedDict", cap: int, v: int):
        if cap <= 0 or v in cache:
            return
        if len(cache) >= cap:
            cache.popitem(last=False)            # oldest insertion (FIFO) / least recent use (LRU)
        cache[v] = True

    glob: "OrderedDict" = OrderedDict()
    loc = [OrderedDict() for _ in range(P)]
    for e in range(epochs):
        for i in range(P):
            for v in sets[i].tolist():
                counted = e >= warmup
                if v in loc[i]:
                    if lru:
                        loc[i].move_to_end(v)
                    hits_l += counted
                elif v in glob:
                    if lru:
                        glob.move_to_end(v)
                    insert(loc[i], cap_local, v)
                    hits_g += counted
                else:
                    insert(glob, cap_global, v)
                    insert(loc[i], cap_local, v)
                    misses += counted
    return int(hits_l), int(hits_g), int(misses)


def influence_score(n_loc: int, n_cols: int, rowptr, col, din, dout, count=None) -> np.ndarray:
    """RAPA's vertex influence score (Eq. 6) of every column vertex of a partition graph.  din[n_loc]: in-degrees
    of the local vertices, dout[n_cols]: out-degrees of the column vertices, count[n_cols]: repetition counts
    (1 when omitted).  A vertex without incident edges scores 0; degrees must be positive where they are used."""
    rowptr = np.ascontiguousarray(rowptr, np.int64)
    col = np.ascontiguousarray(col, np.int32)
    din, dout = _f64(din), _f64(dout)
    cnt = np.ones(n_cols) if count is None else _f64(count)
    S = np.zeros(n_cols, np.float64)
    _lib().orc_influence(n_loc, n_cols, _ptr(rowptr), _ptr(col), _ptr(din), _ptr(dout), _ptr(cnt), _ptr(S))
    return S


def locality_order(method: str, n_loc: int, n_halo: int, rowptr, col) -> np.ndarray:
    """A storage order of the partition's vertices ("we reorder the subgraphs", reorder figure): new2old, a
    permutation that keeps local vertices in [0, n_loc) and halo vertices after them.  method "popularity":
    most referenced first inside each range; "bfs": breadth-first over the local-to-local entries from the
    longest rows, halo vertices by first mention (both defined in full in capgnn_oracle.c)."""
    rowptr = np.ascontiguousarray(rowptr, np.int64)
    col = np.ascontiguousarray(col, np.int32)
    out = np.zeros(n_loc + n_halo, np.int32)
    rc = _lib().orc_locality_order({"popularity": 0, "bfs": 1}[method], n_loc, n_halo, _ptr(rowptr), _ptr(col), _ptr(out))
    if rc != 0:
        raise MemoryError("orc_locality_order")
    return out


def relabel_csr(n_loc: int, rowptr, col, new2old, val=None):
    """The partition's CSR after its vertices moved to the places new2old names: row k of the result is old row
    new2old[k] with every column index replaced by its new place, its entries sorted by that new index (equal
    indices keep their order), so a sorted CSR stays sorted and a symmetric one stays equal to its transpose."""
    rowptr = np.asarray(rowptr, np.int64)
    col = np.asarray(col, np.int64)
    new2old = np.asarray(new2old, np.int64)
    old2new = np.zeros(len(new2old), np.int64)
    for k, o in enumerate(new2old):
        old2new[o] = k
    new_ptr, new_col, new_val = [0], [], []
    for k in range(n_loc):
        o = new2old[k]
        entries = sorted(range(rowptr[o], rowptr[o + 1]), key=lambda e: old2new[col[e]])   # sorted() is stable
        for e in entries:
            new_col.append(old2new[col[e]])
            if val is not None:
                new_val.append(val[e])
        new_ptr.append(len(new_col))
    return (np.array(new_ptr, np.int64), np.array(new_col, np.int32),
            None if val is None else np.array(new_val, np.asarray(val).dtype))


# ------------------------------------------------------------------ graph
@dataclass
class Graph:
    n_loc: int
    n_cols: int
    rowptr: np.ndarray            # int64
    col: np.ndarray               # int32
    r: np.ndarray                 # float64 [n_loc]   row scale
    c: np.ndarray                 # float64 [n_cols]  column scale
    v: Optional[np.ndarray] = None  # float64 [nnz] edge values or None (= 1)


def gcn_graph(n_loc: int, n_halo: int, rowptr, col, halo_degree) -> Graph:
    rowptr = np.ascontiguousarray(rowptr, np.int64)
    col = np.ascontiguousarray(col, np.int32)
    hd = np.ascontiguousarray(halo_degree, np.int64)
    r = np.zeros(n_loc, np.float64)
    c = np.zeros(n_loc + n_halo, np.float64)
    _lib().orc_gcn_scales(n_loc, n_halo, _ptr(rowptr), _ptr(hd), _ptr(r), _ptr(c))
    return Graph(n_loc, n_loc + n_halo, rowptr, col, r, c)


def mean_graph(n_loc: int, n_halo: int, rowptr, col) -> Graph:
    rowptr = np.ascontiguousarray(rowptr, np.int64)
    col = np.ascontiguousarray(col, np.int32)
    r = np.zeros(n_loc, np.float64)
    c = np.zeros(n_loc + n_halo, np.float64)
    _lib().orc_mean_scales(n_loc, n_loc + n_halo, _ptr(rowptr), _ptr(r), _ptr(c))
    return Graph(n_loc, n_loc + n_halo, rowptr, col, r, c)


def spmm_fwd(g: Graph, X) -> np.ndarray:
    X = _f64(X)
    assert X.shape[0] == g.n_cols
    F = X.shape[1]
    Y = np.zeros((g.n_loc, F), np.float64)
    _lib().orc_spmm_fwd(g.n_loc, _ptr(g.rowptr), _ptr(g.col), _ptr(g.r), _ptr(g.c), _ptr(g.v), _ptr(X), F, _ptr(Y))
    return Y


def spmm_bwd(g: Graph, dY) -> np.ndarray:
    dY = _f64(dY)
    assert dY.shape[0] == g.n_loc
    F = dY.shape[1]
    dX = np.zeros((g.n_cols, F), np.float64)
    _lib().orc_spmm_bwd(g.n_loc, g.n_cols, _ptr(g.rowptr), _ptr(g.col), _ptr(g.r), _ptr(g.c), _ptr(g.v),
                        _ptr(dY), F, _ptr(dX))
    return dX


def matmul(A, B, ta: bool = False, tb: bool = False) -> np.ndarray:
    """op(A) op(B) in float64, op = transpose when ta / tb: the dense product of the combination step (Eq. 1's
    COMBINE; Z = (A_hat H) W in the forward rule of Lemma 2's proof) and of its chain rule.  A library primitive:
    numpy's matrix product."""
    A, B = _f64(A), _f64(B)
    return np.ascontiguousarray(np.matmul(A.T if ta else A, B.T if tb else B))


def softmax_ce(Z, y, mask=None, norm: float = 0.0):
    Z = _f64(Z)
    y = np.ascontiguousarray(y, np.int32)
    m = None if mask is None else np.ascontiguousarray(mask, np.uint8)
    dZ = np.zeros_like(Z)
    loss = _lib().orc_softmax_ce(Z.shape[0], Z.shape[1], _ptr(Z), _ptr(y), _ptr(m), float(norm), _ptr(dZ))
    return float(loss), dZ


def sigmoid_bce(Z, Y, mask=None, norm: float = 0.0):
    """Binary cross-entropy on logits, the loss of the multi-label tasks (evaluation setup): per element
    -[y log s(z) + (1-y) log(1-s(z))] with s the logistic function, written in the overflow-free form
    max(z,0) - z y + log(1 + exp(-|z|)); summed over the masked rows and all classes and divided by `norm`
    (default: masked rows x classes, the mean over elements).  Returns (loss, dloss/dZ)."""
    Z, Y = _f64(Z), _f64(Y)
    n, C = Z.shape
    on = np.ones(n, bool) if mask is None else np.asarray(mask).astype(bool)
    if norm <= 0.0:
        norm = float(max(int(on.sum()), 1) * C)
    per = np.maximum(Z, 0.0) - Z * Y + np.log1p(np.exp(-np.abs(Z)))
    loss = float(per[on].sum() / norm)
    e = np.exp(-np.abs(Z))
    s = np.where(Z >= 0, 1.0 / (1.0 + e), e / (1.0 + e))
    dZ = (s - Y) / norm
    dZ[~on] = 0.0
    return loss, dZ


def gin_graph(n_loc: int, n_halo: int, rowptr, col, eps: float = 0.0):
    """Operator of a GIN layer's aggregation, (1 + eps) x_i + sum_{j in N(i)} x_j: the stored entries with unit
    weight plus a diagonal entry (1 + eps) appended to every row; no normalisation.  The layer itself is then
    sigma(A X W + b), i.e. kind 'gcn' on this operator (GIN with a one-layer update function)."""
    rowptr = np.asarray(rowptr, np.int64)
    col = np.asarray(col, np.int32)
    new_ptr = rowptr + np.arange(n_loc + 1, dtype=np.int64)
    new_col = np.zeros(int(new_ptr[-1]), np.int32)
    val = np.ones(int(new_ptr[-1]), np.float64)
    for i in range(n_loc):
        a, b = int(rowptr[i]), int(rowptr[i + 1])
        q = int(new_ptr[i])
        new_col[q: q + b - a] = col[a:b]
        new_col[q + b - a] = i
        val[q + b - a] = 1.0 + eps
    return Graph(n_loc, n_loc + n_halo, new_ptr, new_col, np.ones(n_loc), np.ones(n_loc + n_halo), val)


# ------------------------------------------------------------------ layers
@dataclass
class Layer:
    kind: str                     # 'gcn' | 'sage'
    W: np.ndarray                 # [f_in, f_out]
    bias: Optional[np.ndarray]    # [f_out] or None
    act: str = "relu"             # 'relu' | 'none'
    W_self: Optional[np.ndarray] = None

    @staticmethod
    def of(p) -> "Layer":
        """From a synthetic LayerParams record (float32 arrays widened exactly)."""
        return Layer(p.kind, _f64(p.W), None if p.bias is None else _f64(p.bias), p.act,
                     None if p.W_self is None else _f64(p.W_self))


def layer_fwd(g: Graph, l: Layer, X):
    """X is [n_cols, f_in] = [local rows; halo rows].  Returns (H [n_loc, f_out], saved)."""
    X = _f64(X)
    M = spmm_fwd(g, X)                                   # aggregate
    Z = matmul(M, l.W)                                   # combine
    if l.kind == "sage":
        Z = Z + matmul(X[: g.n_loc], l.W_self)
    if l.bias is not None:
        Z = Z + l.bias[None, :]
    H = np.maximum(Z, 0.0) if l.act == "relu" else Z
    return H, {"M": M, "Z": Z}


def layer_bwd(g: Graph, l: Layer, X, saved, dH, need_dx: bool = True):
    """Chain rule of layer_fwd.  Returns dict(dW, dW_self, db, dX, dZ) with dX over all n_cols rows.  The factor
    sigma'(Z) of the backward recursion is decided here, from this side's own fp64 Z, and by nothing else."""
    X = _f64(X)
    dH = _f64(dH)
    if l.act == "relu":
        dZ = dH * (saved["Z"] > 0.0)                     # sigma'(0) = 0
    else:
        dZ = dH
    out = {"db": dZ.sum(axis=0), "dW": matmul(saved["M"], dZ, ta=True), "dW_self": None, "dX": None, "dZ": dZ}
    if l.kind == "sage":
        out["dW_self"] = matmul(X[: g.n_loc], dZ, ta=True)
    if need_dx:
        dM = matmul(dZ, l.W, tb=True)                    # [n_loc, f_in]
        dX = spmm_bwd(g, dM)                             # [n_cols, f_in]
        if l.kind == "sage":
            dX[: g.n_loc] += matmul(dZ, l.W_self, tb=True)
        out["dX"] = dX
    return out


def epoch(g: Graph, layers: List[Layer], X0_local, halo_tables: Sequence[Optional[np.ndarray]],
          labels, mask=None, loss_norm: float = 0.0, lr: float = 0.0, halo_grad: bool = False,
          loss_kind: str = "ce"):
    """One full-batch forward + backward over the partition.

    halo_tables[l] is the logical [n_halo, f_in(l)] cache table feeding layer l (None when the
    partition has no halo).  loss_kind "ce": labels are class indices (single-label tasks); "bce": labels is the
    [n_loc, classes] 0/1 target matrix (multi-label tasks).  Returns dict(loss, logits, dW, dW_self, db, dX_halo,
    new_W ...) and the intermediate quantities of every layer l: X[l] its input [local rows; halo rows], M[l] the
    aggregated input, hidden[l] = Z_l, dH[l] the loss gradient with respect to its output, dZ[l] = dH[l] (.) sigma'(Z_l).
    """
    n_halo = g.n_cols - g.n_loc
    ids = np.arange(n_halo, dtype=np.int64)
    H = _f64(X0_local)
    Xs, saves = [], []
    for li, l in enumerate(layers):
        if n_halo > 0:
            rows, absent = gather(_f64(halo_tables[li]), ids)    # pick the halo rows from the cache
            assert absent == 0
            X = np.concatenate([H, rows], axis=0)
        else:
            X = H
        H, sv = layer_fwd(g, l, X)
        Xs.append(X)
        saves.append(sv)
    logits = H
    loss, dH = (softmax_ce if loss_kind == "ce" else sigmoid_bce)(logits, labels, mask, loss_norm)
    res = {"loss": loss, "logits": logits, "dW": [None] * len(layers), "dW_self": [None] * len(layers),
           "db": [None] * len(layers), "dX_halo": [None] * len(layers), "hidden": [s["Z"] for s in saves],
           "X": Xs, "M": [s["M"] for s in saves], "dH": [None] * len(layers), "dZ": [None] * len(layers)}
    for li in range(len(layers) - 1, -1, -1):
        need_dx = li > 0 or halo_grad
        res["dH"][li] = dH
        b = layer_bwd(g, layers[li], Xs[li], saves[li], dH, need_dx=need_dx)
        res["dW"][li], res["dW_self"][li], res["db"][li], res["dZ"][li] = b["dW"], b["dW_self"], b["db"], b["dZ"]
        if b["dX"] is not None:
            res["dX_halo"][li] = b["dX"][g.n_loc:]
            dH = b["dX"][: g.n_loc]
    if lr:
        res["new_W"] = [l.W - lr * res["dW"][i] for i, l in enumerate(layers)]
        res["new_W_self"] = [None if l.W_self is None else l.W_self - lr * res["dW_self"][i]
                             for i, l in enumerate(layers)]
        res["new_bias"] = [None if l.bias is None else l.bias - lr * res["db"][i] for i, l in enumerate(layers)]
    return res


# ------------------------------------------------------------------ RAPA: cost model and subgraph adjustment
@dataclass
class RapaDevice:
    """Measured costs of one GPU on the reference operations (section "Communication and Computation Modeling"): the
    time of the reference SpMM and MM, and of the reference transfer host-to-device, device-to-host and between
    devices.  Only the ratios to the largest value among the GPUs enter the cost (reading: F and t are measured costs,
    so that the slowest GPU has ratio 1), and the memory available on the GPU in bytes."""
    t_spmm: float
    t_mm: float
    f_h2d: float
    f_d2h: float
    f_idt: float
    mem_bytes: float


@dataclass
class RapaParams:
    alpha: float            # weight between the SpMM term (edges) and the MM term (inner vertices) of Eq. 4
    epsilon: float          # stop when the standard deviation of the costs falls below it
    m_vertex: float = 8.0   # bytes to store one vertex
    m_edge: float = 12.0    # bytes to store one edge
    m_feat: float = 4.0     # bytes of one feature element
    f_dim: int = 0          # feature width
    beta: float = 100.0 * 2 ** 20   # memory reserved for gradients and the like (the evaluation uses 100 MB)
    max_sweeps: int = 1000


def rapa_cost(n_inner: int, e_all: int, e_outer: int, i: int, devs: Sequence[RapaDevice], prm: RapaParams) -> float:
    """lambda_i = T_comp + T_comm of subgraph i on GPU i (Eq. 3 and Eq. 4):
    T_comm = |E_outer| ((F_h2d/Fmax_h2d + F_d2h/Fmax_d2h)(1 - 1/P) + F_idt/Fmax_idt / P),
    T_comp = alpha |E_all| t_spmm/tmax_spmm + (1 - alpha) |V_inner| t_mm/tmax_mm."""
    P = len(devs)
    d = devs[i]
    mx = lambda name: max(getattr(x, name) for x in devs)
    t_comm = e_outer * ((d.f_h2d / mx("f_h2d") + d.f_d2h / mx("f_d2h")) * (1.0 - 1.0 / P) + d.f_idt / mx("f_idt") * (1.0 / P))
    t_comp = prm.alpha * e_all * (d.t_spmm / mx("t_spmm")) + (1.0 - prm.alpha) * n_inner * (d.t_mm / mx("t_mm"))
    return t_comp + t_comm


def rapa_memory_ok(n_vertices: int, n_edges: int, dev: RapaDevice, prm: RapaParams) -> bool:
    """The memory constraint of Eq. 5 (reading: the feature term counts f_dim elements for every vertex)."""
    need = n_vertices * prm.m_vertex + n_edges * prm.m_edge + n_vertices * prm.f_dim * prm.m_feat + prm.beta
    return dev.mem_bytes >= need


def rapa_do_partition(n_inner: Sequence[int], e_inner: Sequence[int], halo_edges: Sequence[np.ndarray],
                      scores: Sequence[np.ndarray], devs: Sequence[RapaDevice], prm: RapaParams):
    """Alg. 2 (do_partition) around Alg. 3 (adjust_subgraph), step by step.

    Subgraph i has n_inner[i] inner vertices, e_inner[i] edges between inner vertices, and halo vertices k with
    halo_edges[i][k] edges each (all of them outer edges); scores[i][k] is the influence score S_k (Eq. 6).
    Every sweep visits the GPUs from the weakest on (largest alpha t_spmm/tmax + (1 - alpha) t_mm/tmax, ties by
    index): a subgraph whose cost is at most the mean cost and whose memory suffices is marked done (r_i = 1);
    otherwise its halo vertices are taken in ascending score order (ties by index) and removed one by one, with all
    their edges, while the estimated cost exceeds the mean, stopping early once it is at most halfway between the old
    cost and the mean and the memory suffices; a subgraph from which nothing was removed is marked done.  The sweeps
    end when the standard deviation of the costs is below epsilon or every subgraph is marked done.
    Returns dict(keep: per-subgraph boolean arrays, lam: final costs, r: last status vector, sweeps, sigma: the
    standard deviation after every sweep, removed_order: per subgraph the halo vertices in the order of removal)."""
    P = len(devs)
    keep = [np.ones(len(h), bool) for h in halo_edges]
    cnt = [np.asarray(h, np.int64) for h in halo_edges]
    order = [sorted(range(len(cnt[i])), key=lambda k: (float(scores[i][k]), k)) for i in range(P)]
    nxt = [0] * P
    removed_order = [[] for _ in range(P)]
    mx_s, mx_m = max(d.t_spmm for d in devs), max(d.t_mm for d in devs)
    weakest_first = sorted(range(P), key=lambda i: (-(prm.alpha * devs[i].t_spmm / mx_s + (1.0 - prm.alpha) * devs[i].t_mm / mx_m), i))

    def stats(i):
        e_outer = int(cnt[i][keep[i]].sum())
        return n_inner[i], e_inner[i] + e_outer, e_outer, n_inner[i] + int(keep[i].sum())

    def lam(i):
        ni, ea, eo, _ = stats(i)
        return rapa_cost(ni, ea, eo, i, devs, prm)

    def mem_ok(i):
        _, ea, _, nv = stats(i)
        return rapa_memory_ok(nv, ea, devs[i], prm)

    sigma, sweeps, r = [], 0, [0] * P
    while True:
        r = [0] * P
        for i in weakest_first:                                   # ---- adjust_subgraph
            lam_i = lam(i)
            lam_bar = sum(lam(j) for j in range(P)) / P
            if lam_i <= lam_bar and mem_ok(i):
                r[i] = 1
                continue
            removed_now = 0
            lam_hat = lam_i
            while lam_hat > lam_bar and nxt[i] < len(order[i]):
                k = order[i][nxt[i]]
                nxt[i] += 1
                keep[i][k] = False
                removed_order[i].append(k)
                removed_now += 1
                lam_hat = lam(i)
                if lam_hat <= 0.5 * (lam_i + lam_bar) and mem_ok(i):
                    break
            if removed_now == 0:
                r[i] = 1
        sweeps += 1                                               # ---- do_partition
        lams = [lam(i) for i in range(P)]
        mean = sum(lams) / P
        sigma.append(float(np.sqrt(sum((x - mean) ** 2 for x in lams) / P)))
        if sigma[-1] < prm.epsilon or all(r) or sweeps >= prm.max_sweeps:
            break
    return {"keep": keep, "lam": [lam(i) for i in range(P)], "r": r, "sweeps": sweeps, "sigma": sigma,
            "removed_order": removed_order}


def halo_edge_counts(n_loc: int, n_halo: int, rowptr, col):
    """(edges between inner vertices, edges per halo vertex) of a partition graph."""
    col = np.asarray(col, np.int64)
    e_inner = int((col < n_loc).sum())
    cnt = np.zeros(n_halo, np.int64)
    for c in col[col >= n_loc]:
        cnt[c - n_loc] += 1
    return e_inner, cnt


def prune_halo(n_loc: int, n_halo: int, rowptr, col, keep):
    """The subgraph after the halo vertices with keep[k] == False are removed with all their edges ("Remove V_rem and
    E_rem from G_i"): the kept halo vertices are renumbered in their old order.  Returns (rowptr, col, new_index) with
    new_index[k] = the new halo-local index of old halo vertex k, -1 if removed."""
    rowptr = np.asarray(rowptr, np.int64)
    col = np.asarray(col, np.int64)
    keep = np.asarray(keep, bool)
    new_index = np.full(n_halo, -1, np.int64)
    q = 0
    for k in range(n_halo):
        if keep[k]:
            new_index[k] = q
            q += 1
    new_ptr, new_col = [0], []
    for i in range(n_loc):
        for e in range(rowptr[i], rowptr[i + 1]):
            c = col[e]
            if c < n_loc:
                new_col.append(c)
            elif keep[c - n_loc]:
                new_col.append(n_loc + new_index[c - n_loc])
        new_ptr.append(len(new_col))
    return np.array(new_ptr, np.int64), np.array(new_col, np.int32), new_index
