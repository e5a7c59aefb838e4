"""Seeded synthetic inputs: partitions, halo metadata, features, models, labels.

This module feeds BOTH the HIP path and the CPU oracle and therefore contains none of
the method's arithmetic: no normalisation, no aggregation, no placement, no layer maths.
It produces integer graph structure, integer per-vertex metadata (degrees, priorities,
global ids), random feature / weight tensors and the bf16 storage format conversion.

The graphs stand in for the datasets the paper trains on (dataset table of its
evaluation section: Reddit 232,965 nodes / 114.6 M edges / 602 features / 41 classes;
ogbn-products 2,449,029 / 61.9 M / 100 / 47), which are not available here; only those
published shapes are used.  A partition follows the paper's description of a
vertex-centric partition: rows exist for inner (local) vertices only, halo vertices
appear only as sources of cut edges.

Random numbers come from numpy's counter-based Philox generator keyed by
(seed, stream), so every array is reproducible independently of the others.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

BASE_SEED = 13716


def rng_for(seed: int, stream: int) -> np.random.Generator:
    key = np.array([np.uint64(seed), np.uint64(stream)], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


# --------------------------------------------------------------------------- bf16 format
def f32_to_bf16_rne(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns the uint16 bit pattern."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_to_f32(u: np.ndarray) -> np.ndarray:
    """Widen a uint16 bfloat16 bit pattern to float32 exactly."""
    return (np.ascontiguousarray(u, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- degree model
class _PowerLaw:
    """Ranks 0..n-1 drawn with density proportional to (x+i0)^-alpha (continuous inverse-CDF, floored)."""

    def __init__(self, n: int, alpha: float, i0: float):
        self.n, self.alpha, self.i0 = n, alpha, i0
        self.one_minus = 1.0 - alpha
        if abs(self.one_minus) < 1e-9:
            self.a, self.b = np.log(i0), np.log(n + i0)
        else:
            self.a, self.b = i0 ** self.one_minus, (n + i0) ** self.one_minus

    def top_share(self) -> float:
        if abs(self.one_minus) < 1e-9:
            return float((np.log(1.0 + self.i0) - self.a) / (self.b - self.a))
        return float(((1.0 + self.i0) ** self.one_minus - self.a) / (self.b - self.a))

    def draw(self, rng: np.random.Generator, perm: np.ndarray, m: int) -> np.ndarray:
        u = rng.random(m)
        t = self.a + u * (self.b - self.a)
        if abs(self.one_minus) < 1e-9:
            x = np.exp(t)
        else:
            x = np.power(t, 1.0 / self.one_minus)
        idx = (x - self.i0).astype(np.int64)
        np.clip(idx, 0, self.n - 1, out=idx)
        return perm[idx]


def _calibrated(n: int, alpha: float, total: float, max_deg: float) -> _PowerLaw:
    """Offset i0 for which the heaviest vertex expects about max_deg of `total` draws."""
    target = max_deg / max(total, 1.0)
    lo, hi = 1e-3, float(max(n, 2))
    if _PowerLaw(n, alpha, lo).top_share() <= target:
        return _PowerLaw(n, alpha, lo)
    for _ in range(60):
        mid = float(np.sqrt(lo * hi))
        if _PowerLaw(n, alpha, mid).top_share() > target:
            lo = mid
        else:
            hi = mid
    return _PowerLaw(n, alpha, float(np.sqrt(lo * hi)))


@dataclass
class Partition:
    """One GPU's partition-local graph: CSR over local rows, columns = local then halo."""
    name: str
    n_loc: int
    n_halo: int
    rowptr: np.ndarray           # int64 [n_loc+1]
    col: np.ndarray              # int32 [nnz], sorted within a row, < n_loc+n_halo
    halo_gid: np.ndarray         # int64 [n_halo] unique global ids
    halo_prio: np.ndarray        # int64 [n_halo] cache priority (in-partition edge count)
    halo_degree: np.ndarray      # int64 [n_halo] degree of the halo vertex in the whole graph
    self_loops: bool
    symmetric: bool

    @property
    def n_cols(self) -> int:
        return self.n_loc + self.n_halo

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])


def make_partition(name: str, n_loc: int, n_halo: int, nnz: int, *, seed: int,
                   gamma: float = 2.1, max_deg: Optional[int] = None,
                   halo_edge_frac: float = 0.5, self_loops: bool = True,
                   symmetric: bool = False, halo_zipf: Optional[float] = None) -> Partition:
    """Chung-Lu style power-law partition.

    Rows (destinations) and local sources are drawn with probability proportional to
    (rank+i0)^(-1/(gamma-1)) under independent random relabelings, so hubs are scattered
    over the id range like in an unordered real graph.  Every halo vertex receives one
    guaranteed edge; the remaining halo edges follow a power law (or Zipf(halo_zipf)) over
    the halo vertices.  Duplicate edges are removed; self loops (i,i) are added for every
    local row when ``self_loops``.
    """
    n_cols = n_loc + n_halo
    alpha = 1.0 / (gamma - 1.0)
    rng = rng_for(seed, 1)
    md = max_deg if max_deg is not None else max(8, min(n_cols // 4, int(40 * nnz / max(n_loc, 1))))
    row_law = _calibrated(n_loc, alpha, nnz, md)
    row_perm = rng.permutation(n_loc)

    if symmetric:
        assert n_halo == 0
        m = nnz // 2
        u = row_law.draw(rng, row_perm, m)
        v = row_law.draw(rng, row_perm, m)
        keep = u != v
        u, v = u[keep], v[keep]
        rows = np.concatenate([u, v])
        cols = np.concatenate([v, u])
        del u, v
    else:
        n_he = int(round(nnz * halo_edge_frac)) if n_halo > 0 else 0
        n_he = max(n_he, n_halo)
        n_le = max(nnz - n_he, 0)
        col_perm = rng.permutation(n_loc)
        rows_l = row_law.draw(rng, row_perm, n_le)
        cols_l = row_law.draw(rng, col_perm, n_le)
        keep = rows_l != cols_l
        rows_l, cols_l = rows_l[keep], cols_l[keep]
        if n_halo > 0:
            if halo_zipf is not None:
                h_law = _PowerLaw(n_halo, halo_zipf, 1.0)
            else:
                h_law = _calibrated(n_halo, alpha, n_he, max(8, min(n_loc // 2, md)))
            h_perm = rng.permutation(n_halo)
            rows_g = row_law.draw(rng, row_perm, n_halo)            # one guaranteed edge each
            cols_g = np.arange(n_halo, dtype=np.int64) + n_loc
            rows_h = row_law.draw(rng, row_perm, n_he - n_halo)
            cols_h = h_law.draw(rng, h_perm, n_he - n_halo) + n_loc
            rows = np.concatenate([rows_l, rows_g, rows_h])
            cols = np.concatenate([cols_l, cols_g, cols_h])
        else:
            rows, cols = rows_l, cols_l

    if self_loops:
        d = np.arange(n_loc, dtype=np.int64)
        rows = np.concatenate([rows, d])
        cols = np.concatenate([cols, d])
    key = rows.astype(np.int64) * np.int64(n_cols) + cols.astype(np.int64)
    del rows, cols
    key = np.unique(key)                      # dedupe + sort by (row, col)
    rows = key // np.int64(n_cols)
    col = (key - rows * np.int64(n_cols)).astype(np.int32)
    del key
    counts = np.bincount(rows, minlength=n_loc).astype(np.int64)
    del rows
    rowptr = np.zeros(n_loc + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])

    rng2 = rng_for(seed, 2)
    if n_halo > 0:
        prio = np.bincount(col[col >= n_loc].astype(np.int64) - n_loc, minlength=n_halo).astype(np.int64)
        degree = prio * rng2.integers(1, 5, size=n_halo, dtype=np.int64)
        gid = np.unique(rng2.integers(0, 1 << 40, size=int(n_halo * 1.01) + 16, dtype=np.int64))
        while len(gid) < n_halo:               # vanishingly rare: collisions ate the slack
            extra = rng2.integers(0, 1 << 40, size=n_halo, dtype=np.int64)
            gid = np.unique(np.concatenate([gid, extra]))
        gid = rng2.permutation(gid)[:n_halo].astype(np.int64)
    else:
        prio = np.zeros(0, np.int64)
        degree = np.zeros(0, np.int64)
        gid = np.zeros(0, np.int64)
    return Partition(name, n_loc, n_halo, rowptr, col, gid, prio, degree, self_loops, symmetric)


def make_clustered_partition(name: str, n_loc: int, avg_deg: int, window: int, *, seed: int,
                             shuffle: bool = True) -> Partition:
    """Undirected graph with geometric locality and a numbering that hides it: vertex u is joined to about
    avg_deg vertices drawn uniformly from u's `window` nearest positions on a ring, then (with ``shuffle``) the
    vertex labels are permuted at random.  Stand-in for a graph with community structure stored in arrival order,
    the case a locality reordering is for.  No halo, self loops added, both directions stored."""
    rng = rng_for(seed, 5)
    m = n_loc * avg_deg // 2
    u = rng.integers(0, n_loc, size=m, dtype=np.int64)
    off = rng.integers(1, window // 2 + 1, size=m, dtype=np.int64) * rng.choice(np.array([-1, 1], np.int64), size=m)
    v = (u + off) % n_loc
    if shuffle:
        lab = rng.permutation(n_loc).astype(np.int64)
        u, v = lab[u], lab[v]
    d = np.arange(n_loc, dtype=np.int64)
    rows = np.concatenate([u, v, d])
    cols = np.concatenate([v, u, d])
    key = np.unique(rows * np.int64(n_loc) + cols)
    rows = key // np.int64(n_loc)
    col = (key - rows * np.int64(n_loc)).astype(np.int32)
    rowptr = np.zeros(n_loc + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows, minlength=n_loc), out=rowptr[1:])
    z = np.zeros(0, np.int64)
    return Partition(name, n_loc, 0, rowptr, col, z, z, z, True, True)


def make_halo_sets(n: int, nnz: int, n_parts: int, *, seed: int, gamma: float = 2.1, max_deg: Optional[int] = None):
    """Halo sets of a random n_parts-way vertex partition of one power-law graph (the paper's "Random"
    pre-partitioning): H_i = the vertices outside part i that are sources of edges into part i.  Returns
    (list of sorted unique int64 arrays of global vertex ids, part id of every vertex)."""
    alpha = 1.0 / (gamma - 1.0)
    rng = rng_for(seed, 7)
    md = max_deg if max_deg is not None else max(8, min(n // 4, int(40 * nnz / max(n, 1))))
    law = _calibrated(n, alpha, nnz, md)
    dst = law.draw(rng, rng.permutation(n), nnz)
    src = law.draw(rng, rng.permutation(n), nnz)
    part = rng.integers(0, n_parts, size=n, dtype=np.int64)
    cut = part[dst] != part[src]
    dst_part, src_v = part[dst[cut]], src[cut]
    sets = [np.unique(src_v[dst_part == i]).astype(np.int64) for i in range(n_parts)]
    return sets, part


def hand_partition(n_loc: int, n_halo: int, edges, *, seed: int = 7, self_loops: bool = False,
                   name: str = "hand") -> Partition:
    """Partition from an explicit (row, col) edge list (duplicates kept: they act as multiplicity)."""
    n_cols = n_loc + n_halo
    e = np.asarray(list(edges), dtype=np.int64).reshape(-1, 2)
    if self_loops:
        d = np.arange(n_loc, dtype=np.int64)
        e = np.concatenate([e, np.stack([d, d], 1)])
    order = np.lexsort((e[:, 1], e[:, 0])) if len(e) else np.zeros(0, np.int64)
    e = e[order]
    rowptr = np.zeros(n_loc + 1, np.int64)
    if len(e):
        np.cumsum(np.bincount(e[:, 0], minlength=n_loc), out=rowptr[1:])
    col = e[:, 1].astype(np.int32) if len(e) else np.zeros(0, np.int32)
    rng = rng_for(seed, 3)
    prio = np.bincount(col[col >= n_loc].astype(np.int64) - n_loc, minlength=n_halo).astype(np.int64) \
        if n_halo else np.zeros(0, np.int64)
    degree = prio * rng.integers(1, 5, size=n_halo, dtype=np.int64) if n_halo else np.zeros(0, np.int64)
    gid = rng.permutation(np.arange(n_halo, dtype=np.int64) * 7919 + 1000003) if n_halo else np.zeros(0, np.int64)
    assert col.size == 0 or (col.min() >= 0 and col.max() < n_cols)
    return Partition(name, n_loc, n_halo, rowptr, col, gid, prio, degree, self_loops, False)


def make_partitioned_graph(n: int, nnz: int, n_parts: int, *, seed: int, shares: Optional[List[float]] = None,
                           gamma: float = 2.1, max_deg: Optional[int] = None):
    """One power-law graph cut into n_parts subgraphs by a random vertex assignment (part p with probability
    shares[p]; equal shares when omitted), each returned as a Partition: rows = the part's vertices in ascending
    global id, columns = those vertices followed by the part's halo vertices (sources of cut edges, ascending
    global id).  halo_gid = global vertex id, halo_prio = the number of subgraphs whose halo set holds the vertex
    (its repetition count), halo_degree = its in-degree in the whole graph.  Returns (list of Partition, dict with
    part: part id of every vertex, in_degree: in-degree of every vertex in the whole graph)."""
    alpha = 1.0 / (gamma - 1.0)
    rng = rng_for(seed, 8)
    md = max_deg if max_deg is not None else max(8, min(n // 4, int(40 * nnz / max(n, 1))))
    law = _calibrated(n, alpha, nnz, md)
    dst = law.draw(rng, rng.permutation(n), nnz)
    src = law.draw(rng, rng.permutation(n), nnz)
    ok = dst != src
    key = np.unique(dst[ok].astype(np.int64) * np.int64(n) + src[ok].astype(np.int64))      # dedupe, sort by (dst, src)
    dst, src = key // np.int64(n), key % np.int64(n)
    p = np.full(n_parts, 1.0 / n_parts) if shares is None else np.asarray(shares, np.float64) / np.sum(shares)
    part = rng.choice(n_parts, size=n, p=p).astype(np.int64)
    in_degree = np.bincount(dst, minlength=n).astype(np.int64)
    halo_sets = []
    for i in range(n_parts):
        sel = (part[dst] == i) & (part[src] != i)
        halo_sets.append(np.unique(src[sel]))
    repeat = np.zeros(n, np.int64)
    for h in halo_sets:
        repeat[h] += 1
    parts = []
    for i in range(n_parts):
        loc = np.nonzero(part == i)[0].astype(np.int64)
        halo = halo_sets[i]
        lut = np.full(n, -1, np.int64)
        lut[loc] = np.arange(len(loc))
        lut[halo] = len(loc) + np.arange(len(halo))
        sel = part[dst] == i
        rows, cols = lut[dst[sel]], lut[src[sel]]
        assert (rows >= 0).all() and (rows < len(loc)).all() and (cols >= 0).all()
        order = np.lexsort((cols, rows))
        rows, cols = rows[order], cols[order]
        rowptr = np.zeros(len(loc) + 1, np.int64)
        np.cumsum(np.bincount(rows, minlength=len(loc)), out=rowptr[1:])
        parts.append(Partition(f"part{i}of{n_parts}", len(loc), len(halo), rowptr, cols.astype(np.int32), halo.astype(np.int64),
                               repeat[halo], np.maximum(in_degree[halo], 1), False, False))
    return parts, {"part": part, "in_degree": in_degree}


# --------------------------------------------------------------------------- tensors
def pad_to(f: int, mult: int) -> int:
    return (f + mult - 1) // mult * mult


def make_features(n: int, f: int, *, seed: int, stream: int, dtype: str = "f32",
                  ld: Optional[int] = None) -> np.ndarray:
    """~N(0,1) rows, shape (n, ld) with columns [f, ld) zero.  dtype 'f32' -> float32, 'bf16' -> uint16 bits."""
    ld = f if ld is None else ld
    rng = rng_for(seed, stream)
    out = np.zeros((n, ld), dtype=np.float32)
    step = max(1, (1 << 24) // max(f, 1))
    for s in range(0, n, step):
        e = min(n, s + step)
        out[s:e, :f] = rng.standard_normal((e - s, f), dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_rne(out).reshape(n, ld)
    return out


@dataclass
class LayerParams:
    kind: str                    # 'gcn' | 'sage'
    f_in: int
    f_out: int
    act: str                     # 'relu' | 'none'
    W: np.ndarray                # float32 [f_in, f_out]   (GCN weight / SAGE neighbour weight)
    W_self: Optional[np.ndarray] # float32 [f_in, f_out]   (SAGE only)
    bias: np.ndarray             # float32 [f_out]


def make_model(kind: str, dims: List[int], *, seed: int, dtype: str = "f32") -> List[LayerParams]:
    """Glorot-uniform weights, small normal biases; with dtype 'bf16' the weights are pre-rounded to
    bf16-representable float32 values so that both sides consume identical numbers."""
    rng = rng_for(seed, 50)
    layers = []
    for l in range(len(dims) - 1):
        fi, fo = dims[l], dims[l + 1]
        lim = np.sqrt(6.0 / (fi + fo))
        def w():
            a = rng.uniform(-lim, lim, size=(fi, fo)).astype(np.float32)
            return bf16_to_f32(f32_to_bf16_rne(a)).reshape(fi, fo) if dtype == "bf16" else a
        W = w()
        Ws = w() if kind == "sage" else None
        b = (0.01 * rng.standard_normal(fo)).astype(np.float32)
        layers.append(LayerParams(kind, fi, fo, "relu" if l < len(dims) - 2 else "none", W, Ws, b))
    return layers


def make_labels(n: int, n_classes: int, *, seed: int, mask_frac: float = 1.0):
    rng = rng_for(seed, 60)
    y = rng.integers(0, n_classes, size=n, dtype=np.int32)
    if mask_frac >= 1.0:
        mask = np.ones(n, np.uint8)
    else:
        mask = (rng.random(n) < mask_frac).astype(np.uint8)
    return y, mask


def make_multilabels(n: int, n_classes: int, *, seed: int, density: float = 0.3) -> np.ndarray:
    """0/1 target matrix of a multi-label task, uint8 [n, n_classes]; every label set independently."""
    rng = rng_for(seed, 61)
    return (rng.random((n, n_classes)) < density).astype(np.uint8)


# --------------------------------------------------------------------------- named configs
@dataclass
class Config:
    name: str
    kind: str                    # 'gcn' | 'sage' | 'gin' (sum aggregation, extra["gin_eps"]; stored without self loops)
    n_loc: int
    n_halo: int
    nnz: int
    dims: List[int]              # [F_in, hidden..., classes]
    dtype: str                   # 'f32' | 'bf16'
    cache_frac: float            # share of halo vertices held in the GPU tier
    max_deg: Optional[int] = None
    halo_edge_frac: float = 0.5
    halo_zipf: Optional[float] = None
    symmetric: bool = False
    oversample: float = 1.0      # extra draws that make up for duplicate removal
    seed: int = BASE_SEED * 10
    extra: Dict = field(default_factory=dict)   # "loss": "bce" (multi-label targets), "gin_eps": float

    def scaled(self, s: float) -> "Config":
        """Same shape statistics at s times the vertex and edge counts (for quick parity runs)."""
        import copy
        c = copy.deepcopy(self)
        c.name = f"{self.name}@{s:g}"
        c.n_loc = max(64, int(self.n_loc * s))
        c.n_halo = int(self.n_halo * s) if self.n_halo else 0
        c.nnz = max(256, int(self.nnz * s))
        if self.max_deg:
            c.max_deg = max(16, min(self.max_deg, c.n_loc // 2))
        return c


CONFIGS: Dict[str, Config] = {
    # the five workloads named by the build's baseline description, in order
    "C1": Config("C1", "gcn", 4096, 4096, 40_000, [128, 64, 8], "f32", 1.0, max_deg=1000, seed=BASE_SEED * 10 + 1),
    "C2": Config("C2", "gcn", 60_000, 120_000, 28_000_000, [602, 256, 41], "f32", 0.5, max_deg=30_000,
                 oversample=1.1, seed=BASE_SEED * 10 + 2),
    "C3": Config("C3", "sage", 612_000, 700_000, 16_000_000, [100, 256, 256, 47], "f32", 0.3, max_deg=17_000,
                 halo_edge_frac=0.25, oversample=1.03, seed=BASE_SEED * 10 + 3),
    "C4": Config("C4", "gcn", 2_450_000, 0, 124_000_000, [128, 256, 256, 47], "bf16", 0.0, max_deg=17_000,
                 symmetric=True, seed=BASE_SEED * 10 + 4),
    "C5": Config("C5", "gcn", 1_000_000, 2_000_000, 40_000_000, [512, 256, 47], "bf16", 0.1, max_deg=20_000,
                 halo_zipf=1.1, oversample=1.12, seed=BASE_SEED * 10 + 5),
}


def partition_for(cfg: Config) -> Partition:
    return make_partition(cfg.name, cfg.n_loc, cfg.n_halo, int(cfg.nnz * cfg.oversample), seed=cfg.seed, max_deg=cfg.max_deg,
                          halo_edge_frac=cfg.halo_edge_frac, self_loops=(cfg.kind == "gcn"),   # GIN's self term is its own
                          symmetric=cfg.symmetric, halo_zipf=cfg.halo_zipf)


def cap_gpu_for(cfg: Config, part: Partition) -> int:
    return int(round(cfg.cache_frac * part.n_halo))
