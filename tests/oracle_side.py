"""Test helper: runs the CPU oracle on a harness.Problem (the same host arrays the HIP path consumes)."""
import numpy as np

from oracle import oracle as orc
from paper_2508_13716_amd import synth


def widen(a: np.ndarray) -> np.ndarray:
    """float64 view of a float32 array or of a uint16 bf16 bit pattern (exact)."""
    if a.dtype == np.uint16:
        return synth.bf16_to_f32(a).reshape(a.shape).astype(np.float64)
    return a.astype(np.float64)


def oracle_graph(part, kind: str, gin_eps: float = 0.0):
    if kind == "gin":
        return orc.gin_graph(part.n_loc, part.n_halo, part.rowptr, part.col, gin_eps)
    if kind == "gcn":
        return orc.gcn_graph(part.n_loc, part.n_halo, part.rowptr, part.col, part.halo_degree)
    return orc.mean_graph(part.n_loc, part.n_halo, part.rowptr, part.col)


def oracle_epoch(prob, lr: float = 0.0, use_mask: bool = True, halo_grad: bool = False, relu_on=None):
    g = oracle_graph(prob.part, prob.cfg.kind, float(prob.cfg.extra.get("gin_eps", 0.0)))
    layers = [orc.Layer.of(p) for p in prob.model]
    for l in layers:
        if l.kind == "gin":
            l.kind = "gcn"                    # sigma(A X W + b) on the GIN operator
    tables = [widen(t) for t in prob.tables]
    if prob.targets is not None:
        return orc.epoch(g, layers, widen(prob.X0), tables, prob.targets.astype(np.float64), prob.mask if use_mask else None,
                         0.0, lr, halo_grad=halo_grad, relu_on=relu_on, loss_kind="bce")
    return orc.epoch(g, layers, widen(prob.X0), tables, prob.labels, prob.mask if use_mask else None, 0.0, lr,
                     halo_grad=halo_grad, relu_on=relu_on)


def reconcile_relu_decisions(ref, gpu_hidden, band: float):
    """ReLU's backward factor 1[Z > 0] is an integer decided by a floating-point value.  Where the
    oracle's fp64 Z is zero within `band` (relative to max|Z| of the layer) the fp32 path may decide
    differently; there, and only there, the GPU's decision is adopted.  Elsewhere the two must agree.
    Returns (per-layer boolean arrays for oracle_epoch(relu_on=...), number of adopted decisions)."""
    out, adopted = [], 0
    for l, Z in enumerate(ref["hidden"]):
        if l >= len(gpu_hidden) or gpu_hidden[l] is None:
            out.append(None)
            continue
        on_ref = Z > 0.0
        on_gpu = widen(gpu_hidden[l]) > 0.0
        differ = on_ref != on_gpu
        tol = band * np.abs(Z).max()
        assert (np.abs(Z[differ]) <= tol).all(), f"layer {l}: ReLU decisions differ outside the rounding band"
        adopted += int(differ.sum())
        out.append(np.where(np.abs(Z) <= tol, on_gpu, on_ref))
    return out, adopted


def normwise(gpu: np.ndarray, ref: np.ndarray) -> float:
    """max|gpu - ref| / max|ref| (infinity-norm-wise relative error)."""
    ref = np.asarray(ref, np.float64)
    gpu = np.asarray(gpu, np.float64)
    den = np.abs(ref).max() if ref.size else 0.0
    if den == 0.0:
        return float(np.abs(gpu).max()) if gpu.size else 0.0
    return float(np.abs(gpu - ref).max() / den)


# ----------------------------------------------------------------------------- sampled outputs at full size
def sampled_fwd_graph(og, rows):
    """The oracle graph restricted to the output rows `rows` (renumbered 0..k-1) and to the columns those
    rows touch (renumbered; returned as J).  orc.spmm_fwd on it gives exactly the oracle's rows `rows`."""
    rows = np.asarray(rows, np.int64)
    starts, ends = og.rowptr[rows], og.rowptr[rows + 1]
    rowptr = np.zeros(len(rows) + 1, np.int64)
    np.cumsum(ends - starts, out=rowptr[1:])
    eidx = (np.concatenate([np.arange(s, e, dtype=np.int64) for s, e in zip(starts, ends)])
            if len(rows) else np.zeros(0, np.int64))
    J, inv = np.unique(og.col[eidx], return_inverse=True)
    v = None if og.v is None else og.v[eidx]
    return orc.Graph(len(rows), len(J), rowptr, inv.astype(np.int32), og.r[rows], og.c[J], v), J.astype(np.int64)


def sampled_bwd_graph(og, cols):
    """The oracle graph restricted to the entries whose column is in `cols` (columns renumbered in ascending
    order, rows that hold such entries renumbered; returned as R).  orc.spmm_bwd on it gives exactly the
    oracle's transposed product for those columns (entry order inside a column is kept)."""
    cols = np.unique(np.asarray(cols, np.int64))
    lut = np.full(og.n_cols, -1, np.int32)
    lut[cols] = np.arange(len(cols), dtype=np.int32)
    m = lut[og.col]
    eidx = np.nonzero(m >= 0)[0]
    erow = np.searchsorted(og.rowptr, eidx, side="right") - 1
    R, rinv = np.unique(erow, return_inverse=True)
    rowptr = np.zeros(len(R) + 1, np.int64)
    np.cumsum(np.bincount(rinv, minlength=len(R)), out=rowptr[1:])
    v = None if og.v is None else og.v[eidx]
    return orc.Graph(len(R), len(cols), rowptr, m[eidx].astype(np.int32), og.r[R], og.c[cols], v), R.astype(np.int64), cols


def sample_indices(lengths: np.ndarray, k: int, seed: int) -> np.ndarray:
    """k indices: the longest and the shortest few plus random ones (sorted, unique)."""
    n = len(lengths)
    rng = np.random.default_rng(seed)
    order = np.argsort(lengths, kind="stable")
    pick = np.concatenate([order[:8], order[-8:], rng.integers(0, n, size=max(k - 16, 0))])
    return np.unique(pick.astype(np.int64))


# ----------------------------------------------------------------------------- relabelled problems
def relabelled_problem(prob, new2old):
    """The same training problem with its vertices stored in the order new2old (CSR through the oracle's relabel;
    rows of the features, labels, mask, cache tables and halo attributes moved alike)."""
    import dataclasses
    part = prob.part
    nl = part.n_loc
    new2old = np.asarray(new2old, np.int64)
    pl, ph = new2old[:nl], new2old[nl:] - nl
    rowptr, col, _ = orc.relabel_csr(nl, part.rowptr, part.col, new2old)
    part2 = dataclasses.replace(part, name=part.name + "-relabelled", rowptr=rowptr, col=col,
                                halo_gid=part.halo_gid[ph], halo_prio=part.halo_prio[ph],
                                halo_degree=part.halo_degree[ph])
    return dataclasses.replace(prob, part=part2, X0=prob.X0[pl], tables=[t[ph] for t in prob.tables],
                               labels=prob.labels[pl], mask=prob.mask[pl])
