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


def oracle_epoch(prob, lr: float = 0.0, use_mask: bool = True, halo_grad: bool = False):
    g = oracle_graph(prob.part, prob.cfg.kind, float(prob.cfg.extra.get("gin_eps", 0.0)))
    layers = oracle_layers(prob)
    tables = [widen(t) for t in prob.tables]
    if prob.targets is not None:
        return orc.epoch(g, layers, widen(prob.X0), tables, prob.targets.astype(np.float64), prob.mask if use_mask else None,
                         0.0, lr, halo_grad=halo_grad, loss_kind="bce")
    return orc.epoch(g, layers, widen(prob.X0), tables, prob.labels, prob.mask if use_mask else None, 0.0, lr,
                     halo_grad=halo_grad)


def oracle_layers(prob):
    layers = [orc.Layer.of(p) for p in prob.model]
    for l in layers:
        if l.kind == "gin":
            l.kind = "gcn"                    # sigma(A X W + b) on the GIN operator
    return layers


# ----------------------------------------------------------------------------- error metrics
def normwise(gpu: np.ndarray, ref: np.ndarray, slack=None) -> float:
    """max(|gpu - ref| - slack, 0) / max|ref| (infinity-norm-wise relative error; slack: see flip_slack)."""
    ref = np.asarray(ref, np.float64)
    gpu = np.asarray(gpu, np.float64)
    if not ref.size:
        return 0.0
    diff = np.abs(gpu - ref)
    if slack is not None:
        diff = np.maximum(diff - slack, 0.0)
    den = np.abs(ref).max()
    return float(diff.max() if den == 0.0 else diff.max() / den)


def elementwise(gpu: np.ndarray, ref: np.ndarray, slack=None, by_row: bool = False) -> float:
    """max over elements of max(|gpu - ref| - slack, 0) / (|ref| + rms(ref)): the element-wise metric that goes with
    the norm-wise one (a bar of tol means |gpu - ref| <= tol * (|ref| + rms(ref)) for every element).  by_row: rms
    over the element's own row, so that rows of large entries (hub vertices) cannot vouch for rows of small ones
    (rows narrower than 16 elements fall back to the whole tensor: the rms of a handful of signed sums is itself
    a matter of cancellation)."""
    ref = np.asarray(ref, np.float64)
    gpu = np.asarray(gpu, np.float64)
    if not ref.size:
        return 0.0
    diff = np.abs(gpu - ref)
    if slack is not None:
        diff = np.maximum(diff - slack, 0.0)
    if by_row and ref.ndim == 2 and ref.shape[1] >= 16:
        rms = np.sqrt((ref * ref).mean(axis=1, keepdims=True))
    else:
        rms = np.sqrt((ref * ref).mean())
    den = np.abs(ref) + rms
    ok = den > 0
    worst = float((diff[ok] / den[ok]).max()) if ok.any() else 0.0
    if (~ok).any() and diff[~ok].max() > 0:      # reference row identically zero: any deviation counts in full
        worst = max(worst, float(diff[~ok].max()))
    return worst


def rowwise(gpu: np.ndarray, ref: np.ndarray, slack=None) -> float:
    """The norm-wise error of the worst row: max_i ( max_j (|gpu - ref| - slack)[i,j] / max(max_j |ref[i,j]|, rms(ref)) );
    a vector counts as one row.  The per-row metric of the parameter gradients: every element of a weight gradient
    is a sum over all vertices of signed terms, so its rounding noise scales with the row's magnitude, not with its
    own; the floor rms(ref) keeps the rows of (nearly) dead hidden units, whose entries are all but zero, from
    being measured against nothing."""
    ref = np.asarray(ref, np.float64)
    gpu = np.asarray(gpu, np.float64)
    if ref.ndim != 2:
        return normwise(gpu, ref, slack)
    if not ref.size:
        return 0.0
    diff = np.abs(gpu - ref)
    if slack is not None:
        diff = np.maximum(diff - slack, 0.0)
    num = diff.max(axis=1)
    den = np.maximum(np.abs(ref).max(axis=1), np.sqrt((ref * ref).mean()))
    ok = den > 0
    worst = float((num[ok] / den[ok]).max()) if ok.any() else 0.0
    if (~ok).any():
        worst = max(worst, float(num[~ok].max()))
    return worst


# ----------------------------------------------------------------------------- ReLU decisions under rounding
# Unit roundoff of the two storage types (round to nearest even): 24 and 8 significant bits.
UNIT_ROUNDOFF = {"f32": 2.0 ** -24, "bf16": 2.0 ** -8}


def _sq_graph(g):
    return orc.Graph(g.n_loc, g.n_cols, g.rowptr, g.col, g.r * g.r, g.c * g.c, None if g.v is None else g.v * g.v)


def _abs_graph(g):
    return orc.Graph(g.n_loc, g.n_cols, g.rowptr, g.col, np.abs(g.r), np.abs(g.c), None if g.v is None else np.abs(g.v))


def relu_bands(g, layers, ref, dtype: str, lam: float = 4.0):
    """For every hidden layer l, an element-wise band e_l >= |Z_impl - Z_ref| that an implementation of the forward
    pass in `dtype` storage with fp32 accumulation stays inside, from the oracle's own quantities alone.

    sigma'(Z) = 1[Z > 0] is an integer decided by a floating-point value: an implementation whose Z differs from the
    oracle's by rounding can only decide differently where |Z_ref| <= |Z_impl - Z_ref|.  The model is the usual
    root-sum-of-squares one (independent rounding errors): with u_s the unit roundoff of the storage type and
    u = 2^-24 that of the accumulator,
      var(Z) =   A2 var(X) W2                       rounding already present in the layer's input (local rows)
               + u_s^2 (M^2) W2 + u_s^2 A2 (XW)^2   the stored intermediate, whichever association is run
               + u^2 K (A2 X^2) W2                  K = entries of the row + f_in accumulation steps
               (+ the same three terms for the self transform of a GraphSAGE layer)
    where A2, W2 are the operator and the weights squared entry by entry and M = A X; the stored output adds
    u_s^2 Z^2 on its way into the next layer.  e_l = lam * sqrt(var(Z_l)); lam = 4 counts a full unit roundoff as
    one standard deviation (a uniform rounding error has u / sqrt(3)), i.e. about seven of them.
    Returns a list with one array per layer (None for layers without ReLU)."""
    us, ua = UNIT_ROUNDOFF[dtype], UNIT_ROUNDOFF["f32"]
    g2 = _sq_graph(g)
    n_loc = g.n_loc
    deg = np.diff(g.rowptr).astype(np.float64)
    bands, var_in = [], None                               # var_in: variance of the local rows of the layer input
    for l, ly in enumerate(layers):
        X, M, Z = ref["X"][l], ref["M"][l], ref["hidden"][l]
        f_in = X.shape[1]
        W2 = ly.W * ly.W
        X2 = X * X
        P = us * us * (M * M) + (ua * ua) * (deg + f_in)[:, None] * orc.spmm_fwd(g2, X2)
        if var_in is not None:
            vX = np.zeros_like(X)
            vX[:n_loc] = var_in
            P += orc.spmm_fwd(g2, vX)
        var = orc.matmul(P, W2)
        T = orc.matmul(X, ly.W)
        var += us * us * orc.spmm_fwd(g2, T * T)
        if ly.W_self is not None:
            Ws2 = ly.W_self * ly.W_self
            Q = (ua * ua) * f_in * X2[:n_loc]
            if var_in is not None:
                Q += var_in
            var += orc.matmul(Q, Ws2)
            S = orc.matmul(X[:n_loc], ly.W_self)
            var += us * us * (S * S + (Z - S) * (Z - S))   # the two partial results share one stored output
        if ly.act == "relu":
            bands.append(lam * np.sqrt(var))
            var_in = (var + us * us * Z * Z) * (Z > 0.0)
        else:
            bands.append(None)
            var_in = var + us * us * Z * Z
    return bands


def flip_slack(g, layers, ref, bands):
    """How far the gradients of an implementation may lie from the oracle's when its ReLU decisions differ from the
    oracle's inside S_l = {|Z_l| <= bands[l]} and nowhere else - computed from the oracle's quantities alone.

    The backward pass is linear in each layer's 0/1 factor.  With E_l >= |dZ_l(impl decisions) - dZ_l(oracle)|:
      E_l   = D_l (.) (1[Z_l > 0] or S_l)  +  |dH_l| (.) S_l          (D_l: what reaches dH_l from the layers above)
      |dW_l - dW_l^ref| <= |M_l|^T E_l,  |db_l - ..| <= 1^T E_l,  |dW_self,l - ..| <= |X_l,loc|^T E_l
      D_{l-1} = (|A_hat|^T (E_l |W_l|^T))[local rows] + E_l |W_self,l|^T
    Returns dict(dW, dW_self, db: per-layer element-wise slack arrays (None = exactly zero), in_band: |S_l| per layer)."""
    L = len(layers)
    ga = _abs_graph(g)
    n_loc = g.n_loc
    out = {"dW": [None] * L, "dW_self": [None] * L, "db": [None] * L, "in_band": [0] * L}
    D = None
    for l in range(L - 1, -1, -1):
        ly = layers[l]
        Z, dH = ref["hidden"][l], ref["dH"][l]
        if ly.act == "relu" and bands[l] is not None:
            S = np.abs(Z) <= bands[l]
            out["in_band"][l] = int(S.sum())
            E = np.abs(dH) * S
            if D is not None:
                E += D * ((Z > 0.0) | S)
        else:
            E = D
        if E is None or not E.any():
            D = None
            continue
        out["db"][l] = E.sum(axis=0)
        out["dW"][l] = orc.matmul(np.abs(ref["M"][l]), E, ta=True)
        if ly.W_self is not None:
            out["dW_self"][l] = orc.matmul(np.abs(ref["X"][l][:n_loc]), E, ta=True)
        if l > 0:
            D = orc.spmm_bwd(ga, orc.matmul(E, np.abs(ly.W), tb=True))[:n_loc]
            if ly.W_self is not None:
                D += orc.matmul(E, np.abs(ly.W_self), tb=True)
    return out


def relu_decisions_agree(Z_ref, H_impl, band):
    """(number of decisions 1[Z > 0] that differ, whether every one of them lies inside the band)."""
    differ = (Z_ref > 0.0) != (np.asarray(H_impl, np.float64) > 0.0)
    return int(differ.sum()), bool((np.abs(Z_ref[differ]) <= band[differ]).all())


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
