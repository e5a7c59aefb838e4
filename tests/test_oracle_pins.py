"""Pins for the CPU oracle: each oracle routine is checked against something other than itself.

Dense-adjacency brute force written here in numpy, closed forms, the adjoint identity, central
finite differences, textbook special cases, and the perturbation bound of Lemma 2.
None of these tests needs a GPU.
"""
import itertools
import math
import os

import numpy as np
import pytest

from paper_2508_13716_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers
def dense_adj(part, r, c, v=None):
    """A_hat as a dense [n_loc, n_cols] float64 matrix, built edge by edge (duplicates add up)."""
    A = np.zeros((part.n_loc, part.n_cols))
    for i in range(part.n_loc):
        for e in range(part.rowptr[i], part.rowptr[i + 1]):
            A[i, part.col[e]] += (1.0 if v is None else v[e]) * r[i] * c[part.col[e]]
    return A


def tiny_graphs():
    rng = np.random.default_rng(5)
    gs = []
    # random sparse with empty rows and duplicates
    e = [(int(rng.integers(0, 9)), int(rng.integers(0, 15))) for _ in range(40)]
    e = [x for x in e if x[0] not in (3, 7)] + [(0, 1), (0, 1), (0, 1)]
    gs.append(synth.hand_partition(9, 6, e, name="random+dups+empty"))
    # star: row 0 receives from everybody
    gs.append(synth.hand_partition(6, 4, [(0, j) for j in range(10)] + [(2, 9)], name="star"))
    # clique among locals with self loops, no halo
    gs.append(synth.hand_partition(5, 0, [(i, j) for i in range(5) for j in range(5) if i != j],
                                   self_loops=True, name="clique"))
    # generator output, small
    gs.append(synth.make_partition("cl", 40, 30, 400, seed=3, max_deg=25))
    # no edges at all
    gs.append(synth.hand_partition(4, 3, [], name="empty"))
    return gs


def sym_scales(part):
    """Symmetric normalisation written independently of the oracle (numpy)."""
    d = np.maximum(np.diff(part.rowptr), 1).astype(np.float64)
    r = d ** -0.5
    c = np.concatenate([r, np.maximum(part.halo_degree, 1).astype(np.float64) ** -0.5])
    return r, c


# ----------------------------------------------------------------------------- SpMM forward
@pytest.mark.parametrize("gi", range(5))
def test_spmm_fwd_vs_dense_bruteforce(orc, gi):
    part = tiny_graphs()[gi]
    rng = np.random.default_rng(100 + gi)
    r = rng.uniform(0.5, 2.0, part.n_loc)
    c = rng.uniform(0.5, 2.0, part.n_cols)
    v = rng.uniform(-1.0, 1.0, part.nnz)
    X = rng.standard_normal((part.n_cols, 7))
    for vals in (None, v):
        g = orc.Graph(part.n_loc, part.n_cols, part.rowptr, part.col, r, c, vals)
        Y = orc.spmm_fwd(g, X)
        A = dense_adj(part, r, c, vals)
        ref = np.zeros_like(Y)
        for i in range(part.n_loc):              # triple loop, no library product
            for j in range(part.n_cols):
                if A[i, j] != 0.0:
                    ref[i] += A[i, j] * X[j]
        np.testing.assert_allclose(Y, ref, rtol=1e-12, atol=1e-13)
        dX = orc.spmm_bwd(g, rng.standard_normal((part.n_loc, 3)) * 0 + 1.0)
        np.testing.assert_allclose(dX, (A.T @ np.ones((part.n_loc, 3))), rtol=1e-12, atol=1e-13)


def test_gcn_scales_match_definition(orc):
    for part in tiny_graphs():
        g = orc.gcn_graph(part.n_loc, part.n_halo, part.rowptr, part.col, part.halo_degree)
        r, c = sym_scales(part)
        np.testing.assert_allclose(g.r, r, rtol=1e-15)
        np.testing.assert_allclose(g.c, c, rtol=1e-15)


def test_ones_aggregate_to_normalised_degree_sums(orc):
    """X = 1  =>  (A_hat X)[i,:] = r_i * sum_j A_ij c_j."""
    part = synth.make_partition("cl", 200, 150, 3000, seed=11, max_deg=60)
    g = orc.gcn_graph(part.n_loc, part.n_halo, part.rowptr, part.col, part.halo_degree)
    Y = orc.spmm_fwd(g, np.ones((part.n_cols, 4)))
    r, c = sym_scales(part)
    expect = np.array([r[i] * c[part.col[part.rowptr[i]:part.rowptr[i + 1]]].sum() for i in range(part.n_loc)])
    np.testing.assert_allclose(Y, np.repeat(expect[:, None], 4, 1), rtol=1e-13)


def test_regular_symmetric_graph_aggregates_ones_to_one(orc):
    """Ring with self loops: every degree is 3, so A_hat 1 = 1 exactly (up to rounding)."""
    n = 17
    e = [(i, (i + 1) % n) for i in range(n)] + [(i, (i - 1) % n) for i in range(n)]
    part = synth.hand_partition(n, 0, e, self_loops=True)
    g = orc.gcn_graph(n, 0, part.rowptr, part.col, part.halo_degree)
    Y = orc.spmm_fwd(g, np.ones((n, 3)))
    np.testing.assert_allclose(Y, 1.0, rtol=1e-14)
    # symmetric graph: transposed product equals the forward product
    X = np.random.default_rng(0).standard_normal((n, 5))
    np.testing.assert_allclose(orc.spmm_bwd(g, X), orc.spmm_fwd(g, X), rtol=1e-13, atol=1e-14)


def test_mean_aggregator_closed_forms(orc):
    part = tiny_graphs()[0]
    g = orc.mean_graph(part.n_loc, part.n_halo, part.rowptr, part.col)
    Y = orc.spmm_fwd(g, np.ones((part.n_cols, 2)))
    deg = np.diff(part.rowptr)
    np.testing.assert_allclose(Y[deg > 0], 1.0, rtol=1e-14)
    assert np.all(Y[deg == 0] == 0.0)
    # mean of distinct neighbours = numpy mean
    X = np.random.default_rng(1).standard_normal((part.n_cols, 3))
    Y = orc.spmm_fwd(g, X)
    for i in range(part.n_loc):
        nb = part.col[part.rowptr[i]:part.rowptr[i + 1]]
        if len(nb):
            np.testing.assert_allclose(Y[i], X[nb].mean(axis=0), rtol=1e-12, atol=1e-14)


# ----------------------------------------------------------------------------- transposed SpMM
def test_adjoint_identity(orc):
    """<A_hat X, Y> = <X, A_hat^T Y> for random X, Y."""
    part = synth.make_partition("cl", 300, 200, 5000, seed=12, max_deg=80)
    g = orc.gcn_graph(part.n_loc, part.n_halo, part.rowptr, part.col, part.halo_degree)
    rng = np.random.default_rng(2)
    g.v = rng.uniform(0.1, 1.0, part.nnz)
    X = rng.standard_normal((part.n_cols, 6))
    Y = rng.standard_normal((part.n_loc, 6))
    lhs = float((orc.spmm_fwd(g, X) * Y).sum())
    rhs = float((X * orc.spmm_bwd(g, Y)).sum())
    assert abs(lhs - rhs) <= 1e-12 * max(abs(lhs), 1.0)


def test_spmm_bwd_vs_dense_transpose(orc):
    for gi, part in enumerate(tiny_graphs()):
        rng = np.random.default_rng(200 + gi)
        r = rng.uniform(0.5, 2.0, part.n_loc)
        c = rng.uniform(0.5, 2.0, part.n_cols)
        g = orc.Graph(part.n_loc, part.n_cols, part.rowptr, part.col, r, c, None)
        dY = rng.standard_normal((part.n_loc, 4))
        np.testing.assert_allclose(orc.spmm_bwd(g, dY), dense_adj(part, r, c).T @ dY, rtol=1e-12, atol=1e-13)


# ----------------------------------------------------------------------------- dense product, loss
@pytest.mark.parametrize("ta,tb", list(itertools.product([False, True], repeat=2)))
def test_matmul_vs_triple_loop(orc, ta, tb):
    """The dense product of the combination step against its definition, C[i,j] = sum_k A[i,k] B[k,j], written out
    as three loops here (the oracle's routine is a library call; an operand taken transposed must be read so)."""
    rng = np.random.default_rng(3)
    A = rng.standard_normal((9, 13))          # logical [M=9, K=13]
    B = rng.standard_normal((13, 5))
    want = np.zeros((9, 5))
    for i in range(9):
        for j in range(5):
            s = 0.0
            for k in range(13):
                s += A[i, k] * B[k, j]
            want[i, j] = s
    out = orc.matmul(A.T.copy() if ta else A, B.T.copy() if tb else B, ta=ta, tb=tb)
    assert out.shape == (9, 5) and out.flags.c_contiguous
    np.testing.assert_allclose(out, want, rtol=1e-13, atol=1e-14)


def test_loss_closed_forms(orc):
    n, Cc = 11, 7
    y = np.arange(n, dtype=np.int32) % Cc
    loss, dZ = orc.softmax_ce(np.zeros((n, Cc)), y)
    assert abs(loss - math.log(Cc)) < 1e-14              # uniform logits
    np.testing.assert_allclose(dZ.sum(axis=1), 0.0, atol=1e-16)
    # one-hot confident logits -> loss -> 0
    Z = np.full((n, Cc), -50.0)
    Z[np.arange(n), y] = 50.0
    loss, _ = orc.softmax_ce(Z, y)
    assert loss < 1e-40 or loss == 0.0
    # shift invariance and mask
    rng = np.random.default_rng(4)
    Z = rng.standard_normal((n, Cc)) * 3
    mask = (rng.random(n) < 0.5).astype(np.uint8)
    l1, g1 = orc.softmax_ce(Z, y, mask)
    l2, g2 = orc.softmax_ce(Z + 1000.0, y, mask)
    assert abs(l1 - l2) < 1e-10
    assert np.all(g1[mask == 0] == 0.0)
    # against the textbook formula in numpy
    p = np.exp(Z - Z.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    ref = -(np.log(p[np.arange(n), y]) * mask).sum() / mask.sum()
    assert abs(l1 - ref) < 1e-12


def test_identity_graph_layer_is_dense_affine(orc):
    """No edges but self loops, unit scales: the GCN layer is X W + b (a textbook product)."""
    n, fi, fo = 23, 6, 4
    part = synth.hand_partition(n, 0, [], self_loops=True)
    g = orc.gcn_graph(n, 0, part.rowptr, part.col, part.halo_degree)
    rng = np.random.default_rng(6)
    X, W, b = rng.standard_normal((n, fi)), rng.standard_normal((fi, fo)), rng.standard_normal(fo)
    H, _ = orc.layer_fwd(g, orc.Layer("gcn", W, b, "none"), X)
    np.testing.assert_allclose(H, X @ W + b, rtol=1e-13, atol=1e-14)
    H, _ = orc.layer_fwd(g, orc.Layer("gcn", W, b, "relu"), X)
    np.testing.assert_allclose(H, np.maximum(X @ W + b, 0), rtol=1e-13, atol=1e-14)


def test_layer_fwd_vs_dense(orc):
    part = tiny_graphs()[3]
    rng = np.random.default_rng(7)
    X = rng.standard_normal((part.n_cols, 5))
    W, Ws, b = rng.standard_normal((5, 3)), rng.standard_normal((5, 3)), rng.standard_normal(3)
    g = orc.gcn_graph(part.n_loc, part.n_halo, part.rowptr, part.col, part.halo_degree)
    r, c = sym_scales(part)
    H, _ = orc.layer_fwd(g, orc.Layer("gcn", W, b, "relu"), X)
    np.testing.assert_allclose(H, np.maximum(dense_adj(part, r, c) @ X @ W + b, 0), rtol=1e-12, atol=1e-13)
    gm = orc.mean_graph(part.n_loc, part.n_halo, part.rowptr, part.col)
    deg = np.diff(part.rowptr).astype(np.float64)
    rm = np.where(deg > 0, 1.0 / np.maximum(deg, 1), 0.0)
    Am = dense_adj(part, rm, np.ones(part.n_cols))
    H, _ = orc.layer_fwd(gm, orc.Layer("sage", W, b, "none", Ws), X)
    np.testing.assert_allclose(H, X[:part.n_loc] @ Ws + Am @ X @ W + b, rtol=1e-12, atol=1e-13)


# ----------------------------------------------------------------------------- gradients
def _tiny_problem(orc, kind, seed):
    part = synth.make_partition("fd", 14, 9, 60, seed=seed, max_deg=8, self_loops=(kind == "gcn"))
    if kind == "gcn":
        g = orc.gcn_graph(part.n_loc, part.n_halo, part.rowptr, part.col, part.halo_degree)
    else:
        g = orc.mean_graph(part.n_loc, part.n_halo, part.rowptr, part.col)
    dims = [5, 4, 4, 3]
    rng = np.random.default_rng(seed)
    layers = []
    for l in range(3):
        layers.append(orc.Layer(kind, rng.standard_normal((dims[l], dims[l + 1])) * 0.7,
                                rng.standard_normal(dims[l + 1]) * 0.3, "relu" if l < 2 else "none",
                                rng.standard_normal((dims[l], dims[l + 1])) * 0.7 if kind == "sage" else None))
    X0 = rng.standard_normal((part.n_loc, dims[0]))
    tables = [rng.standard_normal((part.n_halo, dims[l])) for l in range(3)]
    y = rng.integers(0, 3, part.n_loc).astype(np.int32)
    mask = (rng.random(part.n_loc) < 0.7).astype(np.uint8)
    mask[0] = 1
    return g, layers, X0, tables, y, mask


@pytest.mark.parametrize("kind", ["gcn", "sage"])
def test_gradients_vs_central_finite_differences(orc, kind):
    g, layers, X0, tables, y, mask = _tiny_problem(orc, kind, 21)
    res = orc.epoch(g, layers, X0, tables, y, mask, halo_grad=True)
    h = 1e-6

    def loss_now():
        return orc.epoch(g, layers, X0, tables, y, mask)["loss"]

    def check(arr, grad, idxs):
        for idx in idxs:
            old = arr[idx]
            arr[idx] = old + h
            lp = loss_now()
            arr[idx] = old - h
            lm = loss_now()
            arr[idx] = old
            fd = (lp - lm) / (2 * h)
            assert abs(fd - grad[idx]) <= 1e-6 * max(1.0, abs(fd)) , (idx, fd, grad[idx])

    rng = np.random.default_rng(9)
    for li, l in enumerate(layers):
        check(l.W, res["dW"][li], list(np.ndindex(*l.W.shape)))
        check(l.bias, res["db"][li], list(np.ndindex(*l.bias.shape)))
        if kind == "sage":
            check(l.W_self, res["dW_self"][li], list(np.ndindex(*l.W_self.shape)))
        # halo rows of every layer input are leaves of the graph: their gradient is dX[n_loc:]
        T = tables[li]
        pick = [tuple(int(v) for v in (rng.integers(0, T.shape[0]), rng.integers(0, T.shape[1]))) for _ in range(8)]
        check(T, res["dX_halo"][li], pick)


def test_sigmoid_bce_textbook_two_class_equivalence_and_finite_differences(orc):
    """Multi-label loss: log 2 at zero logits; the textbook -[y log s + (1-y) log(1-s)] at moderate logits; for a
    single class it is the (already pinned) softmax cross-entropy of the two-class logits (z, 0); extreme logits
    neither overflow nor lose the linear tail; masked-off rows contribute nothing; gradient by central differences."""
    rng = np.random.default_rng(31)
    n, C = 11, 5
    Y = (rng.random((n, C)) < 0.4).astype(np.float64)
    loss, dZ = orc.sigmoid_bce(np.zeros((n, C)), Y)
    assert abs(loss - math.log(2.0)) < 1e-15 and np.allclose(dZ, (0.5 - Y) / (n * C), atol=1e-17)
    Z = rng.standard_normal((n, C)) * 3.0
    mask = (rng.random(n) < 0.6).astype(np.uint8)
    mask[0], mask[1] = 1, 0
    loss, dZ = orc.sigmoid_bce(Z, Y, mask)
    sig = 1.0 / (1.0 + np.exp(-Z))
    per = -(Y * np.log(sig) + (1.0 - Y) * np.log(1.0 - sig))
    on = mask.astype(bool)
    assert abs(loss - per[on].sum() / (on.sum() * C)) < 1e-13
    assert np.all(dZ[~on] == 0.0)
    loss_n, dZ_n = orc.sigmoid_bce(Z, Y, mask, norm=7.0)                       # explicit normaliser
    assert abs(loss_n * 7.0 - loss * on.sum() * C) < 1e-12 and np.allclose(dZ_n * 7.0, dZ * on.sum() * C, atol=1e-15)
    # one class: BCE(z, y) == CE([z, 0], class 0 if y else class 1)
    z1 = rng.standard_normal((n, 1)) * 4.0
    y1 = (rng.random((n, 1)) < 0.5).astype(np.float64)
    l_b, g_b = orc.sigmoid_bce(z1, y1, mask)
    l_c, g_c = orc.softmax_ce(np.concatenate([z1, np.zeros((n, 1))], 1), (1 - y1[:, 0]).astype(np.int32), mask)
    assert abs(l_b - l_c) < 1e-13 and np.allclose(g_b[:, 0], g_c[:, 0], atol=1e-15)
    # extreme logits
    Ze = np.array([[800.0, -800.0, 800.0, -800.0]])
    Ye = np.array([[1.0, 0.0, 0.0, 1.0]])
    le, ge = orc.sigmoid_bce(Ze, Ye)
    assert np.isfinite(le) and abs(le - 1600.0 / 4.0) < 1e-9
    assert np.allclose(ge, np.array([[0.0, 0.0, 1.0, -1.0]]) / 4.0, atol=1e-15)
    # central differences
    h = 1e-6
    for idx in [(0, 0), (0, 4), (5, 2), (10, 1), (1, 3)]:
        Zp, Zm = Z.copy(), Z.copy()
        Zp[idx] += h
        Zm[idx] -= h
        fd = (orc.sigmoid_bce(Zp, Y, mask)[0] - orc.sigmoid_bce(Zm, Y, mask)[0]) / (2 * h)
        assert abs(fd - dZ[idx]) < 1e-9


def test_gin_operator_vs_edge_loops_and_epoch_gradients(orc):
    """GIN aggregation (1+eps) x_i + sum over the stored neighbours, against loops over the edges; eps = -1 leaves
    the neighbour sum, an edgeless graph leaves (1+eps) X; a GIN network trained with the multi-label loss has
    gradients that match central differences (also pins the epoch's loss switch and edge-valued operators)."""
    rng = np.random.default_rng(33)
    part = synth.make_partition("gin", 14, 9, 60, seed=5, max_deg=8, self_loops=False)
    X = rng.standard_normal((part.n_cols, 6))
    for eps in (0.0, 0.3, -1.0):
        g = orc.gin_graph(part.n_loc, part.n_halo, part.rowptr, part.col, eps)
        want = np.zeros((part.n_loc, 6))
        for i in range(part.n_loc):
            want[i] = (1.0 + eps) * X[i]
            for e in range(part.rowptr[i], part.rowptr[i + 1]):
                want[i] += X[part.col[e]]
        assert np.allclose(orc.spmm_fwd(g, X), want, atol=1e-13)
    g0 = orc.gin_graph(4, 0, np.zeros(5, np.int64), np.zeros(0, np.int32), 0.25)
    assert np.allclose(orc.spmm_fwd(g0, X[:4]), 1.25 * X[:4], atol=1e-15)
    g = orc.gin_graph(part.n_loc, part.n_halo, part.rowptr, part.col, 0.3)
    dims = [6, 4, 3]
    layers = [orc.Layer("gcn", rng.standard_normal((dims[l], dims[l + 1])) * 0.5, rng.standard_normal(dims[l + 1]) * 0.2,
                        "relu" if l == 0 else "none") for l in range(2)]
    X0 = rng.standard_normal((part.n_loc, dims[0]))
    tables = [rng.standard_normal((part.n_halo, dims[l])) for l in range(2)]
    Y = (rng.random((part.n_loc, 3)) < 0.4).astype(np.float64)
    mask = (rng.random(part.n_loc) < 0.7).astype(np.uint8)
    mask[0] = 1
    res = orc.epoch(g, layers, X0, tables, Y, mask, loss_kind="bce", halo_grad=True)
    h = 1e-6
    for arr, grad, idxs in [(layers[0].W, res["dW"][0], [(0, 0), (5, 3), (2, 1)]), (layers[1].W, res["dW"][1], [(0, 0), (3, 2)]),
                            (layers[1].bias, res["db"][1], [(1,)]), (tables[1], res["dX_halo"][1], [(0, 0), (8, 3)]),
                            (tables[0], res["dX_halo"][0], [(4, 5)])]:
        for idx in idxs:
            old = arr[idx]
            arr[idx] = old + h
            lp = orc.epoch(g, layers, X0, tables, Y, mask, loss_kind="bce")["loss"]
            arr[idx] = old - h
            lm = orc.epoch(g, layers, X0, tables, Y, mask, loss_kind="bce")["loss"]
            arr[idx] = old
            fd = (lp - lm) / (2 * h)
            assert abs(fd - grad[idx]) <= 1e-6 * max(1.0, abs(fd)), (idx, fd, grad[idx])


def test_sgd_step_is_plain_descent(orc):
    g, layers, X0, tables, y, mask = _tiny_problem(orc, "gcn", 22)
    res = orc.epoch(g, layers, X0, tables, y, mask, lr=0.01)
    for i, l in enumerate(layers):
        np.testing.assert_allclose(res["new_W"][i], l.W - 0.01 * res["dW"][i], rtol=0, atol=0)
    # a small step along the negative gradient lowers the loss
    new_layers = [orc.Layer(l.kind, res["new_W"][i], res["new_bias"][i], l.act) for i, l in enumerate(layers)]
    assert orc.epoch(g, new_layers, X0, tables, y, mask)["loss"] < res["loss"]


# ----------------------------------------------------------------------------- Lemma 2
def test_stale_halo_rows_obey_lemma2_bound(orc):
    """Perturb the halo rows by at most eps in max-norm: max|Z~ - Z| <= eta^2 beta^2 eps (Lemma 2)."""
    part = synth.make_partition("l2", 60, 50, 900, seed=31, max_deg=30)
    g = orc.gcn_graph(part.n_loc, part.n_halo, part.rowptr, part.col, part.halo_degree)
    rng = np.random.default_rng(8)
    fi, fo, eps = 8, 6, 1e-3
    X = rng.uniform(-1, 1, (part.n_cols, fi))
    W = rng.uniform(-1, 1, (fi, fo))
    Xs = X.copy()
    Xs[part.n_loc:] += rng.uniform(-eps, eps, (part.n_halo, fi))
    l = orc.Layer("gcn", W, None, "none")
    Z, _ = orc.layer_fwd(g, l, X)
    Zs, _ = orc.layer_fwd(g, l, Xs)
    eta = max(part.n_cols, fi, fo)                     # largest column count among the factors
    beta = max(1.0, np.abs(X).max(), np.abs(W).max())  # entries of A_hat are <= 1
    assert np.abs(Zs - Z).max() <= eta ** 2 * beta ** 2 * eps
    # and the sharper elementwise bound that the proof's chain of inequalities implies
    r, c = sym_scales(part)
    rowsum = np.array([r[i] * c[part.col[part.rowptr[i]:part.rowptr[i + 1]]].sum() for i in range(part.n_loc)])
    assert np.abs(Zs - Z).max() <= rowsum.max() * fi * np.abs(W).max() * eps * (1 + 1e-12)


# ----------------------------------------------------------------------------- Eq. 6
def test_influence_score_vs_dense_bruteforce_and_closed_forms(orc):
    """Eq. 6 from a dense adjacency matrix, term by term as printed; a directed ring where every degree is 1
    (score = 2 C); a star whose centre feeds d leaves (centre d/sqrt(d) = sqrt(d), each leaf 1/sqrt(d)); and the
    identity sum_v S_v / C_v = 2 sum_e 1/sqrt(Din Dout) (every edge is one outgoing and one incoming term)."""
    rng = np.random.default_rng(15)
    part = synth.make_partition("infl", 40, 25, 400, seed=33, max_deg=20, self_loops=False)
    n_loc, n_cols = part.n_loc, part.n_cols
    A = np.zeros((n_loc, n_cols))                                   # A[i, j] = number of edges j -> i
    for i in range(n_loc):
        for e in range(part.rowptr[i], part.rowptr[i + 1]):
            A[i, part.col[e]] += 1
    din = np.maximum(A.sum(axis=1), 1) * rng.integers(1, 3, n_loc)  # "in the original graph": at least the local count
    dout = np.maximum(A.sum(axis=0), 1)
    C = rng.integers(1, 5, n_cols).astype(np.float64)
    want = np.zeros(n_cols)
    for v in range(n_cols):
        out_part = sum(A[j, v] / np.sqrt(din[j]) / np.sqrt(dout[v]) for j in range(n_loc))
        in_part = sum(A[v, j] / np.sqrt(dout[j]) / np.sqrt(din[v]) for j in range(n_cols)) if v < n_loc else 0.0
        want[v] = (out_part + in_part) * C[v]
    got = orc.influence_score(n_loc, n_cols, part.rowptr, part.col, din, dout, C)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)
    edge_terms = sum(A[i, j] / np.sqrt(din[i] * dout[j]) for i in range(n_loc) for j in range(n_cols))
    np.testing.assert_allclose((got / C).sum(), 2 * edge_terms, rtol=1e-12)
    # directed ring on n vertices, no halo: entry (i, i-1)
    n = 9
    rowptr = np.arange(n + 1, dtype=np.int64)
    col = ((np.arange(n) - 1) % n).astype(np.int32)
    C = np.arange(1, n + 1, dtype=np.float64)
    np.testing.assert_allclose(orc.influence_score(n, n, rowptr, col, np.ones(n), np.ones(n), C), 2 * C, rtol=1e-15)
    # star: halo vertex 0 (column d) feeds the d local leaves
    d = 16
    rowptr = np.arange(d + 1, dtype=np.int64)
    col = np.full(d, d, np.int32)
    dout = np.ones(d + 1)
    dout[d] = d
    S = orc.influence_score(d, d + 1, rowptr, col, np.ones(d), dout)
    np.testing.assert_allclose(S[d], np.sqrt(d), rtol=1e-15)
    np.testing.assert_allclose(S[:d], 1 / np.sqrt(d), rtol=1e-15)


# ----------------------------------------------------------------------------- cache side
def _sym_partition(n, edges, n_halo=0, halo_edges=()):
    """Undirected local graph (both directions stored, rows sorted, no duplicates) plus local->halo entries."""
    und = {(a, b) for a, b in edges if a != b} | {(b, a) for a, b in edges if a != b}
    return synth.hand_partition(n, n_halo, sorted(und) + [(i, n + h) for i, h in halo_edges], name="sym")


def test_locality_order_is_a_valid_order_and_matches_library_bfs(orc):
    """The vertex storage order: a permutation that keeps the local / halo ranges; 'popularity' is checked
    against its definition by brute force; 'bfs' on a connected graph with sorted rows is the textbook
    breadth-first order, taken here from scipy's graph routines; on a relabelled ring it restores bandwidth 2;
    components stay contiguous; halo vertices follow their first mention."""
    from scipy.sparse import csr_matrix
    from scipy.sparse.csgraph import breadth_first_order
    rng = np.random.default_rng(12)
    # validity + popularity on random partitions (duplicates, empty rows, unreferenced halo vertices)
    for seed in range(4):
        part = synth.make_partition("ord", 300, 200, 2500, seed=seed, max_deg=60)
        refs = np.bincount(part.col, minlength=part.n_cols)
        for method in ("popularity", "bfs"):
            o = orc.locality_order(method, part.n_loc, part.n_halo, part.rowptr, part.col)
            assert sorted(o.tolist()) == list(range(part.n_cols))
            assert (o[: part.n_loc] < part.n_loc).all() and (o[part.n_loc:] >= part.n_loc).all()
        o = orc.locality_order("popularity", part.n_loc, part.n_halo, part.rowptr, part.col)
        for seg in (o[: part.n_loc], o[part.n_loc:]):
            key = [(-int(refs[v]), int(v)) for v in seg]
            assert key == sorted(key)
    # bfs == scipy's breadth-first order from the longest row on a connected undirected graph
    n = 400
    ring = [(i, (i + 1) % n) for i in range(n)]
    chords = [(int(a), int(b)) for a, b in rng.integers(0, n, (300, 2))]
    part = _sym_partition(n, ring + chords)
    deg = np.diff(part.rowptr)
    root = int(np.flatnonzero(deg == deg.max())[0])
    A = csr_matrix((np.ones(part.nnz), part.col, part.rowptr), shape=(n, n))
    want = breadth_first_order(A, root, directed=True, return_predecessors=False)
    got = orc.locality_order("bfs", n, 0, part.rowptr, part.col)
    assert len(want) == n and np.array_equal(got, want)
    # a ring whose labels were shuffled: breadth-first relabelling brings every edge within distance 2
    n = 257
    lab = rng.permutation(n)
    part = _sym_partition(n, [(int(lab[i]), int(lab[(i + 1) % n])) for i in range(n)])
    o = orc.locality_order("bfs", n, 0, part.rowptr, part.col)
    ptr2, col2, _ = orc.relabel_csr(n, part.rowptr, part.col, o)
    rows2 = np.repeat(np.arange(n), np.diff(ptr2))
    assert np.abs(rows2 - col2).max() == 2
    ptr0_rows = np.repeat(np.arange(n), np.diff(part.rowptr))
    assert np.abs(ptr0_rows - part.col).max() > 50            # the shuffled labelling had no such locality
    # two rings and an isolated vertex: every component occupies a contiguous range of the new order;
    # halo vertices: first mention decides, never-mentioned ones come last in index order
    a, b = list(range(0, 30)), list(range(30, 50))
    edges = [(a[i], a[(i + 1) % 30]) for i in range(30)] + [(b[i], b[(i + 1) % 20]) for i in range(20)]
    part = _sym_partition(51, edges, n_halo=6, halo_edges=[(35, 4), (2, 1), (50, 0), (2, 3)])
    o = orc.locality_order("bfs", 51, 6, part.rowptr, part.col)
    comp = np.array([0] * 30 + [1] * 20 + [2])[o[:51]]
    assert (np.diff(np.flatnonzero(np.diff(comp) != 0)) > 0).all() and len(np.flatnonzero(np.diff(comp) != 0)) == 2
    where = {int(v): k for k, v in enumerate(o[:51])}
    mentioned = sorted([(where[35], 4), (where[2], 1), (where[50], 0), (where[2], 3)])   # rows are sorted by column
    assert o[51:].tolist() == [51 + h for _, h in mentioned] + [51 + 2, 51 + 5]


def test_relabelled_problem_gives_the_same_epoch_with_rows_permuted(orc):
    """Moving the vertices to new places changes no result: loss and weight gradients stay, per-vertex
    outputs move with their vertex (checked on a GCN and a GraphSAGE problem, both orders)."""
    from tests import oracle_side as O
    from paper_2508_13716_amd import harness as H
    for name in ("C1", "C3"):
        cfg = synth.CONFIGS[name].scaled(0.004) if name == "C3" else synth.CONFIGS[name].scaled(0.25)
        prob = H.make_problem(cfg, mask_frac=0.6)
        ref = O.oracle_epoch(prob, halo_grad=True)
        for method in ("popularity", "bfs"):
            part = prob.part
            o = orc.locality_order(method, part.n_loc, part.n_halo, part.rowptr, part.col)
            assert not np.array_equal(o, np.arange(part.n_cols))
            got = O.oracle_epoch(O.relabelled_problem(prob, o), halo_grad=True)
            pl, ph = o[: part.n_loc], o[part.n_loc:] - part.n_loc
            assert abs(got["loss"] - ref["loss"]) <= 1e-12 * abs(ref["loss"])
            assert O.normwise(got["logits"], ref["logits"][pl]) <= 1e-12
            for l in range(len(prob.model)):
                assert O.normwise(got["hidden"][l], ref["hidden"][l][pl]) <= 1e-12
                assert O.normwise(got["dW"][l], ref["dW"][l]) <= 1e-11
                assert O.normwise(got["db"][l], ref["db"][l]) <= 1e-11
                assert O.normwise(got["dX_halo"][l], ref["dX_halo"][l][ph]) <= 1e-11


def test_cache_update_and_staleness_vs_bruteforce(orc):
    """Vertex update and the bounded-staleness list against plain Python loops, plus what must hold whatever the
    input: untouched rows keep their bytes and stamps, the last of repeated updates stays, absent ids are
    counted and ignored, and the stale list is exactly {h : epoch_now - stamp[h] > max_age} in ascending order."""
    rng = np.random.default_rng(12)
    for dtype in (np.float32, np.uint16):
        n_rows, f = 57, 5
        table = (rng.standard_normal((n_rows, f)) * 100).astype(dtype)
        stamp = np.zeros(n_rows, np.int64)
        ref_t, ref_s = table.copy(), stamp.copy()
        for epoch in range(1, 9):
            n = int(rng.integers(0, 40))
            ids = rng.integers(-3, n_rows + 3, n).astype(np.int64)         # repeats and absent ids
            rows = (rng.standard_normal((n, f)) * 100).astype(dtype)
            absent = orc.cache_update(table, stamp, ids, rows, epoch)
            miss = 0
            for r in range(n):                                            # the definition, spelled out
                if 0 <= ids[r] < n_rows:
                    ref_t[ids[r]] = rows[r]
                    ref_s[ids[r]] = epoch
                else:
                    miss += 1
            assert absent == miss
            assert table.tobytes() == ref_t.tobytes() and np.array_equal(stamp, ref_s)
            for max_age in (0, 1, 3, 100):
                got, oldest = orc.stale_ids(stamp, epoch, max_age)
                want = [h for h in range(n_rows) if epoch - ref_s[h] > max_age]
                assert got.tolist() == want and oldest == ref_s.min()
            # a gather right after the update returns the rows just written (last occurrence of each id)
            ok = (ids >= 0) & (ids < n_rows)
            out, _ = orc.gather(table, ids[ok])
            last = {int(i): r for r, i in enumerate(ids) if 0 <= i < n_rows}
            for pos, i in enumerate(ids[ok]):
                assert out[pos].tobytes() == rows[last[int(i)]].tobytes()
    got, oldest = orc.stale_ids(np.zeros(0, np.int64), 7, 0)
    assert len(got) == 0 and oldest == 7


def test_policy_hit_counts_closed_forms_and_invariants(orc):
    """The policy model against cases whose answer is known without simulating:
    - disjoint halo sets, full-batch sweeps: a cyclic sweep over more vertices than an LRU or FIFO cache holds
      never hits; with room for all of them every counted request hits locally;
    - JACA with static contents hits exactly |local set| + |global set minus local set| per sweep;
    - one vertex shared by all partitions, capacity 1 globally and 0 locally: every request after the first hits;
    - hits + misses = counted requests, capacity 0 everywhere = all misses, and hit counts never decrease
      when JACA's capacities grow."""
    A, Bs = np.arange(0, 50), np.arange(100, 130)
    for pol in ("fifo", "lru"):
        assert orc.policy_hit_counts([A, Bs], pol, 10, 0, epochs=4) == (0, 0, 3 * 80)        # cyclic sweep, cache too small
        assert orc.policy_hit_counts([A, Bs], pol, 50, 0, epochs=4) == (3 * 80, 0, 0)        # everything fits locally
        assert orc.policy_hit_counts([A, Bs], pol, 0, 80, epochs=4) == (0, 3 * 80, 0)        # ... or globally
        assert orc.policy_hit_counts([A, Bs], pol, 0, 0, epochs=3) == (0, 0, 2 * 80)
    # shared vertex 7: R = 3; everything else R = 1
    sets = [np.array([1, 2, 7]), np.array([7, 20]), np.array([7, 30, 31])]
    ids, R = orc.overlap_ratio(sets)
    assert dict(zip(ids.tolist(), R.tolist())) == {1: 1, 2: 1, 7: 3, 20: 1, 30: 1, 31: 1}
    assert orc.policy_hit_counts(sets, "jaca", 0, 1, epochs=2) == (0, 3, 5)                 # the global slot goes to vertex 7
    assert orc.policy_hit_counts(sets, "jaca_low", 0, 1, epochs=2) == (0, 1, 7)             # ... or to vertex 1 (lowest R, lowest id)
    assert orc.policy_hit_counts(sets, "jaca", 1, 1, epochs=2) == (3, 0, 5)                 # each local slot holds 7 as well
    assert orc.policy_hit_counts(sets, "jaca", 2, 0, epochs=3) == (2 * 6, 0, 2 * 2)         # {7,1} {7,20} {7,30}
    # FIFO/LRU, global capacity 1, no local cache: 7 survives only from the end of partition 0's sweep to the
    # start of partition 1's, so each epoch has exactly one hit (by hand: 7 misses + 1 hit per epoch)
    for pol in ("fifo", "lru"):
        assert orc.policy_hit_counts(sets, pol, 0, 1, epochs=2, warmup=0) == (0, 2, 14)
    rng = np.random.default_rng(14)
    sets = [np.unique(rng.integers(0, 300, 120)) for _ in range(4)]
    total = sum(len(h) for h in sets)
    prev = -1
    for cap in (0, 5, 20, 60, 150, 400):
        for pol in ("jaca", "jaca_low", "fifo", "lru"):
            hl, hg, ms = orc.policy_hit_counts(sets, pol, cap, cap, epochs=3)
            assert hl + hg + ms == 2 * total and min(hl, hg, ms) >= 0
            if cap == 0:
                assert (hl, hg) == (0, 0)
            if cap >= 400:
                assert ms == 0
        hl, hg, _ = orc.policy_hit_counts(sets, "jaca", cap, cap, epochs=3)
        assert hl + hg >= prev
        prev = hl + hg
        # high overlap first never does worse than low overlap first on the shared level
        assert hl + hg >= sum(orc.policy_hit_counts(sets, "jaca_low", cap, cap, epochs=3)[:2]) or cap >= 150


def test_placement_vs_bruteforce_and_invariants(orc):
    rng = np.random.default_rng(10)
    for n, cap in [(0, 5), (1, 0), (37, 10), (1000, 1000), (5000, 1234), (300, 400)]:
        gid = rng.permutation(10 * n + 5)[:n].astype(np.int64)
        prio = rng.integers(0, 6, n).astype(np.int64)       # many ties
        order, tier = orc.placement(gid, prio, cap)
        ref = sorted(range(n), key=lambda h: (-int(prio[h]), int(gid[h])))
        assert list(order) == ref
        k = min(cap, n)
        assert int((tier == 0).sum()) == k and int((tier == 1).sum()) == n - k
        assert set(np.nonzero(tier == 0)[0]) == set(ref[:k])
        if 0 < k < n:
            assert prio[tier == 0].min() >= prio[tier == 1].max()


def test_gather_is_a_bit_copy(orc):
    rng = np.random.default_rng(12)
    for dt in (np.float32, np.uint16):
        T = rng.integers(0, 60000, (50, 9)).astype(dt)
        if dt is np.float32:
            T = rng.standard_normal((50, 9)).astype(np.float32)
            T[3, 2] = np.float32("nan")
            T[4, 1] = -0.0
        ids = rng.integers(0, 50, 200).astype(np.int64)        # duplicates, arbitrary order
        out, absent = orc.gather(T, ids)
        assert absent == 0
        assert out.tobytes() == T[ids].tobytes()
        ids[5], ids[17] = -1, 50
        out, absent = orc.gather(T, ids)
        assert absent == 2 and not out[5].any() and not out[17].any()


def test_alg1_capacity_golden(orc):
    for line in open(os.path.join(GOLDEN, "alg1_capacity.txt")):
        if line.startswith("#") or not line.strip():
            continue
        mem, res, dims, ncand, expect = line.split()
        dims = [int(d) for d in dims.split(",")]
        from fractions import Fraction
        assert orc.cal_capacity(Fraction(mem), Fraction(res), dims, int(ncand)) == int(expect)


def test_overlap_ratio_bruteforce(orc):
    """Eq. 2: R(v) = number of partitions whose halo set holds v."""
    halos = [np.array([5, 7, 9, 9]), np.array([7, 8]), np.array([9, 7, 1]), np.array([], dtype=np.int64)]
    ids, cnt = orc.overlap_ratio(halos)
    ref = {v: sum(1 for h in halos if v in set(h.tolist())) for v in {1, 5, 7, 8, 9}}
    assert dict(zip(ids.tolist(), cnt.tolist())) == ref


def test_zipf_hit_fraction_closed_form(orc):
    """A request stream drawn Zipf(s) over N ranked halo vertices hits a top-k GPU tier with
    probability H_{k,s}/H_{N,s} (generalised harmonic numbers); N = 2 M, k = 10 %, s = 1.1 gives 0.926."""
    def harm(n, s):
        return float(np.sum(np.arange(1, n + 1, dtype=np.float64) ** -s))
    assert abs(harm(200_000, 1.1) / harm(2_000_000, 1.1) - 0.926) < 1e-3
    # measured on a sampled stream at a size the CPU handles quickly
    N, k, s = 20_000, 2_000, 1.1
    p = np.arange(1, N + 1, dtype=np.float64) ** -s
    p /= p.sum()
    rng = np.random.default_rng(14)
    gid = rng.permutation(N).astype(np.int64) + 100
    prio = (1e9 * p).astype(np.int64)                    # priority ranks follow the access law
    _, tier = orc.placement(gid, prio, k)
    req = rng.choice(N, size=400_000, p=p)
    hit = float((tier[req] == 0).mean())
    assert abs(hit - harm(k, s) / harm(N, s)) < 5e-3


# ----------------------------------------------------------------------------- RAPA: Alg. 2 / Alg. 3
def _two_gpu_example(orc, epsilon):
    devs = [orc.RapaDevice(2.0, 2.0, 1.0, 1.0, 1.0, 1e18), orc.RapaDevice(1.0, 1.0, 1.0, 1.0, 1.0, 1e18)]
    prm = orc.RapaParams(alpha=0.5, epsilon=epsilon)
    return orc.rapa_do_partition([10, 10], [20, 20], [np.array([3, 1, 2, 4]), np.array([2, 2])],
                                 [np.array([0.5, 0.1, 0.3, 0.9]), np.array([0.2, 0.4])], devs, prm)


def test_rapa_hand_trace_golden(orc):
    """The two-GPU example traced by hand in tests/golden/rapa_hand_trace.txt: costs (Eq. 3-4), the halfway rule and the
    removal order of adjust_subgraph (Alg. 3), and both stopping conditions of do_partition (Alg. 2)."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "rapa_hand_trace.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for eps, sweeps, l0, l1, sig, order0, keep1 in rows:
        res = _two_gpu_example(orc, float(eps))
        assert res["sweeps"] == int(sweeps)
        np.testing.assert_allclose(res["lam"], [float(l0), float(l1)], rtol=1e-14)
        np.testing.assert_allclose(res["sigma"], [float(x) for x in sig.split(",")], rtol=1e-14)
        assert res["removed_order"][0] == [int(x) for x in order0.split(",")]
        assert res["keep"][1].tolist() == [bool(int(x)) for x in keep1.split(",")] and res["removed_order"][1] == []
        assert res["keep"][0].sum() == 4 - len(order0.split(","))
    assert _two_gpu_example(orc, 0.1)["r"] == [1, 1] and _two_gpu_example(orc, 1.0)["r"] == [0, 1]


def test_rapa_cost_model_closed_forms(orc):
    """Eq. 3 / Eq. 4 term by term: one GPU has no peers (only the inter-device term is left, with weight 1/P = 1);
    equal GPUs have all ratios 1; alpha = 1 and alpha = 0 isolate the SpMM and the MM term; the memory constraint
    switches exactly at its bound."""
    one = [orc.RapaDevice(3.0, 5.0, 7.0, 11.0, 13.0, 1e9)]
    p = orc.RapaParams(alpha=0.25, epsilon=0.0)
    assert orc.rapa_cost(10, 100, 40, 0, one, p) == 0.25 * 100 + 0.75 * 10 + 40 * 1.0
    two = [orc.RapaDevice(1.0, 4.0, 2.0, 2.0, 6.0, 1e9), orc.RapaDevice(2.0, 2.0, 1.0, 4.0, 3.0, 1e9)]
    assert orc.rapa_cost(0, 100, 0, 0, two, orc.RapaParams(1.0, 0.0)) == 100 * 0.5          # SpMM term, ratio 1/2
    assert orc.rapa_cost(7, 100, 0, 1, two, orc.RapaParams(0.0, 0.0)) == 7 * 0.5            # MM term, ratio 2/4
    # outer edges only: GPU 0: (2/2 + 2/4) * 1/2 + 6/6 * 1/2 = 1.25 per edge
    assert orc.rapa_cost(0, 8, 8, 0, two, orc.RapaParams(0.0, 0.0)) == 8 * 1.25
    prm = orc.RapaParams(0.5, 0.0, m_vertex=8, m_edge=12, m_feat=4, f_dim=10, beta=100)
    need = 5 * 8 + 20 * 12 + 5 * 10 * 4 + 100
    assert orc.rapa_memory_ok(5, 20, orc.RapaDevice(1, 1, 1, 1, 1, need), prm)
    assert not orc.rapa_memory_ok(5, 20, orc.RapaDevice(1, 1, 1, 1, 1, need - 1), prm)


def test_rapa_invariants_on_random_instances(orc):
    """Properties the two listings fix, on random instances: what is removed from a subgraph is a prefix of its
    ascending-score order (ties by index); a subgraph that starts at or below the mean with ample memory is never
    touched in the first sweep; costs never rise; the loop ends with sigma < epsilon or r = 1; nothing can be pruned
    from subgraphs without halo vertices (r = 1 after one sweep); with too little memory for a cheap subgraph nothing
    is removed from it either (the listing only prunes while the cost exceeds the mean)."""
    rng = np.random.default_rng(17)
    for trial in range(30):
        P = int(rng.integers(2, 6))
        n_inner = rng.integers(50, 500, P).tolist()
        e_inner = rng.integers(100, 5000, P).tolist()
        halo_edges = [rng.integers(1, 30, int(rng.integers(0, 200))) for _ in range(P)]
        scores = [np.round(rng.random(len(h)), 2) for h in halo_edges]                     # rounded: ties do occur
        devs = [orc.RapaDevice(*rng.uniform(0.5, 2.0, 5).tolist(), 1e18) for _ in range(P)]
        prm = orc.RapaParams(alpha=float(rng.uniform(0.1, 0.9)), epsilon=float(rng.uniform(0.0, 50.0)))
        lam0 = [orc.rapa_cost(n_inner[i], e_inner[i] + int(halo_edges[i].sum()), int(halo_edges[i].sum()), i, devs, prm)
                for i in range(P)]
        res = orc.rapa_do_partition(n_inner, e_inner, halo_edges, scores, devs, prm)
        assert res["sigma"][-1] < prm.epsilon or all(res["r"])
        for i in range(P):
            want = sorted(range(len(halo_edges[i])), key=lambda k: (scores[i][k], k))
            assert res["removed_order"][i] == want[: len(res["removed_order"][i])]
            assert set(np.nonzero(~res["keep"][i])[0].tolist()) == set(res["removed_order"][i])
            assert res["lam"][i] <= lam0[i] * (1 + 1e-12)
    # no halo vertex anywhere: one sweep, everything marked done, nothing changes
    devs = [orc.RapaDevice(1, 1, 1, 1, 1, 1e18), orc.RapaDevice(2, 2, 1, 1, 1, 1e18)]
    res = orc.rapa_do_partition([10, 30], [50, 90], [np.zeros(0, np.int64)] * 2, [np.zeros(0)] * 2, devs, orc.RapaParams(0.5, 0.0))
    assert res["sweeps"] == 1 and res["r"] == [1, 1]
    # the cheap subgraph is short of memory: the listing's loop does not run for it (its cost is below the mean)
    devs = [orc.RapaDevice(1, 1, 1, 1, 1, 1e18), orc.RapaDevice(1, 1, 1, 1, 1, 10.0)]
    res = orc.rapa_do_partition([100, 10], [1000, 10], [np.array([5, 5]), np.array([1, 1])], [np.array([0.1, 0.2])] * 2, devs,
                                orc.RapaParams(0.5, 1e9))
    assert res["keep"][1].all() and res["sweeps"] == 1


def test_prune_halo_and_edge_counts_vs_bruteforce(orc):
    part = synth.make_partition("prune", 40, 25, 400, seed=3, max_deg=30, self_loops=False)
    e_inner, cnt = orc.halo_edge_counts(part.n_loc, part.n_halo, part.rowptr, part.col)
    assert e_inner + cnt.sum() == part.nnz and np.array_equal(cnt, part.halo_prio)
    rng = np.random.default_rng(1)
    keep = rng.random(part.n_halo) < 0.5
    rp, cl, new_index = orc.prune_halo(part.n_loc, part.n_halo, part.rowptr, part.col, keep)
    # edge set brute force: (row, old column) pairs that survive, mapped to new numbers
    kept_old = [k for k in range(part.n_halo) if keep[k]]
    assert [new_index[k] for k in kept_old] == list(range(len(kept_old))) and (new_index[~keep] == -1).all()
    want = []
    for i in range(part.n_loc):
        for e in range(part.rowptr[i], part.rowptr[i + 1]):
            c = int(part.col[e])
            if c < part.n_loc:
                want.append((i, c))
            elif keep[c - part.n_loc]:
                want.append((i, part.n_loc + kept_old.index(c - part.n_loc)))
    got = [(i, int(cl[e])) for i in range(part.n_loc) for e in range(rp[i], rp[i + 1])]
    assert got == want and rp[-1] == len(want) == part.nnz - cnt[~keep].sum()
