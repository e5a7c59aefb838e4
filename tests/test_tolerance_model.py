"""Pins for the two tolerance helpers the GPU parity tests rely on (tests/oracle_side.py); no GPU needed.

sigma'(Z) = 1[Z > 0] is an integer decided by a floating-point value, so an fp32 / bf16 implementation may decide
differently from the fp64 oracle where Z is zero within its own rounding.  The parity tests therefore compare
gradients with the PURE oracle under a slack the oracle computes alone:
  * relu_bands: where may decisions differ (element-wise bound on the forward rounding error);
  * flip_slack: how far may the gradients then lie apart (the backward pass is linear in the 0/1 factors).
Here both are checked against something other than themselves: the slack against a dense numpy backward pass with
planted flips, the bands against forward passes carried out in float32 / with bf16-rounded intermediates.
"""
import numpy as np
import pytest

from paper_2508_13716_amd import harness as H, synth
from tests import oracle_side as O
from tests.test_oracle_pins import _tiny_problem, dense_adj


def dense_backward(A, n_loc, layers, ref, masks):
    """Plain numpy chain rule on the oracle's forward quantities, with the 0/1 factor of layer l given by masks[l]."""
    L = len(layers)
    out = {"dW": [None] * L, "dW_self": [None] * L, "db": [None] * L}
    dH = ref["dH"][L - 1]
    for l in range(L - 1, -1, -1):
        ly = layers[l]
        dZ = dH * masks[l] if ly.act == "relu" else dH
        out["dW"][l] = ref["M"][l].T @ dZ
        out["db"][l] = dZ.sum(axis=0)
        if ly.W_self is not None:
            out["dW_self"][l] = ref["X"][l][:n_loc].T @ dZ
        if l > 0:
            dX = A.T @ (dZ @ ly.W.T)
            if ly.W_self is not None:
                dX[:n_loc] += dZ @ ly.W_self.T
            dH = dX[:n_loc]
    return out


@pytest.mark.parametrize("kind", ["gcn", "sage"])
def test_flip_slack_is_zero_without_band_and_covers_planted_flips(orc, kind):
    g, layers, X0, tables, y, mask = _tiny_problem(orc, kind, 33)
    ref = orc.epoch(g, layers, X0, tables, y, mask)
    n_loc = g.n_loc

    class P:      # dense_adj wants a partition-like object
        pass
    p = P()
    p.n_loc, p.n_cols, p.rowptr, p.col = g.n_loc, g.n_cols, g.rowptr, g.col
    A = dense_adj(p, g.r, g.c)
    masks = [Z > 0.0 for Z in ref["hidden"]]
    base = dense_backward(A, n_loc, layers, ref, masks)
    for key in ("dW", "db", "dW_self"):
        for l in range(3):
            if ref[key][l] is not None:
                np.testing.assert_allclose(base[key][l], ref[key][l], rtol=1e-12, atol=1e-14)

    # no element inside a band: no slack at all
    zero = [np.zeros_like(Z) if layers[l].act == "relu" else None for l, Z in enumerate(ref["hidden"])]
    s0 = O.flip_slack(g, layers, ref, zero)
    assert s0["in_band"] == [0, 0, 0]
    assert all(v is None for k in ("dW", "db", "dW_self") for v in s0[k])

    rng = np.random.default_rng(2)
    for trial in range(12):
        # plant one flip in a hidden layer, or one in each
        where = [(0,), (1,), (0, 1)][trial % 3]
        bands = [b.copy() if b is not None else None for b in zero]
        flipped = [m.copy() for m in masks]
        picks = {}
        for l in where:
            cand = np.argwhere(ref["dH"][l] != 0.0)          # a vertex no masked row depends on has a zero gradient
            i, f = (int(v) for v in cand[rng.integers(0, len(cand))])
            bands[l][i, f] = abs(ref["hidden"][l][i, f])
            flipped[l][i, f] = ~flipped[l][i, f]
            picks[l] = (i, f)
        sl = O.flip_slack(g, layers, ref, bands)
        assert [sl["in_band"][l] for l in where] == [1] * len(where)
        got = dense_backward(A, n_loc, layers, ref, flipped)
        moved = 0.0
        for key in ("dW", "db", "dW_self"):
            for l in range(3):
                if ref[key][l] is None:
                    continue
                d = np.abs(got[key][l] - ref[key][l])
                moved = max(moved, d.max())
                if sl[key][l] is None:
                    assert d.max() <= 1e-13, (key, l, where)        # layers above every flip are untouched
                else:
                    assert (d <= sl[key][l] * (1 + 1e-12) + 1e-13).all(), (key, l, where)
        assert moved > 0.0
        # the bound is attained where nothing can cancel: the bias gradient of the topmost flipped layer
        lt = max(where)
        i, f = picks[lt]
        assert np.isclose(sl["db"][lt][f], abs(ref["dH"][lt][i, f]), rtol=1e-12)
        assert np.isclose(abs(got["db"][lt][f] - ref["db"][lt][f]), abs(ref["dH"][lt][i, f]), rtol=1e-9)
        others = np.delete(np.arange(len(sl["db"][lt])), f)
        assert (sl["db"][lt][others] == 0.0).all()


def _sparse(part, og, dtype):
    import scipy.sparse as sp
    rows = np.repeat(np.arange(part.n_loc), np.diff(part.rowptr))
    vals = og.r[rows] * og.c[part.col] * (1.0 if og.v is None else og.v)
    return sp.csr_matrix((vals.astype(dtype), (rows, part.col)), shape=(part.n_loc, part.n_cols))


@pytest.mark.parametrize("name,scale", [("C2", 0.01), ("C3", 0.004), ("C4", 0.001), ("C5", 0.002)])
def test_relu_bands_cover_a_rounded_forward_pass(orc, name, scale):
    """Forward passes carried out the way an implementation would - float32 sums, intermediates and layer outputs
    stored in the configuration's storage type, either association of A_hat X W - stay inside the bands, and the
    bands are not so wide that they would hide anything: a small share of the hidden elements lies inside them."""
    cfg = synth.CONFIGS[name].scaled(scale)
    prob = H.make_problem(cfg, mask_frac=0.5)
    part = prob.part
    og = O.oracle_graph(part, cfg.kind)
    layers = O.oracle_layers(prob)
    ref = O.oracle_epoch(prob)
    bands = O.relu_bands(og, layers, ref, cfg.dtype)
    A32 = _sparse(part, og, np.float32)
    n_loc = part.n_loc

    def store(a):
        a = np.asarray(a, np.float32)
        return synth.bf16_to_f32(synth.f32_to_bf16_rne(a)).reshape(a.shape) if cfg.dtype == "bf16" else a

    for order in ("agg", "xform"):
        Hprev = None
        for l, ly in enumerate(layers):
            table = O.widen(prob.tables[l]).astype(np.float32) if part.n_halo else np.zeros((0, cfg.dims[l]), np.float32)
            loc = O.widen(prob.X0).astype(np.float32) if l == 0 else Hprev
            X = np.concatenate([loc, table], axis=0)
            W = ly.W.astype(np.float32)
            if order == "agg":
                Z = store(A32 @ X) @ W
            else:
                Z = A32 @ store(X @ W)
            if ly.W_self is not None:
                Z = store(X[:n_loc] @ ly.W_self.astype(np.float32)) + Z
            Z = Z + ly.bias.astype(np.float32)[None, :]
            if ly.act != "relu":
                break
            err = np.abs(Z.astype(np.float64) - ref["hidden"][l])
            ratio = float((err / np.maximum(bands[l], 1e-300)).max())
            print(f"{cfg.name} {order} layer {l}: largest error / band = {ratio:.3f}", flush=True)
            assert ratio <= 1.0, (name, order, l, ratio)
            Hprev = store(np.maximum(Z, 0.0))
    sl = O.flip_slack(og, layers, ref, bands)
    n_hidden = sum(Z.size for Z, ly in zip(ref["hidden"], layers) if ly.act == "relu")
    share = sum(sl["in_band"]) / n_hidden
    print(f"{cfg.name}: {sum(sl['in_band'])} of {n_hidden} hidden elements inside the bands ({share:.2e})", flush=True)
    assert share <= (1e-4 if cfg.dtype == "f32" else 5e-2)
