"""Comparisons of the HIP library's epoch with the CPU oracle that the GPU tests share.

Two complementary checks, neither of which hands the oracle anything the GPU computed:

compare_epoch            the whole epoch against the pure oracle.  Forward outputs (every hidden layer, logits, loss)
                         are compared as they are.  sigma'(Z) = 1[Z > 0] is an integer decided by a floating-point
                         value, so the implementation may decide differently where Z is zero within its own rounding;
                         the oracle computes, from its own quantities, the band in which that can happen
                         (oracle_side.relu_bands) and how far the gradients can then lie apart (oracle_side.flip_slack,
                         element by element).  Decisions must agree outside the band, and gradients must agree within
                         tol + that slack.
teacher_forced_layers    every layer's forward and backward on its own, fed with the oracle's layer input, layer output
                         (whose sign pattern is the oracle's sigma') and output gradient, rounded to the storage type.
                         No decision can differ, so there is no slack: this is the sharp check of the backward kernels,
                         and of each layer's forward pass without error carried over from the layers below.

Both assert two metrics per tensor.  Activations and input gradients (one row per vertex): norm-wise
max|gpu - ref| / max|ref|, and element-wise |gpu - ref| <= tol (|ref| + rms of the element's own row), so that the row
of a hub vertex cannot vouch for a short one.  Parameter gradients (every element a sum over all vertices): norm-wise
over the tensor and norm-wise over every row of it.  (The element-wise form is not asserted on parameter gradients: an
element there carries the rounding noise of the whole signed sum whatever its own size, in bf16 about 2^-8 of the
tensor's rms per stored operand, and the largest of 10^4..10^5 such deviations exceeds 2e-2 of the rms although
the tensor is well inside 2e-2 norm-wise - measured on the scaled C4: 6.6e-3 norm-wise, 3.3e-2 element-wise.)
"""
import numpy as np

from paper_2508_13716_amd import synth
from tests import oracle_side as O

TOL = {"f32": 1e-4, "bf16": 2e-2}
# Bar of the element-wise metric on whole-layer / whole-epoch results.  fp32: the norm-wise bar (measured errors are a
# hundred times below it either way).  bf16: an element that has passed through k values stored in bf16 carries k
# rounding errors of standard deviation 2^-8 / sqrt(3) of its scale each, and the largest of N such deviations lies
# sqrt(2 ln N) standard deviations out: with k up to 12 (three layers forward and backward) and N up to 6e8
# (C4: 2.45 M x 256) that is 6.4 * 2.26e-3 * sqrt(12) = 5e-2.  The norm-wise bar, measured against the largest element
# (about four times the rms), stays at 2e-2.
ELEM = {"f32": 1e-4, "bf16": 5e-2}


def say(msg):
    print(msg, flush=True)


def _both(gpu, ref, slack=None, by_row=False):
    """(norm-wise, second metric): element-wise by row for per-vertex tensors, worst row's norm-wise error otherwise."""
    if by_row:
        return O.normwise(gpu, ref, slack), O.elementwise(gpu, ref, slack, by_row=True)
    return O.normwise(gpu, ref, slack), O.rowwise(gpu, ref, slack)


PER_VERTEX = ("H", "logits", "dX")      # tensors with one row per vertex: their second metric is the element-wise one


def _over(errs, tol, dtype):
    """The entries of errs = {name: (norm-wise, second metric)} that exceed their bars."""
    bad = {}
    for k, (a, b) in errs.items():
        bar2 = max(ELEM[dtype], tol) if k.startswith(PER_VERTEX) else tol
        if not (a <= tol and b <= bar2):
            bad[k] = (a, b)
    return bad


def tolerance_model(prob, ref):
    """(oracle graph, oracle layers, bands, slack) of a reference epoch, computed once per reference."""
    if "_tolerance_model" not in ref:
        og = O.oracle_graph(prob.part, prob.cfg.kind, float(prob.cfg.extra.get("gin_eps", 0.0)))
        layers = O.oracle_layers(prob)
        bands = O.relu_bands(og, layers, ref, prob.cfg.dtype)
        ref["_tolerance_model"] = (og, layers, bands, O.flip_slack(og, layers, ref, bands))
    return ref["_tolerance_model"]


def compare_epoch(env, prob, dp, ref, loss, tol, tag):
    got = dp.results()
    og, layers, bands, slack = tolerance_model(prob, ref)
    errs = {}
    n_differ = 0
    for l in range(dp.L - 1):
        Hg = O.widen(dp.hidden(l))
        Z = ref["hidden"][l]
        differ, inside = O.relu_decisions_agree(Z, Hg, bands[l])
        assert inside, f"{tag}: layer {l}: ReLU decisions differ outside the rounding band"
        n_differ += differ
        errs[f"H{l}"] = _both(Hg, np.maximum(Z, 0.0), by_row=True)
    errs["logits"] = _both(got["logits"], ref["logits"], by_row=True)
    for l in range(dp.L):
        errs[f"dW{l}"] = _both(got["dW"][l], ref["dW"][l], slack["dW"][l])
        errs[f"db{l}"] = _both(got["db"][l], ref["db"][l], slack["db"][l])
        if ref["dW_self"][l] is not None:
            errs[f"dWs{l}"] = _both(got["dW_self"][l], ref["dW_self"][l], slack["dW_self"][l])
    e_loss = abs(loss - ref["loss"]) / max(1.0, abs(ref["loss"]))
    say(f"{tag}: loss={e_loss:.2e} " + " ".join(f"{k}={a:.2e}/{b:.2e}" for k, (a, b) in errs.items()) +
        f"  [norm-wise/per-row metric; ReLU decisions inside the band {slack['in_band'][:dp.L - 1]}, differing {n_differ}]")
    bad = _over(errs, tol, prob.cfg.dtype)
    assert not bad and e_loss <= tol, (tag, bad, e_loss)


def _to_storage(a, dtype: str):
    """fp64 oracle array -> the host array the device consumes (float32, or bf16 bits rounded to nearest even)."""
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    return synth.f32_to_bf16_rne(a32).reshape(a32.shape) if dtype == "bf16" else a32


def teacher_forced_layers(env, prob, dp, ref, tol, tag, need_halo=False):
    """Every layer of the model on its own through capgnn_layer_fwd / capgnn_layer_bwd, in the association the epoch
    uses, on the oracle's layer input X_l, output H_l and output gradient dH_l (rounded to the storage type).
    Compares H_l, dW_l, dW_self_l, db_l and the input gradient (local rows, = the oracle's dH_{l-1}; with need_halo
    also the halo rows) with the oracle's, both metrics, no slack."""
    torch, B, H = env["torch"], env["B"], env["H"]
    part, cfg = prob.part, prob.cfg
    dt = cfg.dtype
    per16 = 16 // dp.es
    orders = dp.resolved_orders()
    ws = None
    for l in range(dp.L - 1, -1, -1):
        p = prob.model[l]
        last = l == dp.L - 1
        out_f32 = 1 if (last and dt == "bf16") else 0
        ly = B.make_layer(B.SAGE_MEAN if p.kind == "sage" else B.GCN, p.f_in, p.f_out,
                          B.ACT_RELU if p.act == "relu" else B.ACT_NONE, dp.dtype, dp.W[l], dp.W_self[l], dp.bias[l],
                          orders[l], out_f32=out_f32)
        ldx, ldh = synth.pad_to(p.f_in, per16), synth.pad_to(p.f_out, 4 if out_f32 else per16)
        Z = ref["hidden"][l]
        Href = np.maximum(Z, 0.0) if p.act == "relu" else Z
        Hs = _to_storage(Href, "f32" if out_f32 else dt)
        if p.act == "relu":
            assert np.array_equal(O.widen(Hs) > 0.0, Z > 0.0)          # rounding keeps the oracle's decisions
        Xd = H.padded_matrix(_to_storage(ref["X"][l], dt), ldx)
        Hd_oracle = H.padded_matrix(Hs, ldh)
        dHd = H.padded_matrix(_to_storage(ref["dH"][l], "f32" if out_f32 else dt), ldh)   # the gradient has the type of H
        lddh = dHd.shape[1]
        Hd = torch.zeros_like(Hd_oracle)
        saved = torch.empty(max(B.layer_saved_bytes(dp.graph, ly), 256), dtype=torch.uint8, device="cuda")
        wsb = B.layer_workspace_bytes(dp.graph, ly)
        if ws is None or ws.numel() < wsb:
            ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
        dW = torch.zeros((p.f_in, p.f_out), dtype=torch.float32, device="cuda")
        dWs = torch.zeros_like(dW) if p.kind == "sage" else None
        db = torch.zeros(p.f_out, dtype=torch.float32, device="cuda")
        want_dx = l > 0 or need_halo
        rows = part.n_cols if need_halo else part.n_loc
        dX = torch.zeros((rows, ldx), dtype=Xd.dtype, device="cuda") if want_dx else None
        torch.cuda.synchronize()
        say(f"{tag}: teacher-forced layer {l} ({'agg' if orders[l] == B.AGG_FIRST else 'xform'} first)")
        B.layer_fwd(dp.graph, ly, Xd, ldx, Hd, ldh, saved, ws, wsb, stream=dp.stream)
        B.layer_bwd(dp.graph, ly, Xd, ldx, Hd_oracle, ldh, saved, dHd, lddh, dW, dWs, db, dX, ldx, need_halo, ws, wsb,
                    stream=dp.stream)
        torch.cuda.synchronize()
        errs = {"H": _both(O.widen(H.dev_to_np(Hd[:, :p.f_out].contiguous())), Href, by_row=True),
                "dW": _both(dW.cpu().numpy(), ref["dW"][l]), "db": _both(db.cpu().numpy(), ref["db"][l])}
        if dWs is not None:
            errs["dWs"] = _both(dWs.cpu().numpy(), ref["dW_self"][l])
        if l > 0:
            errs["dX"] = _both(O.widen(H.dev_to_np(dX[: part.n_loc, :p.f_in].contiguous())), ref["dH"][l - 1], by_row=True)
        if need_halo and ref["dX_halo"][l] is not None and part.n_halo:
            errs["dXhalo"] = _both(O.widen(H.dev_to_np(dX[part.n_loc:, :p.f_in].contiguous())), ref["dX_halo"][l], by_row=True)
        say(f"{tag}: teacher-forced layer {l}: " + " ".join(f"{k}={a:.2e}/{b:.2e}" for k, (a, b) in errs.items()))
        bad = _over(errs, tol, dt)
        assert not bad, (tag, l, bad)
        del Xd, Hd, Hd_oracle, dHd, saved, dX
