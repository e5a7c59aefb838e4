"""Parity at the full sizes of the named workloads, in the launch configuration bench.py times.

C2 (the benchmarked configuration) is compared with a full oracle epoch.  For C3-C5 a full fp64 epoch would
take minutes of CPU time, so the epoch runs on the GPU at full size and the oracle recomputes
  * every layer's forward output on sampled rows, one by one, from the GPU's own previous-layer output
    (the oracle graph restricted to those rows) - halo gather, aggregation, transform, epilogue;
  * the loss from the GPU's logits;
  * the last layer's bias gradient, and its weight gradient through bilinear forms u^T dW v that hold at
    any size (u^T dW v = <A_hat (X u), dZ v>, two sparse/dense matrix-vector products in fp64);
  * the transposed aggregation on sampled columns at the width the backward pass uses;
and the full-batch halo gather is compared bit for bit on every row.
"""
import numpy as np
import pytest

from paper_2508_13716_amd import synth

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def env(orc):
    import torch
    from paper_2508_13716_amd import binding as B, harness as H
    from tests import oracle_side as O
    assert torch.cuda.is_available()
    B.lib()
    return dict(torch=torch, B=B, H=H, O=O, orc=orc)


def say(msg):
    print(msg, flush=True)


def test_full_c2_epoch_matches_oracle(env):
    """The benchmarked configuration, whole epoch, every output."""
    from tests.test_gpu_epoch import compare_epoch
    H, O = env["H"], env["O"]
    prob = H.make_problem(synth.CONFIGS["C2"], mask_frac=0.5)
    say(f"C2 full: nnz={prob.part.nnz}")
    dp = H.DeviceProblem(prob)
    loss, _ = dp.run_epoch()
    say("C2 full: GPU epoch done, running the oracle")
    ref = O.oracle_epoch(prob)
    compare_epoch(env, prob, dp, ref, loss, TOL["f32"], "C2 full")
    dp.close()


def layer_input_rows(prob, dp, l, J, hidden_prev):
    """Rows J of layer l's input [local rows; halo rows], widened to fp64: local rows come from the GPU's
    previous-layer output (or the input features), halo rows from the layer's cache table."""
    from tests import oracle_side as O
    n_loc = prob.part.n_loc
    f_in = prob.cfg.dims[l]
    out = np.zeros((len(J), f_in), np.float64)
    loc = J < n_loc
    src = prob.X0 if l == 0 else hidden_prev
    out[loc] = O.widen(np.ascontiguousarray(src[J[loc], :f_in]))
    if (~loc).any():
        out[~loc] = O.widen(np.ascontiguousarray(prob.tables[l][J[~loc] - n_loc, :f_in]))
    return out


@pytest.mark.parametrize("name", ["C3", "C4", "C5"])
def test_full_size_sampled(env, name):
    torch, B, H, O, orc = env["torch"], env["B"], env["H"], env["O"], env["orc"]
    cfg = synth.CONFIGS[name]
    tol = TOL[cfg.dtype]
    prob = H.make_problem(cfg, mask_frac=0.5)
    part = prob.part
    say(f"{name} full: n_loc={part.n_loc} n_halo={part.n_halo} nnz={part.nnz} dims={cfg.dims} {cfg.dtype}")
    dp = H.DeviceProblem(prob)
    loss, _ = dp.run_epoch()
    got = dp.results()
    say(f"{name} full: GPU epoch done (orders {dp.resolved_orders()}), loss {loss:.6f}")
    og = O.oracle_graph(part, cfg.kind)
    L = dp.L
    deg = np.diff(part.rowptr)
    rows = O.sample_indices(deg, 160, seed=3)
    sub, J = O.sampled_fwd_graph(og, rows)

    # ---- forward, layer by layer, on the sampled rows
    hidden_prev = None
    for l in range(L):
        p = prob.model[l]
        XJ = layer_input_rows(prob, dp, l, J, hidden_prev)
        M = orc.spmm_fwd(sub, XJ)
        Z = orc.matmul(M, O.widen(p.W))
        if p.kind == "sage":
            Xs = layer_input_rows(prob, dp, l, rows, hidden_prev)
            Z = Z + orc.matmul(Xs, O.widen(p.W_self))
        Z = Z + p.bias.astype(np.float64)[None, :]
        ref = np.maximum(Z, 0.0) if p.act == "relu" else Z
        out = got["logits"] if l == L - 1 else dp.hidden(l)
        err = O.normwise(O.widen(np.ascontiguousarray(out[rows])), ref)
        say(f"{name} full: layer {l} forward on {len(rows)} sampled rows ({sub.rowptr[-1]} entries): {err:.2e}")
        assert err <= tol, (name, l, err)
        hidden_prev = out

    # ---- loss and the last layer's gradients from the GPU's logits
    ref_loss, dZ = orc.softmax_ce(got["logits"], prob.labels, prob.mask, 0.0)
    assert abs(loss - ref_loss) <= tol * max(1.0, abs(ref_loss)), (loss, ref_loss)
    err_db = O.normwise(got["db"][L - 1], dZ.sum(axis=0))
    say(f"{name} full: loss {loss:.6f} vs {ref_loss:.6f}; last-layer bias gradient {err_db:.2e}")
    assert err_db <= tol
    f_in, f_out = cfg.dims[L - 1], cfg.dims[L]
    h_prev = prob.X0 if L == 1 else dp.hidden(L - 2)

    def times_vector(a, u):          # widen(a[:, :f_in]) @ u in fp64, a chunk of rows at a time
        out = np.zeros(a.shape[0], np.float64)
        for s0 in range(0, a.shape[0], 1 << 18):
            out[s0:s0 + (1 << 18)] = O.widen(np.ascontiguousarray(a[s0:s0 + (1 << 18), :f_in])) @ u
        return out

    rng = np.random.default_rng(5)
    dW = got["dW"][L - 1].astype(np.float64)
    scale = np.abs(dW).max()
    for t in range(4):
        u, v = rng.standard_normal(f_in), rng.standard_normal(f_out)
        Xu = np.concatenate([times_vector(h_prev, u), times_vector(prob.tables[L - 1], u)]) if part.n_halo \
            else times_vector(h_prev, u)
        AXu = orc.spmm_fwd(og, Xu[:, None])[:, 0]
        ref_uv = float(AXu @ (dZ @ v))
        got_uv = float(u @ dW @ v)
        err = abs(got_uv - ref_uv) / (scale * np.abs(u).sum() * np.abs(v).sum() / np.sqrt(f_in * f_out))
        say(f"{name} full: u^T dW v (last layer) {got_uv:.6e} vs {ref_uv:.6e}  rel {err:.2e}")
        assert err <= tol, (name, got_uv, ref_uv)
        if prob.model[L - 1].kind == "sage":
            dWs = got["dW_self"][L - 1].astype(np.float64)
            ref_s = float(Xu[: part.n_loc] @ (dZ @ v))
            got_s = float(u @ dWs @ v)
            err = abs(got_s - ref_s) / (np.abs(dWs).max() * np.abs(u).sum() * np.abs(v).sum() / np.sqrt(f_in * f_out))
            assert err <= tol, (name, got_s, ref_s)

    # ---- transposed aggregation on sampled columns, at the width and dtype of the first backward product
    cdeg = np.bincount(part.col, minlength=part.n_cols)
    cols = O.sample_indices(cdeg, 160, seed=4)
    subT, R, cols = O.sampled_bwd_graph(og, cols)
    F = f_out
    ld = synth.pad_to(F, 16 // dp.es)
    dY = rng.standard_normal((part.n_loc, F)).astype(np.float32)
    dYs = synth.f32_to_bf16_rne(dY).reshape(dY.shape) if cfg.dtype == "bf16" else dY
    dYd = H.padded_matrix(dYs, ld)
    dXd = torch.zeros((part.n_cols, ld), dtype=dYd.dtype, device="cuda")
    wsb = B.spmm_workspace_bytes(dp.graph, F, dp.dtype)
    ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
    B.spmm_bwd(dp.graph, dYd, ld, dXd, ld, F, dp.dtype, ws=ws, ws_bytes=wsb)
    torch.cuda.synchronize()
    ref = orc.spmm_bwd(subT, O.widen(np.ascontiguousarray(dYs[R])))
    out = O.widen(H.dev_to_np(dXd[torch.from_numpy(cols).cuda()][:, :F].contiguous()))
    err = O.normwise(out, ref)
    say(f"{name} full: transposed aggregation F={F} on {len(cols)} sampled columns ({subT.rowptr[-1]} entries): {err:.2e}")
    assert err <= tol
    del dYd, dXd, ws

    # ---- full-batch halo gather, every row, bit for bit (both tiers)
    if part.n_halo:
        for l in range(L):
            f = cfg.dims[l]
            ldg = synth.pad_to(f, 16 // dp.es)
            outd = torch.zeros((part.n_halo, ldg), dtype=dp.tdtype, device="cuda")
            torch.cuda.synchronize()      # the fill ran on torch's stream, the gather runs on the problem's streams
            B.halo_gather(dp.cache, l, None, part.n_halo, outd, ldg, stream=dp.stream, side_stream=dp.side)
            torch.cuda.synchronize()
            same = np.array_equal(H.dev_to_np(outd[:, :f].contiguous()), prob.tables[l][:, :f])
            say(f"{name} full: halo gather layer {l} ({part.n_halo} rows x {f}): {'bit-exact' if same else 'MISMATCH'}")
            assert same
            del outd
    dp.close()
