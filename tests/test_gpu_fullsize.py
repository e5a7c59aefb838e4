"""Parity at the full sizes of the named workloads, in the launch configuration bench.py times.

Every configuration C2-C5 runs one epoch on the GPU at full size and is compared with a full fp64 oracle epoch of
the same problem: every hidden layer, the logits, the loss, and every layer's weight, self-weight and bias gradient
(tests/gpu_compare.compare_epoch: norm-wise and element-wise, ReLU decisions checked against the oracle's own
rounding band).  Then every layer runs on its own from the oracle's layer input, output and output gradient
(teacher_forced_layers): that compares each weight gradient, bias gradient and input gradient - i.e. the transposed
aggregation at the hidden width, over all of its rows, and the products whose split factors only the full sizes
select - with the oracle's, without any slack.  The full-batch halo gather is compared bit for bit on every row.
"""
import time

import numpy as np
import pytest

from paper_2508_13716_amd import synth
from tests.gpu_compare import TOL, compare_epoch, say, teacher_forced_layers

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env(orc):
    import torch
    from paper_2508_13716_amd import binding as B, harness as H
    from tests import oracle_side as O
    assert torch.cuda.is_available()
    B.lib()
    return dict(torch=torch, B=B, H=H, O=O, orc=orc)


def host_memory_available_gb() -> float:
    for line in open("/proc/meminfo"):
        if line.startswith("MemAvailable:"):
            return int(line.split()[1]) / 1e6
    return 0.0


def oracle_epoch_gb(cfg, part) -> float:
    """Rough peak of the fp64 oracle epoch plus its tolerance model: per layer the input [n_cols x f_in], the
    aggregated input [n_loc x f_in] and the output [n_loc x f_out], three times over for the backward pass and the
    model's temporaries."""
    per_layer = sum(part.n_cols * cfg.dims[l] + part.n_loc * (cfg.dims[l] + 2 * cfg.dims[l + 1])
                    for l in range(len(cfg.dims) - 1))
    return 3.0 * per_layer * 8 / 1e9


@pytest.mark.parametrize("name", ["C2", "C3", "C5", "C4"])
def test_full_size_epoch_matches_oracle(env, name):
    torch, B, H, O = env["torch"], env["B"], env["H"], env["O"]
    cfg = synth.CONFIGS[name]
    tol = TOL[cfg.dtype]
    t0 = time.time()
    prob = H.make_problem(cfg, mask_frac=0.5)
    part = prob.part
    say(f"{name} full: n_loc={part.n_loc} n_halo={part.n_halo} nnz={part.nnz} dims={cfg.dims} {cfg.dtype} "
        f"(generated in {time.time() - t0:.0f} s)")
    need, have = oracle_epoch_gb(cfg, part), host_memory_available_gb()
    say(f"{name} full: the fp64 oracle epoch needs about {need:.0f} GB of host memory, {have:.0f} GB available")
    if need > 0.8 * have:
        pytest.skip(f"{name}: the fp64 oracle epoch needs about {need:.0f} GB of host memory, {have:.0f} GB available")
    dp = H.DeviceProblem(prob)
    loss, _ = dp.run_epoch()
    say(f"{name} full: GPU epoch done (orders {dp.resolved_orders()}), loss {loss:.6f}; running the oracle")
    t0 = time.time()
    ref = O.oracle_epoch(prob)
    say(f"{name} full: oracle epoch {time.time() - t0:.0f} s")
    t0 = time.time()
    compare_epoch(env, prob, dp, ref, loss, tol, f"{name} full")
    say(f"{name} full: tolerance model + comparison {time.time() - t0:.0f} s")
    teacher_forced_layers(env, prob, dp, ref, tol, f"{name} full")

    # ---- full-batch halo gather, every row, bit for bit (both tiers)
    if part.n_halo:
        for l in range(dp.L):
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


@pytest.mark.parametrize("name", ["C3", "C4", "C5"])
def test_full_size_sampled_rows(env, name):
    """Sampled output rows one by one (the longest and shortest rows and columns among them), on synthetic inputs only:
    the first layer's forward output on sampled rows (its inputs are the problem's features and cache tables; deeper
    layers' inputs are computed values, which the whole-epoch test above takes from the oracle), and the transposed
    aggregation at the hidden width on sampled columns of a random gradient.  Cheap (seconds), needs little host
    memory, and stays available where the full oracle epoch above does not fit."""
    torch, B, H, O, orc = env["torch"], env["B"], env["H"], env["O"], env["orc"]
    cfg = synth.CONFIGS[name]
    tol = TOL[cfg.dtype]
    prob = H.make_problem(cfg, mask_frac=0.5)
    part = prob.part
    dp = H.DeviceProblem(prob)
    loss, _ = dp.run_epoch()
    og = O.oracle_graph(part, cfg.kind)
    deg = np.diff(part.rowptr)
    rows = O.sample_indices(deg, 160, seed=3)
    sub, J = O.sampled_fwd_graph(og, rows)

    def input_rows(Jr):
        f_in = cfg.dims[0]
        out = np.zeros((len(Jr), f_in), np.float64)
        loc = Jr < part.n_loc
        out[loc] = O.widen(np.ascontiguousarray(prob.X0[Jr[loc], :f_in]))
        if (~loc).any():
            out[~loc] = O.widen(np.ascontiguousarray(prob.tables[0][Jr[~loc] - part.n_loc, :f_in]))
        return out

    p = prob.model[0]
    M = orc.spmm_fwd(sub, input_rows(J))
    Z = orc.matmul(M, O.widen(p.W))
    if p.kind == "sage":
        Z = Z + orc.matmul(input_rows(rows), O.widen(p.W_self))
    Z = Z + p.bias.astype(np.float64)[None, :]
    ref = np.maximum(Z, 0.0) if p.act == "relu" else Z
    g = O.widen(np.ascontiguousarray(dp.hidden(0)[rows]))
    err = (O.normwise(g, ref), O.elementwise(g, ref, by_row=True))
    say(f"{name} full: layer 0 forward on {len(rows)} sampled rows ({sub.rowptr[-1]} entries): {err[0]:.2e} / {err[1]:.2e}")
    assert max(err) <= tol, (name, err)

    rng = np.random.default_rng(5)
    cdeg = np.bincount(part.col, minlength=part.n_cols)
    cols = O.sample_indices(cdeg, 160, seed=4)
    subT, R, cols = O.sampled_bwd_graph(og, cols)
    F = 256
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
    err = (O.normwise(out, ref), O.elementwise(out, ref, by_row=True))
    say(f"{name} full: transposed aggregation F={F} on {len(cols)} sampled columns ({subT.rowptr[-1]} entries): {err[0]:.2e} / {err[1]:.2e}")
    assert max(err) <= tol
    dp.close()
