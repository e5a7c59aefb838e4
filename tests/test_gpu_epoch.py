"""Layer and epoch parity of the HIP library against the CPU oracle (needs an MI355X)."""
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


@pytest.mark.parametrize("orders", ["auto", "agg", "xform"])
@pytest.mark.parametrize("miss_mode", [0, 1, 2])
def test_epoch_config1_matches_oracle(env, orders, miss_mode):
    B, H, O = env["B"], env["H"], env["O"]
    import copy
    cfg = copy.deepcopy(synth.CONFIGS["C1"])
    cfg.cache_frac = 0.4 if miss_mode else 1.0        # config 1 proper caches every halo row on the GPU
    prob = H.make_problem(cfg, mask_frac=0.5)
    ords = None if orders == "auto" else [B.AGG_FIRST if orders == "agg" else B.XFORM_FIRST] * 2
    dp = H.DeviceProblem(prob, orders=ords, miss_mode=miss_mode)
    ref = O.oracle_epoch(prob)
    for rep in range(3 if miss_mode == 2 else 2):       # later runs: buffers (and prefetched rows) are reused
        loss, _ = dp.run_epoch()
        compare_epoch(env, prob, dp, ref, loss, TOL["f32"], f"C1 {orders} miss_mode={miss_mode} rep={rep}")
    if miss_mode == 1:
        teacher_forced_layers(env, prob, dp, O.oracle_epoch(prob, halo_grad=True), TOL["f32"], f"C1 {orders}", need_halo=True)
    dp.close()


@pytest.mark.parametrize("cache_frac", [0.0, 1.0])
def test_epoch_pipelined_with_one_tier_empty(env, cache_frac):
    """Pipelined mode scatters the GPU tier's rows and the staged host rows of a layer in one launch; with either tier
    empty the same call must serve the other one alone."""
    H, O, B = env["H"], env["O"], env["B"]
    import copy
    cfg = copy.deepcopy(synth.CONFIGS["C1"])
    cfg.cache_frac = cache_frac
    prob = H.make_problem(cfg, mask_frac=0.5)
    assert prob.cap_gpu == (0 if cache_frac == 0.0 else prob.part.n_halo)
    dp = H.DeviceProblem(prob, miss_mode=B.MISS_PIPELINED)
    ref = O.oracle_epoch(prob)
    for rep in range(3):
        say(f"pipelined epoch, cache_frac={cache_frac} rep={rep}")
        loss, _ = dp.run_epoch()
        compare_epoch(env, prob, dp, ref, loss, TOL["f32"], f"C1 pipelined cache_frac={cache_frac} rep={rep}")
    dp.close()


@pytest.mark.parametrize("name,scale", [("C2", 0.02), ("C3", 0.01), ("C4", 0.002), ("C5", 0.004), ("C3-bf16", 0.01),
                                        ("C4-f32", 0.002)])
def test_epoch_scaled_configs_match_oracle(env, name, scale):
    """The named workloads at a fraction of their size (same average degree and widths), plus the two crossings the named
    ones leave out: the GraphSAGE model with bf16 storage and the three-layer GCN on the symmetric graph in fp32."""
    B, H, O = env["B"], env["H"], env["O"]
    cfg = synth.CONFIGS[name.split("-")[0]].scaled(scale)
    if "-" in name:
        cfg.dtype = name.split("-")[1]
        cfg.name = f"{cfg.name}-{cfg.dtype}"
    prob = H.make_problem(cfg, mask_frac=0.5)
    say(f"{cfg.name}: n_loc={prob.part.n_loc} n_halo={prob.part.n_halo} nnz={prob.part.nnz} dims={cfg.dims} {cfg.dtype}")
    dp = H.DeviceProblem(prob)
    say(f"orders={dp.resolved_orders()}")
    ref = O.oracle_epoch(prob)
    loss, times = dp.run_epoch(want_times=True)
    compare_epoch(env, prob, dp, ref, loss, TOL[cfg.dtype], cfg.name)
    assert times["total_ms"] > 0 and times["aggregation_ms"] > 0 and len(times["records"]) >= 2 * dp.L
    # without a side stream the result is the same
    dp2 = H.DeviceProblem(prob, use_side_stream=False, orders=[B.XFORM_FIRST if l % 2 else B.AGG_FIRST for l in range(dp.L)])
    loss2, _ = dp2.run_epoch()
    compare_epoch(env, prob, dp2, ref, loss2, TOL[cfg.dtype], cfg.name + " single-stream, mixed orders")
    teacher_forced_layers(env, prob, dp, ref, TOL[cfg.dtype], cfg.name)
    teacher_forced_layers(env, prob, dp2, ref, TOL[cfg.dtype], cfg.name + " mixed orders")
    dp.close()
    dp2.close()


def test_epoch_pipelined_host_tier_sees_refilled_tables(env):
    """Pipelined mode copies the host tier for the next epoch while the current one runs.  Every epoch must
    still consume exactly the tables last loaded: after capgnn_cache_fill the prefetched rows are dropped."""
    B, H, O = env["B"], env["H"], env["O"]
    cfg = synth.CONFIGS["C3"].scaled(0.01)
    prob = H.make_problem(cfg, mask_frac=0.5)
    dp = H.DeviceProblem(prob, miss_mode=B.MISS_PIPELINED)
    ref = O.oracle_epoch(prob)
    for rep in range(3):
        loss, times = dp.run_epoch(want_times=(rep == 1))
        compare_epoch(env, prob, dp, ref, loss, TOL["f32"], f"pipelined rep={rep}")
    for l in (1, 0):
        prob.tables[l] = synth.make_features(prob.part.n_halo, cfg.dims[l], seed=991, stream=70 + l, dtype=cfg.dtype)
        dp.cache.fill(l, prob.tables[l])
    ref2 = O.oracle_epoch(prob)
    assert O.normwise(ref2["logits"], ref["logits"]) > 1e-2          # the new tables do change the result
    for rep in range(2):
        loss, _ = dp.run_epoch()
        compare_epoch(env, prob, dp, ref2, loss, TOL["f32"], f"pipelined after refill rep={rep}")
    dp.close()


@pytest.mark.parametrize("miss_mode", [1, 2])
def test_epoch_after_vertex_update_and_staleness_bound(env, miss_mode):
    """Cached halo rows are overwritten between epochs (capgnn_cache_update).  The next epoch must consume
    exactly the updated tables (also when the previous epoch had already prefetched the old ones), and when
    the update moves the last layer's halo rows by at most eps the logits move by at most the staleness
    bound of Lemma 2, eta^2 beta^2 eps (and by the sharper row-wise bound its chain of inequalities gives)."""
    torch, B, H, O = env["torch"], env["B"], env["H"], env["O"]
    cfg = synth.CONFIGS["C2"].scaled(0.02)
    prob = H.make_problem(cfg, mask_frac=0.5)
    part = prob.part
    dp = H.DeviceProblem(prob, miss_mode=miss_mode)
    ref = O.oracle_epoch(prob)
    for rep in range(2):
        loss, _ = dp.run_epoch()
    compare_epoch(env, prob, dp, ref, loss, TOL["f32"], f"before update (miss_mode {miss_mode})")
    logits_before = dp.results()["logits"].astype(np.float64)
    # stale rows: the last layer's halo inputs move by at most eps
    eps, l = 1e-2, dp.L - 1
    rng = np.random.default_rng(3)
    ids = rng.permutation(part.n_halo)[: part.n_halo // 2].astype(np.int64)
    new_rows = (prob.tables[l][ids] + rng.uniform(-eps, eps, (len(ids), cfg.dims[l]))).astype(np.float32)
    moved = float(np.abs(new_rows.astype(np.float64) - prob.tables[l][ids]).max())
    rows_d = H.np_to_dev(new_rows)
    torch.cuda.synchronize()
    B.cache_update(dp.cache, l, torch.from_numpy(ids).cuda(), len(ids), rows_d, cfg.dims[l], 7, stream=dp.stream)
    prob.tables[l][ids] = new_rows
    ref2 = O.oracle_epoch(prob)
    loss2, times2 = dp.run_epoch(want_times=True)
    compare_epoch(env, prob, dp, ref2, loss2, TOL["f32"], f"after update (miss_mode {miss_mode})")
    if miss_mode == B.MISS_PIPELINED:
        # the copy prefetched before the update was patched, not dropped: per layer the only host-tier transfer of
        # this epoch is the prefetch for the next one
        moves = [r["layer"] for r in times2["records"] if r["kind"] == "gather_miss"]
        assert sorted(moves) == list(range(dp.L)), moves
        loss3, _ = dp.run_epoch()                    # consumes the copy fetched after the update
        compare_epoch(env, prob, dp, ref2, loss3, TOL["f32"], "second epoch after update (pipelined)")
    delta = float(np.abs(dp.results()["logits"].astype(np.float64) - logits_before).max())
    W = prob.model[l].W.astype(np.float64)
    eta = max(part.n_cols, W.shape[0], W.shape[1])
    beta = max(1.0, float(np.abs(ref["hidden"][l - 1]).max()), float(np.abs(prob.tables[l]).max()), float(np.abs(W).max()))
    og = O.oracle_graph(part, cfg.kind)
    halo_rowsum = np.array([og.r[i] * og.c[part.col[part.rowptr[i]:part.rowptr[i + 1]]][part.col[part.rowptr[i]:part.rowptr[i + 1]] >= part.n_loc].sum()
                            for i in range(part.n_loc)])
    sharp = halo_rowsum.max() * W.shape[0] * np.abs(W).max() * moved
    say(f"stale rows moved by {moved:.3e}: logits moved by {delta:.3e}; row-wise bound {sharp:.3e}; Lemma 2 bound {eta ** 2 * beta ** 2 * moved:.3e}")
    assert 0 < delta <= sharp * (1 + 1e-3) + 1e-5 <= eta ** 2 * beta ** 2 * moved
    dp.close()


@pytest.mark.parametrize("graph", ["small", "blocked"])
@pytest.mark.parametrize("kind", ["gcn", "sage"])
@pytest.mark.parametrize("order", ["agg", "xform"])
@pytest.mark.parametrize("product", ["auto", "split"])
def test_layer_fwd_bwd_with_halo_gradient(env, kind, order, graph, product):
    """One layer, both association orders, with and without the halo part of the input gradient.  "blocked": a
    dense-degree partition whose operator gets the column-blocked copy in both directions, so the aggregations run the
    blocked kernels, on rows that the producing kernels have multiplied by the per-source weights (GCN) or with unit
    weights (mean aggregator).  "split": every fp32 product in its three-piece form, which these sizes would not pick by
    themselves; a GraphSAGE layer's two forward products then run as one launch over both weight matrices (the first
    reduction range, 50, ends inside a step)."""
    torch, B, H, O, orc = env["torch"], env["B"], env["H"], env["O"], env["orc"]
    if graph == "small":
        part = synth.make_partition("layer", 900, 700, 12000, seed=41, max_deg=2500, self_loops=(kind == "gcn"))
    else:
        part = synth.make_partition("layer-blk", 37000, 36000, 5200000, seed=43, max_deg=4000, halo_edge_frac=0.5,
                                    self_loops=(kind == "gcn"))
    fi, fo = 50, 36
    rng = np.random.default_rng(7)
    X = rng.standard_normal((part.n_cols, fi)).astype(np.float32)
    W = (rng.standard_normal((fi, fo)) * 0.2).astype(np.float32)
    Ws = (rng.standard_normal((fi, fo)) * 0.2).astype(np.float32) if kind == "sage" else None
    b = rng.standard_normal(fo).astype(np.float32)
    dH = rng.standard_normal((part.n_loc, fo)).astype(np.float32)
    og = O.oracle_graph(part, kind)
    ol = orc.Layer(kind, W.astype(np.float64), b.astype(np.float64), "relu", None if Ws is None else Ws.astype(np.float64))
    Href, saved = orc.layer_fwd(og, ol, X.astype(np.float64))
    bref = orc.layer_bwd(og, ol, X.astype(np.float64), saved, dH.astype(np.float64), need_dx=True)

    r, c = B.norm_scales(B.NORM_SYM if kind == "gcn" else B.NORM_MEAN, part.n_loc, part.n_halo, part.rowptr, part.halo_degree)
    g = B.Graph(part.n_loc, part.n_halo, part.rowptr, part.col, r, c)
    Wd, Wsd, bd = H.np_to_dev(W), (None if Ws is None else H.np_to_dev(Ws)), H.np_to_dev(b)
    ly = B.make_layer(B.GCN if kind == "gcn" else B.SAGE_MEAN, fi, fo, B.ACT_RELU, B.F32, Wd, Wsd, bd,
                      B.AGG_FIRST if order == "agg" else B.XFORM_FIRST,
                      f32_product=B.F32_PRODUCT_SPLIT if product == "split" else B.F32_PRODUCT_AUTO)
    ldx, ldh = 52, 36
    Xd = H.padded_matrix(X, ldx)
    Hd = torch.zeros((part.n_loc, ldh), device="cuda")
    saved_d = torch.empty(max(B.layer_saved_bytes(g, ly), 256), dtype=torch.uint8, device="cuda")
    wsb = B.layer_workspace_bytes(g, ly)
    ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
    B.layer_fwd(g, ly, Xd, ldx, Hd, ldh, saved_d, ws, wsb)
    torch.cuda.synchronize()
    Hgot = Hd.cpu().numpy()
    assert O.normwise(Hgot, Href) <= TOL["f32"] and O.elementwise(Hgot, Href, by_row=True) <= TOL["f32"]
    # backward from the oracle's own forward output: its sign pattern is the oracle's sigma', so no decision can differ
    Hd = H.padded_matrix(Href.astype(np.float32), ldh)
    assert np.array_equal(Href.astype(np.float32) > 0, saved["Z"] > 0)
    for need_halo in (True, False):
        dHd = H.np_to_dev(dH)
        dW, dWs, db = torch.zeros_like(Wd), (None if Ws is None else torch.zeros_like(Wd)), torch.zeros_like(bd)
        rows = part.n_cols if need_halo else part.n_loc
        dX = torch.full((rows, ldx), 5.0, device="cuda")
        B.layer_bwd(g, ly, Xd, ldx, Hd, ldh, saved_d, dHd, fo, dW, dWs, db, dX, ldx, need_halo, ws, wsb)
        torch.cuda.synchronize()
        say(f"layer {kind} {order} need_halo={need_halo}")
        for name, a, want in (("dW", dW, bref["dW"]), ("db", db, bref["db"])) + ((("dWs", dWs, bref["dW_self"]),) if Ws is not None else ()):
            assert O.normwise(a.cpu().numpy(), want) <= TOL["f32"] and O.rowwise(a.cpu().numpy(), want) <= TOL["f32"], name
        got = dX.cpu().numpy()
        assert O.normwise(got[:, :fi], bref["dX"][:rows]) <= TOL["f32"]
        assert O.elementwise(got[:, :fi], bref["dX"][:rows], by_row=True) <= TOL["f32"]
        assert (got[:, fi:] == 5.0).all()
    g.close()


def test_epoch_sgd_step_and_no_halo(env):
    """Partition without halo vertices (cache is NULL) and the in-place W <- W - lr dW update."""
    torch, B, H, O = env["torch"], env["B"], env["H"], env["O"]
    cfg = synth.Config("nohalo", "gcn", 3000, 0, 30000, [40, 32, 5], "f32", 0.0, max_deg=400, symmetric=True, seed=77)
    prob = H.make_problem(cfg, mask_frac=0.7)
    dp = H.DeviceProblem(prob)
    ref = O.oracle_epoch(prob, lr=0.05)
    loss, _ = dp.run_epoch(lr=0.05)
    compare_epoch(env, prob, dp, ref, loss, TOL["f32"], "no-halo symmetric")
    torch.cuda.synchronize()
    for l in range(dp.L):
        assert O.normwise(H.dev_to_np(dp.W[l]), ref["new_W"][l]) <= TOL["f32"]
        assert O.normwise(H.dev_to_np(dp.bias[l]), ref["new_bias"][l]) <= TOL["f32"]
    dp.close()


def test_epoch_rejects_bad_arguments(env):
    torch, B, H = env["torch"], env["B"], env["H"]
    import copy
    cfg = copy.deepcopy(synth.CONFIGS["C1"]).scaled(0.1)
    prob = H.make_problem(cfg)
    dp = H.DeviceProblem(prob)
    with pytest.raises(B.CapgnnError) as e:       # workspace too small
        B.epoch(dp.graph, dp.cache, dp.layers, dp.X0, dp.ld0, dp.labels, dp.mask, 0.0, dp.logits, dp.dW, None,
                dp.dbias, 0.0, dp.ws, 1024, dp.stream, dp.side)
    assert e.value.code == B.ENOMEM
    with pytest.raises(B.CapgnnError) as e:       # halo vertices but no cache
        B.epoch(dp.graph, None, dp.layers, dp.X0, dp.ld0, dp.labels, dp.mask, 0.0, dp.logits, dp.dW, None,
                dp.dbias, 0.0, dp.ws, dp.ws_bytes, dp.stream, dp.side)
    assert e.value.code == B.EINVAL
    dp.close()


@pytest.mark.parametrize("case", ["C1", "C2-host-tier", "C1-sgd"])
def test_epoch_graph_replays_match_eager_epochs(env, case):
    """capgnn_epoch recorded as a HIP graph: every replay must give exactly what the eager epoch gives on the same buffer
    contents (same kernels, same order: bit for bit), also after the buffers' contents changed between replays (a cache
    update), with eager work and synchronisations between the replays, and with host-tier rows travelling inside the
    graph.  The first eager result is compared with the oracle."""
    torch, B, H, O = env["torch"], env["B"], env["H"], env["O"]
    if case == "C2-host-tier":
        cfg = synth.CONFIGS["C2"].scaled(0.02)
        prob = H.make_problem(cfg, mask_frac=0.5)
    else:
        cfg = synth.CONFIGS["C1"]
        prob = H.make_problem(cfg, mask_frac=0.5)
    lr = 0.05 if case == "C1-sgd" else 0.0
    part = prob.part
    # the eager side runs on one stream too (no side stream), as the recorded epoch does
    dp = H.DeviceProblem(prob, miss_mode=B.MISS_STAGED, use_side_stream=False)
    ref = O.oracle_epoch(prob)

    def snapshot():
        r = dp.results()
        return [r["logits"].copy()] + [a.copy() for a in r["dW"]] + [a.copy() for a in r["db"]]

    W0 = [w.clone() for w in dp.W]
    b0 = [b.clone() for b in dp.bias]

    def reset_weights():
        for w, w0 in zip(dp.W, W0):
            w.copy_(w0)
        for b, bb in zip(dp.bias, b0):
            b.copy_(bb)
        torch.cuda.synchronize()

    # eager: three epochs (with the SGD step they differ), a cache update before the third
    rng = np.random.default_rng(11)
    l_upd = dp.L - 1
    ids = rng.permutation(part.n_halo)[: max(part.n_halo // 3, 1)].astype(np.int64)
    new_rows = rng.standard_normal((len(ids), cfg.dims[l_upd])).astype(np.float32)
    ids_d, rows_d = torch.from_numpy(ids).cuda(), H.np_to_dev(new_rows)
    old_rows_d = H.np_to_dev(np.ascontiguousarray(prob.tables[l_upd][ids]))
    eager = []
    for it in range(3):
        if it == 2:
            B.cache_update(dp.cache, l_upd, ids_d, len(ids), rows_d, cfg.dims[l_upd], 5, stream=dp.stream)
        loss, _ = dp.run_epoch(lr=lr)
        eager.append((loss, snapshot()))
        if it == 0:
            compare_epoch(env, prob, dp, ref, loss, TOL["f32"], f"graph case {case}: eager epoch")
    # back to the start: weights, cache rows
    B.cache_update(dp.cache, l_upd, ids_d, len(ids), old_rows_d, cfg.dims[l_upd], 6, stream=dp.stream)
    reset_weights()
    for t in [dp.logits] + dp.dW + dp.dbias:
        t.zero_()
    torch.cuda.synchronize()

    eg, loss_dev = dp.capture_epoch(lr=lr)
    assert np.isnan(loss_dev.cpu().numpy()[0]) and not dp.logits.any()        # recording ran nothing
    scratch = torch.empty(1 << 20, device="cuda")
    for it in range(3):
        if it == 2:
            B.cache_update(dp.cache, l_upd, ids_d, len(ids), rows_d, cfg.dims[l_upd], 7, stream=dp.stream)
        eg.launch(dp.stream)
        torch.cuda.synchronize()
        got = snapshot()
        loss_g = float(loss_dev.cpu().numpy()[0])
        scratch.normal_()                        # the program's own eager work between the replays
        _ = float(scratch.sum().cpu())
        say(f"graph case {case}: replay {it}: loss {loss_g:.6f} (eager {eager[it][0]:.6f})")
        assert loss_g == eager[it][0], (it, loss_g, eager[it][0])
        for a, b in zip(got, eager[it][1]):
            assert np.array_equal(a, b), f"replay {it} differs from the eager epoch"
    if lr == 0.0:
        assert not np.array_equal(eager[2][1][0], eager[1][1][0])      # the update did change the result
    else:
        assert not np.array_equal(eager[1][1][0], eager[0][1][0])      # and so did the SGD step
    eg.close()
    with pytest.raises(B.CapgnnError):
        B.EpochGraph(dp.graph, dp.cache, dp.layers, dp.X0, dp.ld0, dp.labels, dp.mask, 0.0, dp.logits, dp.dW, None, dp.dbias,
                     0.0, None, dp.ws, dp.ws_bytes, None)             # the default stream cannot be captured
    # the stream is usable after the failed call, and after a successful capture
    loss, _ = dp.run_epoch(lr=0.0)
    assert np.isfinite(loss)
    dp.close()


@pytest.mark.parametrize("kind", ["gcn", "sage"])
def test_training_run_tracks_the_oracle(env, kind):
    """Twelve epochs with the in-place step W <- W - lr * dW (the update of the convergence theorem's proof): the loss of
    every epoch and the weights at the end must follow the oracle's own fp64 training run, which carries its weights in
    fp64 from step to step and takes nothing from the GPU.  The loss must also go down in the oracle's run: a sign error
    in the step would show there first."""
    torch, B, H, O, orc = env["torch"], env["B"], env["H"], env["O"], env["orc"]
    cfg = synth.Config(f"train-{kind}", kind, 2500, 1800, 40000, [48, 32, 7], "f32", 0.5, max_deg=600, seed=91)
    prob = H.make_problem(cfg, mask_frac=0.6)
    dp = H.DeviceProblem(prob, miss_mode=B.MISS_PIPELINED)
    lr, steps = 0.2, 12
    og = O.oracle_graph(prob.part, kind)
    layers = O.oracle_layers(prob)
    tables = [O.widen(t) for t in prob.tables]
    X0 = O.widen(prob.X0)
    ref_losses, gpu_losses = [], []
    for it in range(steps):
        ref = orc.epoch(og, layers, X0, tables, prob.labels, prob.mask, 0.0, lr)
        ref_losses.append(ref["loss"])
        for l, ly in enumerate(layers):
            ly.W = ref["new_W"][l]
            ly.bias = ref["new_bias"][l]
            if ly.W_self is not None:
                ly.W_self = ref["new_W_self"][l]
        loss, _ = dp.run_epoch(lr=lr)
        gpu_losses.append(loss)
    say(f"training {kind}: oracle loss {ref_losses[0]:.5f} -> {ref_losses[-1]:.5f}, GPU {gpu_losses[0]:.5f} -> {gpu_losses[-1]:.5f}")
    assert all(b < a for a, b in zip(ref_losses, ref_losses[1:])), ref_losses
    for a, b in zip(gpu_losses, ref_losses):
        assert abs(a - b) <= 1e-4 * max(1.0, abs(b)), (gpu_losses, ref_losses)
    torch.cuda.synchronize()
    for l, ly in enumerate(layers):
        assert O.normwise(H.dev_to_np(dp.W[l]), ly.W) <= 1e-3, l
        assert O.normwise(H.dev_to_np(dp.bias[l]), ly.bias) <= 1e-3, l
        if ly.W_self is not None:
            assert O.normwise(H.dev_to_np(dp.W_self[l]), ly.W_self) <= 1e-3, l
    dp.close()


@pytest.mark.parametrize("miss_mode", [1, 2])
def test_epoch_graph_with_side_stream_matches_eager_epochs(env, miss_mode):
    """The two-stream epoch recorded as a HIP graph (host-tier rows on the side stream; in pipelined mode every replay
    consumes what the run before it prefetched and prefetches for the next).  Replays must equal eager epochs bit for bit:
    on the static tables, after a cache update between replays (which patches the prefetched copy), and after a refill
    followed by one eager epoch that primes the prefetch again; recording a pipelined epoch that nothing has primed is an
    argument error, and eager epochs after the replays still see the right rows."""
    torch, B, H, O = env["torch"], env["B"], env["H"], env["O"]
    cfg = synth.CONFIGS["C2"].scaled(0.02)
    prob = H.make_problem(cfg, mask_frac=0.5)
    part = prob.part
    dp = H.DeviceProblem(prob, miss_mode=miss_mode)
    ref = O.oracle_epoch(prob)

    def snapshot():
        r = dp.results()
        return [r["logits"].copy()] + [a.copy() for a in r["dW"]] + [a.copy() for a in r["db"]]

    if miss_mode == B.MISS_PIPELINED:
        with pytest.raises(B.CapgnnError):
            dp.capture_epoch(two_streams=True)                   # nothing has prefetched the host tier yet
    loss0, _ = dp.run_epoch()
    compare_epoch(env, prob, dp, ref, loss0, TOL["f32"], f"two-stream graph (miss_mode {miss_mode}): eager epoch")
    base = snapshot()
    eg, loss_dev = dp.capture_epoch(two_streams=True)
    scratch = torch.empty(1 << 20, device="cuda")
    for it in range(3):
        eg.launch(dp.stream)
        torch.cuda.synchronize()
        scratch.normal_()
        _ = float(scratch.sum().cpu())
        assert float(loss_dev.cpu()[0]) == loss0
        for a, b in zip(snapshot(), base):
            assert np.array_equal(a, b), f"replay {it} differs from the eager epoch"
    # rows rewritten between replays, in both tiers
    rng = np.random.default_rng(17)
    l_upd = dp.L - 1
    ids = rng.permutation(part.n_halo)[: part.n_halo // 2].astype(np.int64)
    new_rows = rng.standard_normal((len(ids), cfg.dims[l_upd])).astype(np.float32)
    B.cache_update(dp.cache, l_upd, torch.from_numpy(ids).cuda(), len(ids), H.np_to_dev(new_rows), cfg.dims[l_upd], 3,
                   stream=dp.stream)
    prob.tables[l_upd][ids] = new_rows
    ref2 = O.oracle_epoch(prob)
    for it in range(2):
        eg.launch(dp.stream)
        torch.cuda.synchronize()
        compare_epoch(env, prob, dp, ref2, float(loss_dev.cpu()[0]), TOL["f32"], f"two-stream graph after update, replay {it}")
    upd = snapshot()
    loss_e, _ = dp.run_epoch()                                   # an eager epoch after the replays: same rows, same result
    for a, b in zip(snapshot(), upd):
        assert np.array_equal(a, b)
    # a refill drops the prefetched copy: one eager epoch primes it again, then the replays see the new table
    prob.tables[0] = synth.make_features(part.n_halo, cfg.dims[0], seed=5, stream=3, dtype=cfg.dtype)
    dp.cache.fill(0, prob.tables[0])
    ref3 = O.oracle_epoch(prob)
    loss3, _ = dp.run_epoch()
    compare_epoch(env, prob, dp, ref3, loss3, TOL["f32"], "two-stream graph: eager epoch after refill")
    want = snapshot()
    for it in range(2):
        eg.launch(dp.stream)
        torch.cuda.synchronize()
        for a, b in zip(snapshot(), want):
            assert np.array_equal(a, b), f"replay {it} after refill differs"
    eg.close()
    dp.close()
