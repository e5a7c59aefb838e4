"""Per-kernel parity of the HIP library against the CPU oracle (needs an MI355X).

fp32 results must agree within 1e-4, bf16 within 2e-2, in the norm-wise metric
max|gpu - ref| / max|ref| and, for the aggregations, also element by element:
|gpu - ref| <= tol (|ref| + rms of the element's own row), so that the rows of hub vertices cannot vouch
for short rows; cache lookup and gather must agree bit for bit.
"""
import numpy as np
import pytest

from paper_2508_13716_amd import synth

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4
TOL_BF16 = 2e-2


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


def adversarial_graphs():
    rng = np.random.default_rng(17)
    gs = [synth.hand_partition(9, 6, [(int(rng.integers(0, 9)), int(rng.integers(0, 15))) for _ in range(40)] +
                               [(0, 1), (0, 1)], name="dups+empty"),
          synth.hand_partition(6, 5000, [(0, j) for j in range(6, 5006)] + [(2, 9), (5, 5)], name="one-5000-row"),
          synth.hand_partition(4, 3, [], name="no-edges"),
          synth.hand_partition(1, 0, [(0, 0)], name="single"),
          synth.make_partition("cl-small", 700, 500, 9000, seed=5, max_deg=300),
          synth.make_partition("cl-long", 300, 9000, 40000, seed=6, max_deg=9000, halo_edge_frac=0.9)]
    return gs


def run_spmm(env, part, F, ld, dtype, with_vals, seed, blocked=False, unit_weights=False):
    torch, B, H, O, orc = env["torch"], env["B"], env["H"], env["O"], env["orc"]
    rng = np.random.default_rng(seed)
    r = rng.uniform(0.5, 1.5, part.n_loc).astype(np.float32)
    c = rng.uniform(0.5, 1.5, part.n_cols).astype(np.float32)
    if unit_weights:       # every entry weighs 1 in both directions: the kernels read bare source rows
        r, c = np.ones_like(r), np.ones_like(c)
    v = rng.uniform(-1, 1, part.nnz).astype(np.float32) if with_vals else None
    X = rng.standard_normal((part.n_cols, F)).astype(np.float32)
    dY = rng.standard_normal((part.n_loc, F)).astype(np.float32)
    if dtype == "bf16":
        Xs, dYs = synth.f32_to_bf16_rne(X).reshape(X.shape), synth.f32_to_bf16_rne(dY).reshape(dY.shape)
    else:
        Xs, dYs = X, dY
    g = B.Graph(part.n_loc, part.n_halo, part.rowptr, part.col, r, c, v)
    dt = B.BF16 if dtype == "bf16" else B.F32
    Xd, dYd = H.padded_matrix(Xs, ld), H.padded_matrix(dYs, ld)
    # sentinel-filled outputs: whatever the kernel must not touch stays recognisable
    Yd = torch.full((part.n_loc, ld), 7.0, dtype=Xd.dtype, device="cuda")
    dXd = torch.full((part.n_cols, ld), 7.0, dtype=Xd.dtype, device="cuda")
    ws, wsb = None, 0
    if blocked:       # with scratch the column-blocked kernel runs, or very long rows are cut into pieces
        wsb = B.spmm_workspace_bytes(g, F, dt)
        assert wsb > 0, "graph or width qualifies neither for the column-blocked kernel nor for cut rows"
        ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    B.spmm_fwd(g, Xd, ld, Yd, ld, F, dt, ws=ws, ws_bytes=wsb)
    B.spmm_bwd(g, dYd, ld, dXd, ld, F, dt, ws=ws, ws_bytes=wsb)
    torch.cuda.synchronize()
    og = orc.Graph(part.n_loc, part.n_cols, part.rowptr, part.col, r.astype(np.float64), c.astype(np.float64),
                   None if v is None else v.astype(np.float64))
    Yref = orc.spmm_fwd(og, O.widen(Xs))
    dXref = orc.spmm_bwd(og, O.widen(dYs))
    Y, dX = O.widen(H.dev_to_np(Yd)), O.widen(H.dev_to_np(dXd))
    tol = TOL_BF16 if dtype == "bf16" else TOL_F32
    errs = (O.normwise(Y[:, :F], Yref), O.elementwise(Y[:, :F], Yref, by_row=True),
            O.normwise(dX[:, :F], dXref), O.elementwise(dX[:, :F], dXref, by_row=True))
    say(f"   fwd {errs[0]:.2e} norm-wise, {errs[1]:.2e} element-wise by row; transposed {errs[2]:.2e}, {errs[3]:.2e}")
    assert max(errs) <= tol, (part.name, F, ld, dtype, errs)
    assert (Y[:, F:] == 7.0).all() and (dX[:, F:] == 7.0).all(), "padding columns were written"
    g.close()


@pytest.mark.parametrize("gi", range(6))
def test_spmm_adversarial_graphs_f32(env, gi):
    part = adversarial_graphs()[gi]
    for F, ld in [(1, 1), (7, 7), (8, 8), (41, 44), (64, 64), (100, 100), (130, 132)]:
        say(f"spmm f32 {part.name} F={F} ld={ld}")
        run_spmm(env, part, F, ld, "f32", with_vals=(F % 2 == 1), seed=gi * 100 + F)


@pytest.mark.parametrize("F,ld", [(602, 602), (602, 608), (256, 256), (800, 800), (1000, 1001)])
def test_spmm_wide_rows_f32(env, F, ld):
    part = synth.make_partition("cl-wide", 500, 400, 8000, seed=8, max_deg=2500)
    say(f"spmm f32 wide F={F} ld={ld}")
    run_spmm(env, part, F, ld, "f32", with_vals=False, seed=F)


@pytest.mark.parametrize("F,ld", [(3, 3), (16, 16), (47, 48), (128, 128), (512, 512), (600, 600), (1500, 1504)])
def test_spmm_bf16(env, F, ld):
    for part in adversarial_graphs()[:2] + adversarial_graphs()[4:]:
        say(f"spmm bf16 {part.name} F={F} ld={ld}")
        run_spmm(env, part, F, ld, "bf16", with_vals=False, seed=F)


@pytest.mark.parametrize("shape", ["wide", "tall"])
def test_spmm_column_blocked(env, shape):
    """Dense-degree operators get a column-blocked copy (several source blocks, long (block,row) groups);
    with scratch the blocked kernel + its fixed-order reduction run.  'wide' blocks the forward product,
    'tall' the transposed one; ragged last block, empty groups, partial last slice, edge values."""
    if shape == "wide":
        part = synth.make_partition("blk-wide", 2500, 38000, 330000, seed=21, max_deg=9000, halo_edge_frac=0.9)
    else:
        part = synth.make_partition("blk-tall", 37000, 2000, 2600000, seed=22, max_deg=4000, halo_edge_frac=0.2)
    for F, ld, dtype, vals in [(32, 32, "f32", False), (41, 44, "f32", True), (256, 256, "f32", False),
                               (602, 604, "f32", False), (64, 64, "bf16", False), (200, 200, "bf16", True),
                               (256, 264, "bf16", False)]:
        say(f"spmm blocked {part.name} F={F} ld={ld} {dtype}")
        run_spmm(env, part, F, ld, dtype, vals, seed=F, blocked=True)


@pytest.mark.parametrize("shape", ["wide", "tall"])
def test_spmm_column_blocked_unit_weights(env, shape):
    """The same operators with every weight equal to 1 (no edge values, scales of 1): the blocked kernel then reads
    its entries as 2-byte row numbers inside the source block, exchanges no weights between lanes and adds instead of
    multiplying.  Widths span one partial slice, several slices and a ragged last slice, both storage types."""
    if shape == "wide":
        part = synth.make_partition("blk-wide-1", 2500, 38000, 330000, seed=31, max_deg=9000, halo_edge_frac=0.9)
    else:
        part = synth.make_partition("blk-tall-1", 37000, 2000, 2600000, seed=32, max_deg=4000, halo_edge_frac=0.2)
    for F, ld, dtype in [(32, 32, "f32"), (41, 44, "f32"), (256, 256, "f32"), (602, 604, "f32"), (64, 64, "bf16"),
                         (200, 200, "bf16")]:
        say(f"spmm blocked, unit weights {part.name} F={F} ld={ld} {dtype}")
        run_spmm(env, part, F, ld, dtype, False, seed=F, blocked=True, unit_weights=True)


def test_spmm_rows_cut_into_pieces(env):
    """Rows and columns far longer than one workgroup's share: with scratch they are cut into pieces whose
    partial sums are combined in a fixed order.  One row of 40000 entries, one exactly at the cutting
    threshold plus one, two halo columns referenced by 33000 rows (ragged last piece), the rest short."""
    rng = np.random.default_rng(5)
    n_loc, n_halo = 45000, 50
    n_cols = n_loc + n_halo
    rows = [rng.integers(0, n_cols, 40000), rng.integers(0, n_cols, 16385)]
    for i in range(2, n_loc):
        extra = [n_loc, n_loc + 1] if i < 33002 else []
        rows.append(np.array(list(rng.integers(0, n_cols, 3)) + extra))
    rowptr = np.zeros(n_loc + 1, np.int64)
    np.cumsum([len(r) for r in rows], out=rowptr[1:])
    col = np.concatenate(rows).astype(np.int32)
    part = synth.Partition("cut", n_loc, n_halo, rowptr, col, np.arange(n_halo, dtype=np.int64),
                           np.ones(n_halo, np.int64), np.ones(n_halo, np.int64), False, False)
    for F, ld, dtype, vals in [(32, 32, "f32", False), (41, 44, "f32", True), (256, 256, "bf16", False),
                               (100, 104, "bf16", True), (7, 7, "f32", False)]:
        say(f"spmm cut rows F={F} ld={ld} {dtype}")
        run_spmm(env, part, F, ld, dtype, vals, seed=F, blocked=True)


def test_spmm_exact_on_small_integers(env):
    """Integer features, unit scales: every partial sum is exactly representable, so fp32 and bf16
    results must equal the oracle exactly."""
    torch, B, H, O, orc = env["torch"], env["B"], env["H"], env["O"], env["orc"]
    part = synth.make_partition("ints", 400, 300, 3000, seed=9, max_deg=100)
    rng = np.random.default_rng(1)
    X = rng.integers(-2, 3, (part.n_cols, 24)).astype(np.float32)
    g = B.Graph(part.n_loc, part.n_halo, part.rowptr, part.col)
    og = orc.Graph(part.n_loc, part.n_cols, part.rowptr, part.col, np.ones(part.n_loc), np.ones(part.n_cols))
    ref = orc.spmm_fwd(og, X.astype(np.float64))
    assert np.abs(ref).max() <= 256
    for dt, Xs in ((B.F32, X), (B.BF16, synth.f32_to_bf16_rne(X).reshape(X.shape))):
        Xd = H.np_to_dev(Xs)
        Yd = torch.zeros((part.n_loc, 24), dtype=Xd.dtype, device="cuda")
        B.spmm_fwd(g, Xd, 24, Yd, 24, 24, dt)
        torch.cuda.synchronize()
        assert np.array_equal(O.widen(H.dev_to_np(Yd)), ref)
    g.close()


def test_spmm_on_config1_graph(env):
    cfg = synth.CONFIGS["C1"]
    part = synth.partition_for(cfg)
    say("spmm C1")
    run_spmm(env, part, 128, 128, "f32", False, 1)
    run_spmm(env, part, 64, 64, "f32", False, 2)


def test_graph_create_rejects_malformed_input(env):
    B = env["B"]
    with pytest.raises(B.CapgnnError):
        B.Graph(2, 0, np.array([0, 1, 3]), np.array([0, 5, 1], np.int32))       # column out of range
    with pytest.raises(B.CapgnnError):
        B.Graph(2, 0, np.array([0, 2, 1]), np.array([0, 1], np.int32))          # rowptr decreases
    with pytest.raises(B.CapgnnError):
        B.Graph(2, 0, np.array([1, 2, 3]), np.array([0, 1, 1], np.int32))       # rowptr[0] != 0
    with pytest.raises(B.CapgnnError):                                          # claims symmetry, is not
        B.Graph(2, 0, np.array([0, 1, 1]), np.array([1], np.int32), flags=B.GRAPH_SYMMETRIC)


# ----------------------------------------------------------------------------- cache
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("cap_frac", [0.0, 0.37, 1.0])
def test_cache_placement_lookup_gather_bit_exact(env, dtype, cap_frac):
    torch, B, H, O, orc = env["torch"], env["B"], env["H"], env["O"], env["orc"]
    part = synth.make_partition("cache", 300, 5000, 30000, seed=21, max_deg=200)
    n = part.n_halo
    cap = int(cap_frac * n)
    dims = [602, 47, 8]
    dt = B.BF16 if dtype == "bf16" else B.F32
    tables = [synth.make_features(n, d, seed=3, stream=30 + i, dtype=dtype) for i, d in enumerate(dims)]
    say(f"cache dtype={dtype} cap={cap}/{n}")
    c = B.Cache(part.halo_gid, part.halo_prio, cap, dims, dt, B.MAP_HASH)
    for l in range(3):
        c.fill(l, tables[l])
    # placement: tier membership equals the oracle's
    _, tier_ref = orc.placement(part.halo_gid, part.halo_prio, cap)
    tier, slot = c.query(np.arange(n))
    assert np.array_equal(tier, tier_ref)
    assert sorted(slot[tier == 0]) == list(range(cap)) and sorted(slot[tier == 1]) == list(range(n - cap))
    tier_g, slot_g = c.query(part.halo_gid, by_gid=True)
    assert np.array_equal(tier_g, tier) and np.array_equal(slot_g, slot)
    # device lookup, including absent keys
    rng = np.random.default_rng(4)
    absent = rng.integers(1 << 41, 1 << 42, 1000).astype(np.int64)
    ids = np.concatenate([part.halo_gid[rng.integers(0, n, 3000)], absent])
    ids_d = torch.from_numpy(ids).cuda()
    t_d = torch.empty(len(ids), dtype=torch.int8, device="cuda")
    s_d = torch.empty(len(ids), dtype=torch.int64, device="cuda")
    c.lookup(ids_d, t_d, s_d, by_gid=True)
    torch.cuda.synchronize()
    t_h, s_h = c.query(ids, by_gid=True, check=False)
    assert np.array_equal(t_d.cpu().numpy(), t_h) and np.array_equal(s_d.cpu().numpy(), s_h)
    assert (t_h[-1000:] == -1).all() and (t_h[:3000] >= 0).all()

    side = torch.cuda.Stream()
    main = torch.cuda.Stream()
    stg = torch.empty(max(c.staging_bytes, 256), dtype=torch.uint8, device="cuda")
    for l, d in enumerate(dims):
        per16 = 16 // (2 if dtype == "bf16" else 4)
        for ld in (d, synth.pad_to(d, per16)):
            ref_all, _ = orc.gather(tables[l], np.arange(n))
            for staging, sd in ((None, None), (None, side), (stg, side), (stg, None)):
                out = torch.full((n, ld), 3.0, dtype=H.np_to_dev(tables[l][:1]).dtype, device="cuda")
                rc, st = B.halo_gather(c, l, None, n, out, ld, stream=main, side_stream=sd, staging=staging, want_stats=True)
                got = H.dev_to_np(out)
                assert got[:, :d].tobytes() == ref_all.tobytes(), (l, ld, staging is not None, sd is not None)
                assert (O.widen(got[:, d:]) == 3.0).all()
                assert (st.hits, st.misses, st.absent) == (cap, n - cap, 0)
            # request list: duplicates, arbitrary order, by halo-local index and by global id, absent ids
            req = rng.integers(0, n, 7001).astype(np.int64)
            ref, _ = orc.gather(tables[l], req)
            for by_gid, sd in ((False, None), (True, side)):
                ids_h = part.halo_gid[req] if by_gid else req
                out = torch.full((len(req), ld), 3.0, dtype=H.np_to_dev(tables[l][:1]).dtype, device="cuda")
                rc, st = B.halo_gather(c, l, torch.from_numpy(ids_h).cuda(), len(req), out, ld, by_gid=by_gid,
                                       stream=main, side_stream=sd, want_stats=True)
                assert H.dev_to_np(out)[:, :d].tobytes() == ref.tobytes()
                assert st.hits == int((tier[req] == 0).sum()) and st.misses == int((tier[req] == 1).sum())
            bad = req.copy()
            bad[10], bad[500] = -5, n + 3
            ref, n_abs = orc.gather(tables[l], bad)
            out = torch.full((len(req), ld), 3.0, dtype=H.np_to_dev(tables[l][:1]).dtype, device="cuda")
            rc, st = B.halo_gather(c, l, torch.from_numpy(bad).cuda(), len(bad), out, ld, stream=main,
                                   want_stats=True, check=False)
            assert rc == B.ENOTFOUND and st.absent == n_abs == 2
            assert H.dev_to_np(out)[:, :d].tobytes() == ref.tobytes()
    c.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("cap_frac", [0.0, 0.37, 1.0])
def test_cache_update_and_stale_list_bit_exact(env, dtype, cap_frac):
    """Vertex update (both tiers, repeated and absent ids, by index and by global id) and the
    bounded-staleness list against the oracle: every cached byte and every stamp afterwards."""
    torch, B, H, O, orc = env["torch"], env["B"], env["H"], env["O"], env["orc"]
    part = synth.make_partition("cache-upd", 300, 5000, 30000, seed=23, max_deg=200)
    n = part.n_halo
    cap = int(cap_frac * n)
    dims = [70, 256]
    dt = B.BF16 if dtype == "bf16" else B.F32
    tables = [synth.make_features(n, d, seed=5, stream=40 + i, dtype=dtype) for i, d in enumerate(dims)]
    stamps = [np.zeros(n, np.int64) for _ in dims]
    c = B.Cache(part.halo_gid, part.halo_prio, cap, dims, dt, B.MAP_HASH)
    for l in range(len(dims)):
        c.fill(l, tables[l])
    tier, _ = c.query(np.arange(n))
    rng = np.random.default_rng(6)
    main = torch.cuda.Stream()
    ids_out = torch.empty(n, dtype=torch.int64, device="cuda")
    for epoch in range(1, 6):
        for l, d in enumerate(dims):
            per16 = 16 // (2 if dtype == "bf16" else 4)
            ld = d if epoch % 2 else synth.pad_to(d, per16) + per16
            m = int(rng.integers(1, 3000))
            ids = rng.integers(-2, n + 2, m).astype(np.int64)                      # repeats and absent ids
            by_gid = bool(epoch % 2 == 0)
            ids_call = np.where((ids >= 0) & (ids < n), part.halo_gid[np.clip(ids, 0, n - 1)], (1 << 45) + ids) if by_gid else ids
            rows = synth.make_features(m, d, seed=100 + epoch, stream=50 + l, dtype=dtype)
            say(f"cache update dtype={dtype} cap={cap}/{n} epoch={epoch} layer={l} m={m} ld={ld} by_gid={by_gid}")
            rows_d = H.padded_matrix(rows, ld)
            torch.cuda.synchronize()
            st = B.cache_update(c, l, torch.from_numpy(ids_call).cuda(), m, rows_d, ld, epoch, by_gid=by_gid, stream=main,
                                want_stats=True)
            n_abs = orc.cache_update(tables[l], stamps[l], ids, rows, epoch)
            last = np.full(n, -1, np.int64)
            ok = (ids >= 0) & (ids < n)
            last[ids[ok]] = np.nonzero(ok)[0]                                      # one write per distinct vertex
            touched = np.nonzero(last >= 0)[0]
            assert st.absent == n_abs
            assert st.hits == int((tier[touched] == 0).sum()) and st.misses == int((tier[touched] == 1).sum())
            out = torch.full((n, ld), 3.0, dtype=rows_d.dtype, device="cuda")
            torch.cuda.synchronize()
            B.halo_gather(c, l, None, n, out, ld, stream=main)
            torch.cuda.synchronize()
            assert H.dev_to_np(out)[:, :d].tobytes() == tables[l].tobytes()
            for max_age in (0, 2):
                cnt, oldest = B.cache_stale(c, l, epoch, max_age, ids_out, stream=main)
                ref_ids, ref_old = orc.stale_ids(stamps[l], epoch, max_age)
                assert cnt == len(ref_ids) and oldest == ref_old
                assert np.array_equal(ids_out[:cnt].cpu().numpy(), ref_ids)
    # a refill starts the layer's history again
    c.fill(0, tables[0])
    cnt, oldest = B.cache_stale(c, 0, 5, 0, ids_out, stream=main)
    assert cnt == n and oldest == 0
    c.close()


def test_cache_edge_cases(env):
    torch, B = env["torch"], env["B"]
    with pytest.raises(B.CapgnnError):
        B.Cache(np.array([5, 5], np.int64), np.array([1, 2], np.int64), 1, [4], B.F32)     # duplicate gid
    c = B.Cache(np.zeros(0, np.int64), np.zeros(0, np.int64), 10, [4], B.F32)                # empty halo
    out = torch.zeros((1, 4), device="cuda")
    assert B.halo_gather(c, 0, None, 0, out, 4) == B.OK
    with pytest.raises(B.CapgnnError):
        B.halo_gather(c, 1, None, 0, out, 4)                                                 # no such layer
    c.close()


def test_zipf_request_stream_hit_rate(env):
    """Requests drawn Zipf(1.1) over halo vertices ranked by priority, top 10 % on the GPU:
    the measured hit fraction equals H_{k,s}/H_{N,s} up to sampling noise."""
    torch, B = env["torch"], env["B"]
    N, k, s = 200_000, 20_000, 1.1
    p = np.arange(1, N + 1, dtype=np.float64) ** -s
    p /= p.sum()
    rng = np.random.default_rng(5)
    gid = rng.permutation(N).astype(np.int64) * 3 + 11
    prio = (1e12 * p).astype(np.int64)
    c = B.Cache(gid, prio, k, [16], B.F32, B.MAP_HASH)
    c.fill(0, np.zeros((N, 16), np.float32))
    req = rng.choice(N, size=1_000_000, p=p)
    out = torch.empty((len(req), 16), device="cuda")
    rc, st = B.halo_gather(c, 0, torch.from_numpy(gid[req]).cuda(), len(req), out, 16, by_gid=True, want_stats=True)
    expect = float(np.sum(np.arange(1, k + 1, dtype=np.float64) ** -s) / np.sum(np.arange(1, N + 1, dtype=np.float64) ** -s))
    assert abs(st.hits / len(req) - expect) < 3e-3
    c.close()


# ----------------------------------------------------------------------------- dense products
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_gemm_vs_oracle(env, dtype, ta, tb):
    torch, B, H, O, orc = env["torch"], env["B"], env["H"], env["O"], env["orc"]
    rng = np.random.default_rng(ta * 2 + tb)
    dt = B.BF16 if dtype == "bf16" else B.F32
    tol = TOL_BF16 if dtype == "bf16" else TOL_F32
    for (M, N, K) in [(1, 1, 1), (130, 41, 602), (257, 256, 100), (1000, 47, 256), (64, 200, 33), (300, 8, 5000)]:
        say(f"gemm {dtype} ta={ta} tb={tb} M={M} N={N} K={K}")
        A = rng.standard_normal((K, M) if ta else (M, K)).astype(np.float32)
        Bm = rng.standard_normal((N, K) if tb else (K, N)).astype(np.float32)
        bias = rng.standard_normal(N).astype(np.float32)
        if dtype == "bf16":
            A, Bm = synth.f32_to_bf16_rne(A).reshape(A.shape), synth.f32_to_bf16_rne(Bm).reshape(Bm.shape)
        ref = orc.matmul(O.widen(A), O.widen(Bm), ta=bool(ta), tb=bool(tb))
        for pad in (0, 3):
            lda, ldb, ldc = A.shape[1] + pad, Bm.shape[1] + pad, N + pad
            Ad, Bd = H.padded_matrix(A, lda), H.padded_matrix(Bm, ldb)
            Ad[:, A.shape[1]:] = float("nan")            # whatever the padding holds must not reach the result
            Bd[:, Bm.shape[1]:] = float("nan")
            wsb = B.gemm_workspace_bytes(ta, M, N, K)
            ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
            Cd = torch.full((M, ldc), 2.0, dtype=torch.float32, device="cuda")
            B.gemm(ta, tb, M, N, K, Ad, lda, Bd, ldb, Cd, ldc, dt, out_f32=1, ws=ws, ws_bytes=wsb)
            torch.cuda.synchronize()
            got = Cd.cpu().numpy()
            assert O.normwise(got[:, :N], ref) <= tol
            assert (got[:, N:] == 2.0).all()
            # epilogue: accumulate + bias + relu, output in the storage dtype
            Cd2 = torch.full((M, ldc), 0.5, dtype=Ad.dtype, device="cuda")
            B.gemm(ta, tb, M, N, K, Ad, lda, Bd, ldb, Cd2, ldc, dt, accumulate=1, bias=H.np_to_dev(bias), relu=1,
                   ws=ws, ws_bytes=wsb)
            torch.cuda.synchronize()
            ref2 = np.maximum(ref + 0.5 + bias[None, :], 0.0)
            assert O.normwise(O.widen(H.dev_to_np(Cd2))[:, :N], ref2) <= tol


@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_gemm_bf16_matrix_core_path(env, ta, tb):
    """bf16 operands with 16-byte aligned rows take the bf16 MFMA kernel (weights of plain products are
    repacked, so their pitch may be anything).  Small-integer operands make every product and partial sum
    exactly representable: the result must equal the oracle exactly, which pins the operand lane layout;
    random operands are compared within the bf16 tolerance.  Sizes span several tiles and ragged tails."""
    torch, B, H, O, orc = env["torch"], env["B"], env["H"], env["O"], env["orc"]
    rng = np.random.default_rng(10 + ta * 2 + tb)
    for (M, N, K) in [(333, 47, 256), (130, 256, 40), (257, 130, 1000), (64, 64, 32), (500, 41, 4100)]:
        for ints in (True, False):
            say(f"gemm bf16 mfma ta={ta} tb={tb} M={M} N={N} K={K} ints={ints}")
            shapeA, shapeB = ((K, M) if ta else (M, K)), ((N, K) if tb else (K, N))
            if ints:
                A = rng.integers(-2, 3, shapeA).astype(np.float32)
                Bm = rng.integers(-2, 3, shapeB).astype(np.float32)
            else:
                A = rng.standard_normal(shapeA).astype(np.float32)
                Bm = rng.standard_normal(shapeB).astype(np.float32)
            A, Bm = synth.f32_to_bf16_rne(A).reshape(A.shape), synth.f32_to_bf16_rne(Bm).reshape(Bm.shape)
            ref = orc.matmul(O.widen(A), O.widen(Bm), ta=bool(ta), tb=bool(tb))
            lda = synth.pad_to(A.shape[1], 8)
            ldb = synth.pad_to(Bm.shape[1], 8) if ta else Bm.shape[1] + 1     # a weight's pitch is free
            ldc = N + 3
            Ad, Bd = H.padded_matrix(A, lda), H.padded_matrix(Bm, ldb)
            Ad[:, A.shape[1]:] = float("nan")            # a ragged last column group is read up to the pitch: the padding
            Bd[:, Bm.shape[1]:] = float("nan")            # must end up nowhere in the result
            wsb = B.gemm_workspace_bytes(ta, M, N, K)
            ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
            Cd = torch.full((M, ldc), 2.0, dtype=torch.float32, device="cuda")
            B.gemm(ta, tb, M, N, K, Ad, lda, Bd, ldb, Cd, ldc, B.BF16, out_f32=1, ws=ws, ws_bytes=wsb)
            torch.cuda.synchronize()
            got = Cd.cpu().numpy()
            if ints:
                assert np.array_equal(got[:, :N].astype(np.float64), ref)
            else:
                assert O.normwise(got[:, :N], ref) <= TOL_BF16
            assert (got[:, N:] == 2.0).all()


@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 0)])
def test_gemm_f32_split_product(env, ta, tb):
    """fp32 operands cut into three bf16 pieces and multiplied on the bf16 matrix cores.  (1) With one operand a signed
    selection matrix (one +-2^e entry per output column / row) every output is a single product that fp32 holds exactly, so
    all 24 bits of the other operand must come through: bit-exact, which pins the cut, the piece order and both LDS
    layouts.  (2) Random operands: within the fp32 tolerance of the fp64 oracle, and no further from it than four times
    the distance of the fp32 matrix instruction plus 2^-23, the bound on the three piece products that are dropped (both
    distances are rounding noise of the fp32 accumulation, a hundred times below the tolerance)."""
    torch, B, H, O, orc = env["torch"], env["B"], env["H"], env["O"], env["orc"]
    rng = np.random.default_rng(40 + ta * 2 + tb)

    def run(mode, A, Bm, M, N, K, pad):
        lda, ldb, ldc = A.shape[1] + pad, Bm.shape[1] + pad, N + pad
        Ad, Bd = H.padded_matrix(A, lda), H.padded_matrix(Bm, ldb)
        wsb = B.gemm_workspace_bytes(ta, M, N, K)
        ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
        Cd = torch.full((M, ldc), 2.0, dtype=torch.float32, device="cuda")
        B.gemm(ta, tb, M, N, K, Ad, lda, Bd, ldb, Cd, ldc, B.F32, out_f32=1, ws=ws, ws_bytes=wsb, f32_product=mode)
        torch.cuda.synchronize()
        got = Cd.cpu().numpy()
        assert (got[:, N:] == 2.0).all()
        return got[:, :N]

    for (M, N, K) in [(1, 1, 1), (130, 41, 602), (257, 256, 100), (300, 130, 1000), (602, 256, 5000), (64, 200, 33)]:
        shapeA, shapeB = ((K, M) if ta else (M, K)), ((N, K) if tb else (K, N))
        for which in ("select_b", "select_a", "random"):
            say(f"gemm f32 split ta={ta} tb={tb} M={M} N={N} K={K} {which}")
            full = lambda shape: (rng.integers(1 << 23, 1 << 24, shape) * rng.choice([-1.0, 1.0], shape)
                                  * 2.0 ** rng.integers(-20, 20, shape)).astype(np.float32)
            if which == "select_b":              # B[k_j, j] = +-2^e, zero elsewhere
                A = full(shapeA)
                sel = np.zeros((K, N), np.float32)
                sel[rng.integers(0, K, N), np.arange(N)] = rng.choice([-1.0, 1.0], N) * 2.0 ** rng.integers(-8, 8, N)
                Bm = np.ascontiguousarray(sel.T) if tb else sel
            elif which == "select_a":            # A[i, k_i] = +-2^e (op(A) is M x K)
                Bm = full(shapeB)
                sel = np.zeros((M, K), np.float32)
                sel[np.arange(M), rng.integers(0, K, M)] = rng.choice([-1.0, 1.0], M) * 2.0 ** rng.integers(-8, 8, M)
                A = np.ascontiguousarray(sel.T) if ta else sel
            else:
                A = rng.standard_normal(shapeA).astype(np.float32)
                Bm = rng.standard_normal(shapeB).astype(np.float32)
            ref = orc.matmul(A, Bm, ta=bool(ta), tb=bool(tb))
            for pad in (0, 3):
                got = run(B.F32_PRODUCT_SPLIT, A, Bm, M, N, K, pad)
                if which != "random":
                    assert np.array_equal(got.astype(np.float64), ref)
                    continue
                nat = run(B.F32_PRODUCT_NATIVE, A, Bm, M, N, K, pad)
                e_split, e_nat = O.normwise(got, ref), O.normwise(nat, ref)
                say(f"   normwise error: split {e_split:.3e}, fp32 instruction {e_nat:.3e}")
                assert e_split <= TOL_F32 and e_nat <= TOL_F32
                assert e_split <= 4.0 * e_nat + 2.0 ** -23
    one = torch.zeros(1, device="cuda")
    with pytest.raises(B.CapgnnError):          # an unknown form is an argument error
        B.gemm(0, 0, 1, 1, 1, one, 1, one, 1, one, 1, B.F32, f32_product=7)


def test_mfma_peak_loop_runs_and_counts_its_work(env):
    """The register-resident matrix-instruction loop: the reported work is 4 tiles x 4 waves x iterations x workgroups x
    the instruction's 2 * 32 * 32 * k FLOPs, and every thread writes a finite, positive checksum (its operands are
    positive)."""
    torch, B = env["torch"], env["B"]
    wgs, iters = 8, 16
    out = torch.full((wgs * 256,), -1.0, dtype=torch.float32, device="cuda")
    for dt, k in ((B.F32, 2), (B.BF16, 16)):
        flop = B.mfma_peak(dt, wgs, iters, out)
        torch.cuda.synchronize()
        assert flop == 2.0 * 32 * 32 * k * 4 * iters * 4 * wgs
        got = out.cpu().numpy()
        assert np.isfinite(got).all() and (got > 0).all()
    with pytest.raises(B.CapgnnError):
        B.mfma_peak(B.F32, 0, iters, out)


def test_gemm_relu_mask_epilogue(env):
    torch, B, H, O, orc = env["torch"], env["B"], env["H"], env["O"], env["orc"]
    rng = np.random.default_rng(3)
    M, N, K = 333, 70, 50
    A, Bm = rng.standard_normal((M, K)).astype(np.float32), rng.standard_normal((N, K)).astype(np.float32)
    mask = rng.standard_normal((M, N)).astype(np.float32)
    mask[0, :5] = 0.0
    Cd = torch.zeros((M, N), device="cuda")
    B.gemm(0, 1, M, N, K, H.np_to_dev(A), K, H.np_to_dev(Bm), K, Cd, N, B.F32, relu_mask=H.np_to_dev(mask), ldm=N)
    torch.cuda.synchronize()
    ref = orc.matmul(A, Bm, tb=True) * (mask > 0)
    assert O.normwise(Cd.cpu().numpy(), ref) <= TOL_F32


# ----------------------------------------------------------------------------- loss
@pytest.mark.parametrize("C", [1, 8, 41, 47, 100, 300])
def test_softmax_ce_vs_oracle(env, C):
    torch, B, H, O, orc = env["torch"], env["B"], env["H"], env["O"], env["orc"]
    rng = np.random.default_rng(C)
    n = 1237
    Z = (rng.standard_normal((n, C)) * 4).astype(np.float32)
    y = rng.integers(0, C, n).astype(np.int32)
    mask = (rng.random(n) < 0.6).astype(np.uint8)
    ws_b = B.loss_workspace_bytes(n)
    ws = torch.empty(ws_b, dtype=torch.uint8, device="cuda")
    for m, norm in ((mask, 0.0), (None, 0.0), (mask, 777.0)):
        loss_d = torch.zeros(1, device="cuda")
        dZ = torch.full((n, C + 2), 9.0, device="cuda")
        B.softmax_ce(n, C, H.np_to_dev(Z), C, H.np_to_dev(y), None if m is None else H.np_to_dev(m), norm, loss_d, dZ,
                     C + 2, B.F32, ws, ws_b)
        torch.cuda.synchronize()
        ref_loss, ref_dZ = orc.softmax_ce(Z.astype(np.float64), y, m, norm)
        assert abs(float(loss_d.item()) - ref_loss) <= 1e-5 * max(1.0, abs(ref_loss))
        got = dZ.cpu().numpy()
        assert O.normwise(got[:, :C], ref_dZ) <= TOL_F32
        assert (got[:, C:] == 9.0).all()
