"""RAPA's subgraph adjustment (Alg. 2 / Alg. 3 with the cost model of Eq. 3-5) in the library against the CPU oracle.

The removal decisions are integers decided by double-precision costs and by the order of the influence scores, so:
  * on identical score arrays (exactly representable values) the library's keep masks, status vector and sweep count
    must equal the oracle's exactly, and its costs to the last bits (no GPU needed);
  * end to end on a synthetic 4-way partition, with the scores of capgnn_influence_score (fp32, GPU) on one side and
    the oracle's own fp64 scores on the other, sweeps, status vector and the number of removed vertices must be equal,
    the masks may differ only among vertices whose oracle scores lie within fp32 rounding of one another (a run of
    near-ties may be ordered differently by the two precisions), and the pruned subgraphs must equal the oracle's.
"""
import numpy as np
import pytest

from paper_2508_13716_amd import synth


def _devices(rng, P, mem=1e18):
    """Synthetic heterogeneous GPUs: measured costs spread over a factor of four (one GPU machine has one GPU; the rates of the
    others are made up, as the cost model only asks for per-GPU numbers)."""
    return [tuple(rng.uniform(0.5, 2.0, 5).tolist()) + (mem,) for _ in range(P)]


def _both_devices(orc, B, spec):
    return [orc.RapaDevice(*d) for d in spec], [B.RapaDevice(*d) for d in spec]


def _params(orc, B, alpha, eps, **kw):
    o = orc.RapaParams(alpha=alpha, epsilon=eps, **kw)
    return o, B.RapaParams(o.alpha, o.epsilon, o.m_vertex, o.m_edge, o.m_feat, o.f_dim, o.beta, o.max_sweeps)


def test_rapa_adjust_matches_oracle_exactly_on_identical_scores(orc):
    from paper_2508_13716_amd import binding as B
    B.lib()
    rng = np.random.default_rng(23)
    for trial in range(60):
        P = int(rng.integers(1, 7))
        n_inner = rng.integers(50, 5000, P)
        e_inner = rng.integers(100, 50000, P)
        halo_edges = [rng.integers(1, 40, int(rng.integers(0, 400))).astype(np.int64) for _ in range(P)]
        scores = [(rng.integers(0, 64, len(h)) / 64.0).astype(np.float32) for h in halo_edges]      # many exact ties
        mem = 1e18 if trial % 3 else float(rng.uniform(2e5, 2e6))                                     # sometimes memory binds
        spec = _devices(rng, P, mem)
        od, bd = _both_devices(orc, B, spec)
        op, bp = _params(orc, B, float(rng.uniform(0.0, 1.0)), float(rng.uniform(0.0, 200.0)), f_dim=int(rng.integers(0, 64)),
                         beta=1000.0)
        ref = orc.rapa_do_partition(n_inner.tolist(), e_inner.tolist(), halo_edges, scores, od, op)
        got = B.rapa_adjust(n_inner, e_inner, halo_edges, scores, bd, bp)
        assert got["sweeps"] == ref["sweeps"] and got["r"] == ref["r"], trial
        for i in range(P):
            assert np.array_equal(got["keep"][i].astype(bool), ref["keep"][i]), (trial, i)
        np.testing.assert_array_equal(got["lam"], np.array(ref["lam"]))                                # same operations, same order
        assert abs(got["sigma"] - ref["sigma"][-1]) <= 1e-12 * max(1.0, ref["sigma"][-1])
    # the hand-traced example of tests/golden/rapa_hand_trace.txt through the library
    od, bd = _both_devices(orc, B, [(2.0, 2.0, 1.0, 1.0, 1.0, 1e18), (1.0, 1.0, 1.0, 1.0, 1.0, 1e18)])
    _, bp = _params(orc, B, 0.5, 1.0)
    got = B.rapa_adjust([10, 10], [20, 20], [np.array([3, 1, 2, 4]), np.array([2, 2])],
                        [np.array([0.5, 0.1, 0.3, 0.9]), np.array([0.2, 0.4])], bd, bp)
    assert got["sweeps"] == 3 and got["lam"].tolist() == [15.0, 14.5] and got["sigma"] == 0.25
    assert got["keep"][0].tolist() == [0, 0, 0, 0] and got["keep"][1].tolist() == [1, 1] and got["r"] == [0, 1]
    # argument errors
    with pytest.raises(B.CapgnnError):
        B.rapa_adjust([10], [20], [np.array([1])], [np.array([0.5])], [B.RapaDevice(0.0, 1, 1, 1, 1, 1e18)], bp)    # cost of 0
    bad = B.RapaParams(1.5, 0.0, 8, 12, 4, 0, 0, 10)
    with pytest.raises(B.CapgnnError):
        B.rapa_adjust([10], [20], [np.array([1])], [np.array([0.5])], [B.RapaDevice(1, 1, 1, 1, 1, 1e18)], bad)      # alpha > 1


def test_halo_edge_counts_and_prune_match_oracle(orc):
    from paper_2508_13716_amd import binding as B
    B.lib()
    parts, _ = synth.make_partitioned_graph(6000, 90000, 3, seed=4, shares=[3, 2, 1])
    rng = np.random.default_rng(8)
    for p in parts + [synth.hand_partition(3, 0, [(0, 1), (2, 0)]), synth.hand_partition(2, 3, [])]:
        e_ref, c_ref = orc.halo_edge_counts(p.n_loc, p.n_halo, p.rowptr, p.col)
        e_got, c_got = B.halo_edge_counts(p.n_loc, p.n_halo, p.rowptr, p.col)
        assert e_got == e_ref and np.array_equal(c_got, c_ref)
        for frac in (0.0, 0.4, 1.0):
            keep = (rng.random(p.n_halo) < frac).astype(np.uint8)
            rp, cl, ni = B.prune_halo(p.n_loc, p.n_halo, p.rowptr, p.col, keep)
            rp_ref, cl_ref, ni_ref = orc.prune_halo(p.n_loc, p.n_halo, p.rowptr, p.col, keep)
            assert np.array_equal(rp, rp_ref) and np.array_equal(cl, cl_ref) and np.array_equal(ni, ni_ref)
    with pytest.raises(B.CapgnnError):
        B.halo_edge_counts(2, 1, np.array([0, 1, 2]), np.array([0, 9], np.int32))


@pytest.mark.gpu
def test_rapa_end_to_end_on_a_four_way_partition(orc):
    """Influence scores on the GPU (Eq. 6), adjustment and pruning in the library, everything again in the oracle."""
    import torch
    from paper_2508_13716_amd import binding as B
    B.lib()
    P = 4
    parts, info = synth.make_partitioned_graph(40000, 900000, P, seed=synth.BASE_SEED * 10 + 11, shares=[4, 3, 2, 1])
    rng = np.random.default_rng(5)
    spec = _devices(rng, P)
    od, bd = _both_devices(orc, B, spec)
    n_inner, e_inner, he, s_gpu, s_ref = [], [], [], [], []
    for p in parts:
        ei, cnt = B.halo_edge_counts(p.n_loc, p.n_halo, p.rowptr, p.col)
        n_inner.append(p.n_loc); e_inner.append(ei); he.append(cnt)
        # Eq. 6: in-degrees of the original graph for the rows (every in-neighbour of an inner vertex is in the subgraph),
        # out-degrees in the subgraph, repetition count = in how many subgraphs the vertex appears
        din = np.maximum(np.diff(p.rowptr), 1)
        dout = np.maximum(np.bincount(p.col, minlength=p.n_cols), 1)
        count = np.concatenate([np.ones(p.n_loc), p.halo_prio.astype(np.float64)])
        g = B.Graph(p.n_loc, p.n_halo, p.rowptr, p.col)
        S = torch.zeros(p.n_cols, device="cuda")
        B.influence_score(g, torch.from_numpy((1.0 / np.sqrt(din)).astype(np.float32)).cuda(),
                          torch.from_numpy((1.0 / np.sqrt(dout)).astype(np.float32)).cuda(),
                          torch.from_numpy(count.astype(np.float32)).cuda(), S)
        torch.cuda.synchronize()
        g.close()
        s_gpu.append(S.cpu().numpy()[p.n_loc:])
        s_ref.append(orc.influence_score(p.n_loc, p.n_cols, p.rowptr, p.col, din, dout, count)[p.n_loc:])
        assert np.abs(s_gpu[-1] - s_ref[-1]).max() <= 1e-5 * np.abs(s_ref[-1]).max()
    lam0 = [orc.rapa_cost(n_inner[i], e_inner[i] + int(he[i].sum()), int(he[i].sum()), i, od, orc.RapaParams(0.5, 0.0)) for i in range(P)]
    op, bp = _params(orc, B, 0.5, 0.01 * float(np.mean(lam0)), f_dim=128)          # epsilon = 1 % of the mean cost (evaluation setup)
    ref = orc.rapa_do_partition(n_inner, e_inner, he, s_ref, od, op)
    got = B.rapa_adjust(n_inner, e_inner, he, s_gpu, bd, bp)
    print(f"RAPA on {P} subgraphs: sweeps {got['sweeps']} (oracle {ref['sweeps']}), halo vertices kept "
          f"{[int(k.sum()) for k in got['keep']]} of {[p.n_halo for p in parts]}, costs {np.round(lam0, 0).tolist()} -> "
          f"{np.round(got['lam'], 0).tolist()}, sigma {got['sigma']:.1f}", flush=True)
    assert sum(int((~k).sum()) for k in ref["keep"]) > 0, "the example prunes nothing"
    assert got["sweeps"] == ref["sweeps"] and got["r"] == ref["r"]
    for i, p in enumerate(parts):
        same = np.array_equal(got["keep"][i].astype(bool), ref["keep"][i])
        if not same:
            # scores that are equal in fp64 but not in fp32 (or the reverse) may swap places inside a run of ties: the two
            # masks may then differ only among vertices whose oracle scores are within fp32 rounding of one another
            d = np.nonzero(got["keep"][i].astype(bool) != ref["keep"][i])[0]
            spread = s_ref[i][d].max() - s_ref[i][d].min()
            print(f"subgraph {i}: {len(d)} vertices differ, their oracle scores span {spread:.3e}", flush=True)
            assert spread <= 1e-5 * s_ref[i].max() and got["keep"][i].sum() == ref["keep"][i].sum(), (i, len(d), spread)
        np.testing.assert_allclose(got["lam"][i], ref["lam"][i], rtol=1e-9 if same else 1e-3)
        rp, cl, ni = B.prune_halo(p.n_loc, p.n_halo, p.rowptr, p.col, got["keep"][i])
        rp_ref, cl_ref, ni_ref = orc.prune_halo(p.n_loc, p.n_halo, p.rowptr, p.col, got["keep"][i].astype(bool))
        assert np.array_equal(rp, rp_ref) and np.array_equal(cl, cl_ref) and np.array_equal(ni, ni_ref)
