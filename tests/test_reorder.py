"""Vertex storage order (the subgraph reordering step): the library's host routines against the oracle's
(bit-exact, no GPU needed), and the epoch on a relabelled partition against the oracle (GPU)."""
import numpy as np
import pytest

from paper_2508_13716_amd import synth

METHODS = {"popularity": 0, "bfs": 1}


def _graphs():
    rng = np.random.default_rng(3)
    gs = [synth.make_partition("ord-a", 300, 200, 2500, seed=1, max_deg=60),
          synth.make_partition("ord-b", 5000, 0, 60000, seed=2, max_deg=900),
          synth.make_partition("ord-c", 64, 4000, 3000, seed=3, max_deg=200, halo_edge_frac=0.9),
          synth.partition_for(synth.CONFIGS["C1"]),
          synth.partition_for(synth.CONFIGS["C3"].scaled(0.02)),
          synth.hand_partition(5, 3, [], name="no-edges"),
          synth.hand_partition(0, 0, [], name="empty")]
    n = 500
    lab = rng.permutation(n)
    ring = [(int(lab[i]), int(lab[(i + 1) % n])) for i in range(n)]
    gs.append(synth.hand_partition(n, 0, ring + [(b, a) for a, b in ring], name="shuffled-ring"))
    return gs


def test_library_order_and_relabelling_equal_the_oracle(orc):
    from paper_2508_13716_amd import binding as B
    rng = np.random.default_rng(4)
    for part in _graphs():
        for name, mid in METHODS.items():
            want = orc.locality_order(name, part.n_loc, part.n_halo, part.rowptr, part.col)
            got = B.locality_order(mid, part.n_loc, part.n_halo, part.rowptr, part.col)
            assert np.array_equal(got, want), (part.name, name)
            if part.nnz <= 70000:        # the oracle's relabelling is a pure-Python loop
                val = rng.standard_normal(part.nnz).astype(np.float32)
                rp, cl, vl = B.relabel_csr(part.n_loc, part.n_halo, part.rowptr, part.col, got, val)
                rp0, cl0, vl0 = orc.relabel_csr(part.n_loc, part.rowptr, part.col, want, val)
                assert np.array_equal(rp, rp0) and np.array_equal(cl, cl0) and np.array_equal(vl, vl0), part.name


def test_relabelling_rejects_what_is_not_a_range_keeping_permutation():
    from paper_2508_13716_amd import binding as B
    rowptr, col = np.array([0, 2, 3, 5]), np.array([1, 3, 2, 0, 4], np.int32)
    for bad in ([0, 0, 1, 3, 4], [0, 1, 3, 2, 4], [0, 1, 2, 3, 5], [0, 1, 2, 4, 4]):
        with pytest.raises(B.CapgnnError):
            B.relabel_csr(3, 2, rowptr, col, np.array(bad, np.int32))
    with pytest.raises(B.CapgnnError):
        B.locality_order(7, 3, 2, rowptr, col)
    with pytest.raises(B.CapgnnError):
        B.locality_order(0, 3, 2, rowptr, np.array([1, 3, 2, 0, 5], np.int32))     # column out of range


@pytest.mark.gpu
@pytest.mark.parametrize("name,scale", [("C1", 1.0), ("C2", 0.02), ("C3", 0.01), ("C5", 0.004)])
def test_epoch_on_relabelled_partition_matches_oracle_and_the_original(orc, name, scale):
    """The library's order, applied by the host harness, against the oracle's own relabelled problem; and the
    per-vertex outputs of the relabelled run against the original run's, moved with their vertices."""
    import torch
    from paper_2508_13716_amd import binding as B, harness as H
    from tests import oracle_side as O
    from tests.gpu_compare import compare_epoch, TOL
    env = dict(torch=torch, B=B, H=H, O=O, orc=orc)
    cfg = synth.CONFIGS[name] if scale == 1.0 else synth.CONFIGS[name].scaled(scale)
    prob = H.make_problem(cfg, mask_frac=0.5)
    part = prob.part
    dp0 = H.DeviceProblem(prob)
    loss0, _ = dp0.run_epoch()
    logits0 = dp0.results()["logits"]
    dp0.close()
    for mname, mid in METHODS.items():
        print(f"{cfg.name} relabelled by {mname}", flush=True)
        prob2, new2old = H.relabel_problem(prob, mid)
        want = O.relabelled_problem(prob, orc.locality_order(mname, part.n_loc, part.n_halo, part.rowptr, part.col))
        assert np.array_equal(prob2.part.rowptr, want.part.rowptr) and np.array_equal(prob2.part.col, want.part.col)
        assert np.array_equal(prob2.X0, want.X0) and np.array_equal(prob2.part.halo_gid, want.part.halo_gid)
        dp = H.DeviceProblem(prob2)
        loss, _ = dp.run_epoch()
        compare_epoch(env, want, dp, O.oracle_epoch(want), loss, TOL[cfg.dtype], f"{cfg.name} {mname}")
        logits = dp.results()["logits"]
        assert O.normwise(logits, logits0[new2old[: part.n_loc]]) <= TOL[cfg.dtype]
        assert abs(loss - loss0) <= TOL[cfg.dtype] * max(1.0, abs(loss0))
        dp.close()
