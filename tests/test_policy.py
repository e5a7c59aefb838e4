"""Policy layer: the native two-level cache policy simulator against the oracle's model (host code, no GPU
needed), and the overlap-ratio kernel against the oracle (GPU)."""
import numpy as np
import pytest

from paper_2508_13716_amd import synth

POLICIES = {"jaca": 0, "jaca_low": 1, "fifo": 2, "lru": 3}


def test_native_policy_simulator_matches_the_oracle_exactly(orc):
    from paper_2508_13716_amd import binding as B
    rng = np.random.default_rng(21)
    cases = [[np.unique(rng.integers(0, 400, 150)) for _ in range(4)],
             [np.arange(0, 50), np.arange(100, 130)],
             [np.array([1, 2, 7]), np.array([7, 20]), np.array([7, 30, 31])],
             [np.zeros(0, np.int64), np.array([5])]]
    sets, _ = synth.make_halo_sets(3000, 40000, 5, seed=17)
    cases.append(sets)
    for sets in cases:
        sets = [np.asarray(h, np.int64) for h in sets]
        biggest = max(len(h) for h in sets)
        for name, pid in POLICIES.items():
            for cap_l, cap_g in [(0, 0), (1, 1), (7, 3), (biggest // 3, biggest // 2), (biggest, 10 * biggest), (0, biggest)]:
                for epochs, warmup in [(3, 1), (2, 0), (1, 1)]:
                    want = orc.policy_hit_counts(sets, name, cap_l, cap_g, epochs, warmup)
                    got = B.policy_simulate(sets, pid, cap_l, cap_g, epochs, warmup)
                    assert got == want, (name, cap_l, cap_g, epochs, warmup)
    with pytest.raises(B.CapgnnError):                         # a halo set must be ascending and duplicate-free
        B.policy_simulate([np.array([3, 3, 4], np.int64)], 0, 1, 1, 2)


def test_hit_rate_curves_have_the_shape_the_evaluation_reports(orc):
    """On a random 4-way partition of a power-law graph: prioritising high-overlap vertices beats low-overlap
    ones, JACA's hit rate grows with capacity and reaches 100 %, and FIFO / LRU, swept cyclically by full-batch
    training, stay behind it until the caches hold everything."""
    from paper_2508_13716_amd import binding as B
    sets, _ = synth.make_halo_sets(20000, 400000, 4, seed=18)
    total = sum(len(h) for h in sets)
    union = len(np.unique(np.concatenate(sets)))
    rate = lambda c: (c[0] + c[1]) / (c[0] + c[1] + c[2])
    prev = -1.0
    for frac in (0.05, 0.2, 0.5, 1.0):
        cap_g = int(frac * union)
        cap_l = cap_g // 8 if frac < 1.0 else cap_g          # a small local level lets the shared level show
        jaca = rate(B.policy_simulate(sets, B.POLICY_JACA, cap_l, cap_g, 3))
        low = rate(B.policy_simulate(sets, B.POLICY_JACA_LOW, cap_l, cap_g, 3))
        fifo = rate(B.policy_simulate(sets, B.POLICY_FIFO, cap_l, cap_g, 3))
        lru = rate(B.policy_simulate(sets, B.POLICY_LRU, cap_l, cap_g, 3))
        print(f"global capacity {frac:4.0%} of {union} halo vertices, local {cap_l} ({total} requests/epoch): "
              f"JACA {jaca:.3f}  low-overlap-first {low:.3f}  FIFO {fifo:.3f}  LRU {lru:.3f}")
        assert jaca >= low and jaca >= fifo and jaca >= lru and jaca > prev
        if frac < 1.0:
            assert jaca > low                                 # the overlap ratio is what the shared level gains from
        prev = jaca
    assert prev == 1.0


@pytest.mark.gpu
def test_overlap_ratio_kernel_matches_the_oracle(orc):
    import torch
    from paper_2508_13716_amd import binding as B
    n = 50000
    sets, _ = synth.make_halo_sets(n, 600000, 6, seed=19)
    ids, cnt = orc.overlap_ratio(sets)
    ref = np.zeros(n, np.int32)
    ref[ids] = cnt
    flat = np.concatenate(sets + [np.array([-4, n, n + 9], np.int64)])       # ids outside the range are ignored
    R = torch.full((n,), 77, dtype=torch.int32, device="cuda")
    B.overlap_ratio(torch.from_numpy(flat).cuda(), len(flat), n, R)
    torch.cuda.synchronize()
    assert np.array_equal(R.cpu().numpy(), ref)
    assert ref.max() <= 6 and (ref >= 0).all()
    B.overlap_ratio(None, 0, n, R)                                            # no requests: all zero
    torch.cuda.synchronize()
    assert int(R.abs().sum()) == 0


@pytest.mark.gpu
@pytest.mark.parametrize("name,scale", [("C1", 1.0), ("C2", 0.05), ("C3", 0.02)])
def test_influence_score_kernel_matches_the_oracle(orc, name, scale):
    """Eq. 6 on partition graphs (self loops, a 20 000-entry row, halo vertices without rows) within the fp32
    tolerance, with and without repetition counts; the score of a vertex without incident edges is 0."""
    import torch
    from paper_2508_13716_amd import binding as B
    from tests import oracle_side as O
    cfg = synth.CONFIGS[name].scaled(scale) if scale != 1.0 else synth.CONFIGS[name]
    part = synth.partition_for(cfg)
    rng = np.random.default_rng(2)
    din = np.maximum(np.diff(part.rowptr), 1) * rng.integers(1, 4, part.n_loc)       # degrees "in the original graph"
    dout = np.maximum(np.bincount(part.col, minlength=part.n_cols), 1)
    count = rng.integers(1, 6, part.n_cols).astype(np.float32)
    g = B.Graph(part.n_loc, part.n_halo, part.rowptr, part.col)
    rs_in = torch.from_numpy((1.0 / np.sqrt(din)).astype(np.float32)).cuda()
    rs_out = torch.from_numpy((1.0 / np.sqrt(dout)).astype(np.float32)).cuda()
    S = torch.full((part.n_cols,), -1.0, device="cuda")
    for cnt in (None, count):
        B.influence_score(g, rs_in, rs_out, None if cnt is None else torch.from_numpy(cnt).cuda(), S)
        torch.cuda.synchronize()
        ref = orc.influence_score(part.n_loc, part.n_cols, part.rowptr, part.col, din, dout, cnt)
        err = O.normwise(S.cpu().numpy(), ref)
        print(f"influence score {cfg.name}: {part.n_cols} vertices, {part.nnz} edges, normwise error {err:.2e}", flush=True)
        assert err <= 1e-4
    g.close()
