"""Second workload variants: the multi-label loss (binary cross-entropy on logits) and GIN layers (sum aggregation
with a (1 + eps) self term), against the oracle."""
import copy

import numpy as np
import pytest

from paper_2508_13716_amd import synth


def test_gin_operator_equals_the_oracle(orc):
    from paper_2508_13716_amd import binding as B
    for part in (synth.make_partition("gin-a", 300, 200, 2500, seed=1, max_deg=60, self_loops=False),
                 synth.hand_partition(5, 3, [], name="no-edges"),
                 synth.hand_partition(0, 0, [], name="empty")):
        for eps in (0.0, 0.25, -1.0):
            rp, cl, vl = B.gin_operator(part.n_loc, part.n_halo, part.rowptr, part.col, eps)
            g = orc.gin_graph(part.n_loc, part.n_halo, part.rowptr, part.col, eps)
            assert np.array_equal(rp, g.rowptr) and np.array_equal(cl, g.col)
            assert np.array_equal(vl, g.v.astype(np.float32))


@pytest.mark.gpu
@pytest.mark.parametrize("dz", ["f32", "bf16"])
def test_sigmoid_bce_kernel_matches_oracle(orc, dz):
    import torch
    from paper_2508_13716_amd import binding as B, harness as H
    from tests import oracle_side as O
    rng = np.random.default_rng(41)
    for n, C, ld, use_mask, norm in [(1, 1, 1, False, 0.0), (37, 5, 8, True, 0.0), (1000, 47, 48, True, 0.0),
                                     (5000, 130, 130, False, 0.0), (300, 41, 44, True, 123.0)]:
        print(f"sigmoid_bce n={n} C={C} ld={ld} mask={use_mask} dz={dz}", flush=True)
        Z = (rng.standard_normal((n, C)) * 4.0).astype(np.float32)
        Z.flat[:: max(1, Z.size // 7)] = 90.0                      # saturated both ways
        Z.flat[1:: max(1, Z.size // 5)] = -90.0
        Y = (rng.random((n, C)) < 0.3).astype(np.uint8)
        mask = (rng.random(n) < 0.6).astype(np.uint8) if use_mask else None
        if mask is not None:
            mask[0] = 1
        Zd = H.padded_matrix(Z, ld)
        Yd = torch.zeros((n, ld + 3), dtype=torch.uint8, device="cuda")
        Yd[:, :C] = torch.from_numpy(Y).cuda()
        md = None if mask is None else torch.from_numpy(mask).cuda()
        dZd = torch.full((n, ld), 7.0, dtype=torch.float32 if dz == "f32" else torch.bfloat16, device="cuda")
        loss_d = torch.zeros(1, dtype=torch.float32, device="cuda")
        wsb = B.loss_workspace_bytes(n)
        ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
        B.sigmoid_bce(n, C, Zd, ld, Yd, ld + 3, md, norm, loss_d, dZd, ld, B.F32 if dz == "f32" else B.BF16, ws, wsb)
        torch.cuda.synchronize()
        want_loss, want_dZ = orc.sigmoid_bce(Z.astype(np.float64), Y.astype(np.float64), mask, norm)
        got = O.widen(H.dev_to_np(dZd))
        assert abs(loss_d.item() - want_loss) <= 1e-5 * max(1.0, abs(want_loss))
        assert O.normwise(got[:, :C], want_dZ) <= (1e-5 if dz == "f32" else 8e-3)
        assert (got[:, C:] == 7.0).all(), "padding columns were written"
        if mask is not None:
            assert (got[mask == 0][:, :C] == 0.0).all()


@pytest.mark.gpu
@pytest.mark.parametrize("kind,dtype", [("gin", "f32"), ("gcn", "f32"), ("sage", "f32"), ("gin", "bf16")])
def test_epoch_with_multilabel_loss_and_gin_layers(orc, kind, dtype):
    import torch
    from paper_2508_13716_amd import binding as B, harness as H
    from tests import oracle_side as O
    from tests.gpu_compare import compare_epoch, TOL
    env = dict(torch=torch, B=B, H=H, O=O, orc=orc)
    cfg = synth.Config(f"ML-{kind}-{dtype}", kind, 3000, 2500, 45_000, [96, 64, 24], dtype, 0.4, max_deg=400,
                       seed=synth.BASE_SEED * 10 + 8, extra={"loss": "bce", "gin_eps": 0.1})
    prob = H.make_problem(cfg, mask_frac=0.5)
    if kind == "gin":
        # a sum over up to 400 neighbours of N(0,1) rows: keep the activations O(1) so that the loss is not saturated
        for p in prob.model:
            p.W *= np.float32(0.125)
    assert prob.targets is not None and prob.targets.shape == (prob.part.n_loc, 24)
    for orders in (None, [B.AGG_FIRST, B.XFORM_FIRST]):
        dp = H.DeviceProblem(prob, orders=orders)
        ref = O.oracle_epoch(prob)
        for rep in range(2):
            loss, _ = dp.run_epoch()
            compare_epoch(env, prob, dp, ref, loss, TOL[dtype], f"{cfg.name} orders={orders} rep={rep}")
        dp.close()
