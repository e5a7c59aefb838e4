"""Test helper: runs the CPU oracle on a harness.Problem (the same host arrays the HIP path consumes)."""
import numpy as np

from oracle import oracle as orc
from paper_2508_13716_amd import synth


def widen(a: np.ndarray) -> np.ndarray:
    """float64 view of a float32 array or of a uint16 bf16 bit pattern (exact)."""
    if a.dtype == np.uint16:
        return synth.bf16_to_f32(a).reshape(a.shape).astype(np.float64)
    return a.astype(np.float64)


def oracle_graph(part, kind: str):
    if kind == "gcn":
        return orc.gcn_graph(part.n_loc, part.n_halo, part.rowptr, part.col, part.halo_degree)
    return orc.mean_graph(part.n_loc, part.n_halo, part.rowptr, part.col)


def oracle_epoch(prob, lr: float = 0.0, use_mask: bool = True, halo_grad: bool = False, relu_on=None):
    g = oracle_graph(prob.part, prob.cfg.kind)
    layers = [orc.Layer.of(p) for p in prob.model]
    tables = [widen(t) for t in prob.tables]
    return orc.epoch(g, layers, widen(prob.X0), tables, prob.labels, prob.mask if use_mask else None, 0.0, lr,
                     halo_grad=halo_grad, relu_on=relu_on)


def reconcile_relu_decisions(ref, gpu_hidden, band: float):
    """ReLU's backward factor 1[Z > 0] is an integer decided by a floating-point value.  Where the
    oracle's fp64 Z is zero within `band` (relative to max|Z| of the layer) the fp32 path may decide
    differently; there, and only there, the GPU's decision is adopted.  Elsewhere the two must agree.
    Returns (per-layer boolean arrays for oracle_epoch(relu_on=...), number of adopted decisions)."""
    out, adopted = [], 0
    for l, Z in enumerate(ref["hidden"]):
        if l >= len(gpu_hidden) or gpu_hidden[l] is None:
            out.append(None)
            continue
        on_ref = Z > 0.0
        on_gpu = widen(gpu_hidden[l]) > 0.0
        differ = on_ref != on_gpu
        tol = band * np.abs(Z).max()
        assert (np.abs(Z[differ]) <= tol).all(), f"layer {l}: ReLU decisions differ outside the rounding band"
        adopted += int(differ.sum())
        out.append(np.where(np.abs(Z) <= tol, on_gpu, on_ref))
    return out, adopted


def normwise(gpu: np.ndarray, ref: np.ndarray) -> float:
    """max|gpu - ref| / max|ref| (infinity-norm-wise relative error)."""
    ref = np.asarray(ref, np.float64)
    gpu = np.asarray(gpu, np.float64)
    den = np.abs(ref).max() if ref.size else 0.0
    if den == 0.0:
        return float(np.abs(gpu).max()) if gpu.size else 0.0
    return float(np.abs(gpu - ref).max() / den)
