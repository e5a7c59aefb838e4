"""Host-side harness: turns a synthetic problem into device buffers and library handles.

Marshalling only.  torch allocates device / pinned memory and creates the two HIP streams; all
computation happens in libcapgnn through ``binding``.  Used by the GPU tests, ``bench.py`` and the
smoke check.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional

import numpy as np

from . import binding as B
from . import synth


@dataclass
class Problem:
    """Everything one epoch consumes, as host arrays (shared verbatim with the CPU oracle)."""
    cfg: synth.Config
    part: synth.Partition
    X0: np.ndarray                     # [n_loc, F0]  float32, or uint16 bf16 bits
    tables: List[np.ndarray]           # per layer l: [n_halo, dims[l]] same dtype as X0
    model: List[synth.LayerParams]
    labels: np.ndarray                 # int32 [n_loc]
    mask: np.ndarray                   # uint8 [n_loc]
    cap_gpu: int
    targets: Optional[np.ndarray] = None   # uint8 [n_loc, classes]: multi-label task (binary cross-entropy)


def make_problem(cfg: synth.Config, mask_frac: float = 1.0, part: Optional[synth.Partition] = None) -> Problem:
    part = part if part is not None else synth.partition_for(cfg)
    L = len(cfg.dims) - 1
    X0 = synth.make_features(part.n_loc, cfg.dims[0], seed=cfg.seed, stream=10, dtype=cfg.dtype)
    tables = [synth.make_features(part.n_halo, cfg.dims[l], seed=cfg.seed, stream=20 + l, dtype=cfg.dtype)
              for l in range(L)]
    model = synth.make_model(cfg.kind, cfg.dims, seed=cfg.seed, dtype=cfg.dtype)
    labels, mask = synth.make_labels(part.n_loc, cfg.dims[-1], seed=cfg.seed, mask_frac=mask_frac)
    targets = None
    if cfg.extra.get("loss") == "bce":
        targets = synth.make_multilabels(part.n_loc, cfg.dims[-1], seed=cfg.seed)
    return Problem(cfg, part, X0, tables, model, labels, mask, synth.cap_gpu_for(cfg, part), targets)


def relabel_problem(prob: Problem, method: int):
    """The same problem with its vertices stored in the library's locality order.  Returns (problem, new2old);
    per-vertex rows of the result k correspond to old rows new2old[k]."""
    import dataclasses
    part = prob.part
    nl = part.n_loc
    new2old = B.locality_order(method, nl, part.n_halo, part.rowptr, part.col)
    rowptr, col, _ = B.relabel_csr(nl, part.n_halo, part.rowptr, part.col, new2old)
    pl, ph = new2old[:nl].astype(np.int64), new2old[nl:].astype(np.int64) - nl
    part2 = dataclasses.replace(part, name=part.name + "-relabelled", rowptr=rowptr, col=col,
                                halo_gid=part.halo_gid[ph], halo_prio=part.halo_prio[ph],
                                halo_degree=part.halo_degree[ph])
    prob2 = dataclasses.replace(prob, part=part2, X0=prob.X0[pl], tables=[t[ph] for t in prob.tables],
                                labels=prob.labels[pl], mask=prob.mask[pl])
    return prob2, new2old


def _torch():
    import torch
    return torch


def np_to_dev(a: np.ndarray):
    """numpy -> device tensor; uint16 arrays (bf16 bit patterns) become torch.bfloat16."""
    torch = _torch()
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def dev_to_np(t) -> np.ndarray:
    """device tensor -> numpy; bf16 comes back as its uint16 bit pattern."""
    torch = _torch()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def padded_matrix(a: np.ndarray, ld: int, rows: Optional[int] = None):
    """Device buffer [rows, ld] whose top-left corner holds `a`; the rest is zero."""
    torch = _torch()
    rows = a.shape[0] if rows is None else rows
    if a.dtype == np.uint16:
        buf = torch.zeros((rows, ld), dtype=torch.bfloat16, device="cuda")
    else:
        buf = torch.zeros((rows, ld), dtype=torch.from_numpy(a[:0]).dtype, device="cuda")
    if a.size:
        buf[: a.shape[0], : a.shape[1]] = np_to_dev(a)
    return buf


class DeviceProblem:
    """Library handles + device buffers for one Problem."""

    def __init__(self, prob: Problem, orders: Optional[List[int]] = None, miss_mode: int = B.MISS_STAGED,
                 map_kind: int = B.MAP_DIRECT, use_side_stream: bool = True, f32_product: int = B.F32_PRODUCT_AUTO):
        torch = _torch()
        self.prob = prob
        self.miss_mode = miss_mode
        cfg, part = prob.cfg, prob.part
        self.dtype = B.BF16 if cfg.dtype == "bf16" else B.F32
        self.es = 2 if self.dtype == B.BF16 else 4
        self.tdtype = torch.bfloat16 if self.dtype == B.BF16 else torch.float32
        L = len(prob.model)
        self.L = L
        self.stream = torch.cuda.Stream()
        self.side = torch.cuda.Stream() if (use_side_stream and part.n_halo > 0) else None

        if cfg.kind == "gin":
            rp, cl, vl = B.gin_operator(part.n_loc, part.n_halo, part.rowptr, part.col, float(cfg.extra.get("gin_eps", 0.0)))
            self.graph = B.Graph(part.n_loc, part.n_halo, rp, cl, None, None, vl, 0)
        else:
            kind = B.NORM_SYM if cfg.kind == "gcn" else B.NORM_MEAN
            r, c = B.norm_scales(kind, part.n_loc, part.n_halo, part.rowptr, part.halo_degree)
            flags = B.GRAPH_SYMMETRIC if part.symmetric else 0
            self.graph = B.Graph(part.n_loc, part.n_halo, part.rowptr, part.col, r, c, None, flags)

        self.cache = None
        if part.n_halo > 0:
            self.cache = B.Cache(part.halo_gid, part.halo_prio, prob.cap_gpu, cfg.dims[:L], self.dtype, map_kind)
            for l in range(L):
                self.cache.fill(l, prob.tables[l])
            self.cache.set_miss_mode(miss_mode)

        # input rows start on cache-line boundaries: a 32-float step of a product then reads one line per row, and the
        # halo gather writes whole lines
        self.ld0 = synth.pad_to(cfg.dims[0], 128 // self.es)
        self.X0 = padded_matrix(prob.X0, self.ld0, rows=part.n_cols)

        self.W, self.W_self, self.bias = [], [], []
        self.dW, self.dW_self, self.dbias = [], [], []
        self.layers: List[B.Layer] = []
        for l, p in enumerate(prob.model):
            if self.dtype == B.BF16:
                W = np_to_dev(synth.f32_to_bf16_rne(p.W).reshape(p.W.shape))
                Ws = np_to_dev(synth.f32_to_bf16_rne(p.W_self).reshape(p.W.shape)) if p.W_self is not None else None
            else:
                W = np_to_dev(p.W)
                Ws = np_to_dev(p.W_self) if p.W_self is not None else None
            b = np_to_dev(p.bias)
            self.W.append(W); self.W_self.append(Ws); self.bias.append(b)
            self.dW.append(torch.zeros(p.W.shape, dtype=torch.float32, device="cuda"))
            self.dW_self.append(torch.zeros(p.W.shape, dtype=torch.float32, device="cuda") if Ws is not None else None)
            self.dbias.append(torch.zeros(p.f_out, dtype=torch.float32, device="cuda"))
            order = B.ORDER_AUTO if orders is None else orders[l]
            self.layers.append(B.make_layer(B.SAGE_MEAN if p.kind == "sage" else B.GCN, p.f_in, p.f_out,
                                            B.ACT_RELU if p.act == "relu" else B.ACT_NONE, self.dtype, W, Ws, b, order,
                                            out_f32=1 if (l == L - 1 and self.dtype == B.BF16) else 0,
                                            f32_product=f32_product))
        self.labels = torch.from_numpy(prob.labels).cuda()
        self.mask = torch.from_numpy(prob.mask).cuda()
        self.targets = None if prob.targets is None else torch.from_numpy(np.ascontiguousarray(prob.targets)).cuda()
        self.logits = torch.zeros((part.n_loc, cfg.dims[-1]), dtype=torch.float32, device="cuda")
        self.ws_bytes = B.epoch_workspace_bytes(self.graph, self.cache, self.layers)
        if self.ws_bytes == 0:
            raise B.CapgnnError(B.EINVAL, B.last_error())
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()

    def resolved_orders(self) -> List[int]:
        return [B.layer_order(self.graph, l, i > 0) for i, l in enumerate(self.layers)]

    def run_epoch(self, lr: float = 0.0, want_loss: bool = True, want_times: bool = False, mask=True):
        return B.epoch(self.graph, self.cache, self.layers, self.X0, self.ld0, self.labels,
                       self.mask if mask else None, 0.0, self.logits, self.dW,
                       self.dW_self if any(t is not None for t in self.dW_self) else None, self.dbias, lr,
                       self.ws, self.ws_bytes, self.stream, self.side, want_loss=want_loss, want_times=want_times,
                       targets=self.targets, ldt=0 if self.targets is None else self.targets.shape[1])

    def capture_epoch(self, lr: float = 0.0, mask=True, two_streams: bool = False):
        """The epoch as a HIP graph on this problem's buffers; returns (graph, device float the replays write the loss to).
        two_streams: record the epoch with its side stream (in pipelined mode one eager epoch must have run before)."""
        torch = _torch()
        if self.targets is not None:
            raise ValueError("the recorded epoch takes class labels")
        loss_dev = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        eg = B.EpochGraph(self.graph, self.cache, self.layers, self.X0, self.ld0, self.labels, self.mask if mask else None, 0.0,
                          self.logits, self.dW, self.dW_self if any(t is not None for t in self.dW_self) else None, self.dbias,
                          lr, loss_dev, self.ws, self.ws_bytes, self.stream, self.side if two_streams else None)
        return eg, loss_dev

    def hidden(self, l: int) -> np.ndarray:
        """Output of hidden layer l after the last epoch, [n_loc, f_out(l)] (bf16 as uint16 bits)."""
        torch = _torch()
        torch.cuda.synchronize()
        ptr, ld = B.epoch_activation(self.graph, self.cache, self.layers, l, self.ws)
        off = ptr - self.ws.data_ptr()
        n_loc, f = self.prob.part.n_loc, self.prob.model[l].f_out
        raw = self.ws[off: off + n_loc * ld * self.es].view(self.tdtype).view(n_loc, ld)
        return dev_to_np(raw[:, :f].contiguous())

    def results(self) -> Dict:
        _torch().cuda.synchronize()
        return {"logits": dev_to_np(self.logits),
                "dW": [dev_to_np(t) for t in self.dW],
                "dW_self": [None if t is None else dev_to_np(t) for t in self.dW_self],
                "db": [dev_to_np(t) for t in self.dbias]}

    def close(self):
        _torch().cuda.synchronize()     # a pipelined epoch may have left a prefetch into the workspace in flight
        if self.cache is not None:
            self.cache.close()
        self.graph.close()
