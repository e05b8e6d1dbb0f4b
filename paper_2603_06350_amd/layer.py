"""Device buffers for one MoE layer and the four-call forward.

PyTorch is used for device memory and the stream handle only; the arithmetic is
in libmoe_gfx950.so.  `MoeBuffers` owns every output and scratch tensor of the
layer so that repeated forwards allocate nothing.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def to_device(a: np.ndarray, device="cuda"):
    """Host array from synth_inputs -> device tensor (uint16 bf16 bits become torch.bfloat16)."""
    if a is None:
        return None
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> host array (torch.bfloat16 comes back as uint16 bit patterns)."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


class MoeBuffers:
    def __init__(self, T, d, E, k, F, dtype, renorm, device="cuda", split_tiles=False):
        self.shape = B.make_shape(T, d, E, k, F, dtype, renorm)
        self.T, self.d, self.E, self.k, self.F = T, d, E, k, F
        tdt = torch.float32 if dtype == B.MOE_F32 else torch.bfloat16
        A = T * k
        kw = dict(device=device)
        self.topk_idx = torch.empty((T, k), dtype=torch.int32, **kw)
        self.topk_w = torch.empty((T, k), dtype=torch.float32, **kw)
        self.scores = torch.empty((T, E), dtype=torch.float32, **kw)
        self.counts = torch.empty((E,), dtype=torch.int32, **kw)
        self.offsets = torch.empty((E + 1,), dtype=torch.int32, **kw)
        self.dst_row = torch.empty((A,), dtype=torch.int32, **kw)
        self.src_assign = torch.empty((A,), dtype=torch.int32, **kw)
        self.x_perm = torch.empty((A, d), dtype=tdt, **kw)
        self.h = torch.empty((A, F), dtype=tdt, **kw)
        self.y_perm = torch.empty((A, d), dtype=tdt, **kw)
        self.y = torch.empty((T, d), dtype=tdt, **kw)
        self.ws_bytes = B.moe_workspace_bytes(self.shape)
        self.workspace = torch.empty((self.ws_bytes,), dtype=torch.uint8, **kw)
        # optional: the workspace that lets the grouped FFN cut the tiles of an under-filled last
        # round along K (moe_grouped_ffn_ws)
        self.ffn_ws_bytes = B.moe_ffn_workspace_bytes(self.shape) if split_tiles else 0
        self.ffn_ws = torch.empty((self.ffn_ws_bytes,), dtype=torch.uint8, **kw) if split_tiles else None

    def forward(self, x, w_gate, w1, w3, w2, gate_bias=None, stream=None, export_scores=False,
                gather_in_ffn=False, combine_in_ffn=False):
        """The whole hot path: route -> count+permute -> grouped FFN -> combine.
        gather_in_ffn: the up-projection reads x through the permutation map and x_perm is not
        materialised (same results, bit for bit).
        combine_in_ffn (k = 1 layers): the down-projection stores the weighted rows straight to y
        (moe_grouped_ffn_combine_k1); x_perm, y_perm and moe_combine are not used."""
        s = torch.cuda.current_stream() if stream is None else stream
        B.moe_route_ws(self.shape, x, w_gate, gate_bias, self.topk_idx, self.topk_w,
                       self.scores if export_scores else None, self.workspace, self.ws_bytes, s)
        B.moe_count_and_permute(self.shape, x, self.topk_idx, self.counts, self.offsets,
                                self.dst_row, self.src_assign,
                                None if (gather_in_ffn or combine_in_ffn) else self.x_perm,
                                self.workspace, self.ws_bytes, s)
        if combine_in_ffn:
            B.moe_grouped_ffn_combine_k1(self.shape, x, self.src_assign, self.offsets, w1, w3, w2,
                                         self.topk_w, self.h, self.y, s)
            return self.y
        if self.ffn_ws is not None:
            B.moe_grouped_ffn_ws(self.shape, x if gather_in_ffn else self.x_perm,
                                 self.src_assign if gather_in_ffn else None, self.offsets, w1, w3, w2,
                                 self.h, self.y_perm, 3, self.ffn_ws, self.ffn_ws_bytes, s)
        elif gather_in_ffn:
            B.moe_grouped_ffn_gather(self.shape, x, self.src_assign, self.offsets, w1, w3, w2,
                                     self.h, self.y_perm, s)
        else:
            B.moe_grouped_ffn(self.shape, self.x_perm, self.offsets, w1, w3, w2, self.h,
                              self.y_perm, s)
        B.moe_combine(self.shape, self.y_perm, self.dst_row, self.topk_w, self.y, s)
        return self.y


class LoadPredictor:
    """Speculative expert-load prediction for a later layer (paper, Section 4.1): the hidden states
    that enter layer l go through the gate of layer l+d (a replica of that gate, fine-tuned or
    not) to estimate that layer's per-expert token counts ahead of time, and Algorithm 1 turns the
    estimate into replica counts.  Everything is enqueued on one stream, meant to be a side stream
    next to the layer's own forward (Section 5: predictors run asynchronously on dedicated
    streams); nothing is read back to the host.

    enqueue() = moe_route (predictor weights) -> moe_count_and_permute without the row gather ->
    moe_scale_replicas -> moe_replica_segments.  Outputs stay in `counts`, `offsets`, `replicas`,
    `cv` ([before, after]), `seg_offsets`, `seg_expert`, `n_segments`."""

    def __init__(self, T, d, E, k, dtype, renorm, max_extra_replicas, n_gpus=0, device="cuda"):
        # F does not enter any of the calls used here; 8 keeps the shape valid for both dtypes
        self.shape = B.make_shape(T, d, E, k, 8, dtype, renorm)
        self.E = E
        self.max_extra = int(max_extra_replicas)
        A = T * k
        kw = dict(device=device)
        self.topk_idx = torch.empty((T, k), dtype=torch.int32, **kw)
        self.topk_w = torch.empty((T, k), dtype=torch.float32, **kw)
        self.counts = torch.empty((E,), dtype=torch.int32, **kw)
        self.offsets = torch.empty((E + 1,), dtype=torch.int32, **kw)
        self.dst_row = torch.empty((A,), dtype=torch.int32, **kw)
        self.src_assign = torch.empty((A,), dtype=torch.int32, **kw)
        self.ws_bytes = B.moe_workspace_bytes(self.shape)
        self.workspace = torch.empty((self.ws_bytes,), dtype=torch.uint8, **kw)
        self.replicas = torch.empty((E,), dtype=torch.int32, **kw)
        self.cv = torch.empty((2,), dtype=torch.float64, **kw)
        self.max_segments = E + self.max_extra
        self.seg_offsets = torch.empty((self.max_segments + 1,), dtype=torch.int32, **kw)
        self.seg_expert = torch.empty((self.max_segments,), dtype=torch.int32, **kw)
        self.n_segments = torch.empty((1,), dtype=torch.int32, **kw)
        # Algorithm 2 (optional): two sets of placement buffers, the previous round's is the warm set
        self.n_gpus = int(n_gpus)
        self.round = 0
        if self.n_gpus > 0:
            self.gpu_of = [torch.full((self.max_segments,), -1, dtype=torch.int32, **kw) for _ in range(2)]
            self.placed_replicas = [torch.zeros((E,), dtype=torch.int32, **kw) for _ in range(2)]
            self.gpu_load = torch.empty((self.n_gpus,), dtype=torch.float64, **kw)
            self.gpu_count = torch.empty((self.n_gpus,), dtype=torch.int32, **kw)
            self.n_warm = torch.empty((1,), dtype=torch.int32, **kw)

    def enqueue(self, x, w_pred, gate_bias=None, cv_threshold=0.2, stream=None):
        s = torch.cuda.current_stream() if stream is None else stream
        B.moe_route_ws(self.shape, x, w_pred, gate_bias, self.topk_idx, self.topk_w, None,
                       self.workspace, self.ws_bytes, s)
        B.moe_count_and_permute(self.shape, None, self.topk_idx, self.counts, self.offsets,
                                self.dst_row, self.src_assign, None, self.workspace, self.ws_bytes, s)
        # memory in units of one expert: the cap is the number of additional replicas
        B.moe_scale_replicas(self.E, self.counts, 1, self.max_extra, cv_threshold, self.replicas,
                             self.cv, s)
        B.moe_replica_segments(self.E, self.offsets, self.replicas, self.max_segments,
                               self.seg_offsets, self.seg_expert, self.n_segments, s)
        if self.n_gpus > 0:
            cur, prev = self.round & 1, (self.round & 1) ^ 1
            with torch.cuda.stream(s):          # keep these replica counts: the next call's warm set
                self.placed_replicas[cur].copy_(self.replicas, non_blocking=True)
            B.moe_place_replicas(self.E, self.counts, self.replicas, self.n_gpus,
                                 self.placed_replicas[prev] if self.round > 0 else None,
                                 self.gpu_of[prev] if self.round > 0 else None, None,
                                 self.max_segments, self.gpu_of[cur], self.gpu_load, self.gpu_count,
                                 self.n_warm, s)
            self.round += 1


def predicted_vs_actual_loads(pred: LoadPredictor, x_now, x_later, w_pred, gate_bias=None, stream=None):
    """How well the loads predicted from the current hidden states match those the same gate sees
    one layer later (paper, Section 4.1 and its accuracy study): both passes are the library's
    routing and counting; the comparison of the two small count vectors is host arithmetic.
    Returns (predicted counts, actual counts, fraction of (token, slot) choices that the later
    routing also makes for that token)."""
    s = torch.cuda.current_stream() if stream is None else stream
    pred.enqueue(x_now, w_pred, gate_bias, stream=s)
    with torch.cuda.stream(s):
        c_pred = pred.counts.clone()
        idx_pred = pred.topk_idx.clone()
    pred.enqueue(x_later, w_pred, gate_bias, stream=s)
    with torch.cuda.stream(s):
        same = (idx_pred.unsqueeze(2) == pred.topk_idx.unsqueeze(1)).any(dim=2).float().mean()
    s.synchronize()
    return c_pred.cpu().numpy(), pred.counts.cpu().numpy(), float(same.item())
