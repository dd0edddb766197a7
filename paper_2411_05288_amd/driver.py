"""Host driver: runs the p shards of one configuration in sequence on one GPU.

This is launch ordering and buffer ownership only.  It follows Algorithm 1 of the paper:
pass S on every shard (vp_output_fwd), barrier C1 (vp_combine_stats, standing in for the two
all-reduces), pass T on every shard (vp_output_bwd) with the reduce C2 realised as fp32
accumulation into one dH buffer in ascending shard order.  With algorithm=2 it follows
Algorithm 2: pass S also forms A and B (vp_output_fwd_alg2), the input gradient is
accumulated inside the single barrier (vp_output_dx_alg2), and pass T is dW alone.  All device buffers are allocated
once, when the plan is built; a step allocates nothing.
"""
from __future__ import annotations

import contextlib
from dataclasses import dataclass
from typing import List, Optional

import torch

from . import binding as B


@dataclass
class OutputLayerResult:
    loss: torch.Tensor            # [1] fp32
    loss_rows: torch.Tensor       # [N] fp32
    global_max: torch.Tensor      # [N]
    global_sumexp: torch.Tensor   # [N]
    local_max: torch.Tensor       # [p, N]
    local_sumexp: torch.Tensor    # [p, N]
    local_target: torch.Tensor    # [p, N]
    dH: torch.Tensor              # [N, h] fp32
    dW: List[torch.Tensor]        # p x [Vs, h] fp32
    logits: Optional[List[torch.Tensor]]


class OutputLayerPlan:
    """Buffers and launch order for one output-layer workload of p shards.

    Shards may have different numbers of rows (a short last shard); shard r owns the global
    vocabulary rows [offsets[r], offsets[r] + rows_r).  ``vocab_size`` states the true
    vocabulary when the table was padded to split evenly (the paper pads V to a multiple of
    2p): rows at or beyond it are padding.  Padding never reaches the kernels -- a shard is
    passed as its valid prefix, which is the same as giving the padded logits -inf -- and
    the padding rows of dW are zero."""

    def __init__(self, H: torch.Tensor, W_shards: List[torch.Tensor], labels: torch.Tensor,
                 save_logits: bool = True, grad_scale: Optional[float] = None, vocab_size: Optional[int] = None,
                 algorithm: int = 1):
        if algorithm not in (1, 2):
            raise B.VPError("algorithm must be 1 (two barriers) or 2 (one barrier)")
        self.algorithm = algorithm
        self.H, self.W, self.labels = H, W_shards, labels
        self.N, self.h = H.shape
        self.p = len(W_shards)
        self.rows = [int(w.shape[0]) for w in W_shards]
        self.Vs = self.rows[0]
        for w in W_shards:
            if w.dim() != 2 or w.shape[1] != self.h:
                raise B.VPError("every shard must be [rows, h]")
        self.offsets = [0]
        for n in self.rows[:-1]:
            self.offsets.append(self.offsets[-1] + n)
        total = self.offsets[-1] + self.rows[-1]
        self.vocab_size = total if vocab_size is None else int(vocab_size)
        if not 0 < self.vocab_size <= total:
            raise B.VPError("vocab_size must be in (0, total rows]")
        # valid (non-padding) rows of every shard
        self.valid = [max(0, min(n, self.vocab_size - off)) for n, off in zip(self.rows, self.offsets)]
        self.dt = B.VP_F32 if H.dtype == torch.float32 else B.VP_BF16
        self.save_logits = save_logits
        self.grad_scale = (1.0 / self.N) if grad_scale is None else float(grad_scale)
        dev = H.device
        f32 = dict(dtype=torch.float32, device=dev)
        N, h, p = self.N, self.h, self.p
        self.local_max = torch.empty((p, N), **f32)
        self.local_sumexp = torch.empty((p, N), **f32)
        self.local_target = torch.empty((p, N), **f32)
        self.global_max = torch.empty((N,), **f32)
        self.global_sumexp = torch.empty((N,), **f32)
        self.loss_rows = torch.empty((N,), **f32)
        self.loss = torch.empty((1,), **f32)
        self.dH = torch.empty((N, h), **f32)
        self.dW = [torch.empty((n, h), **f32) for n in self.rows]
        self.logits = ([torch.empty((N, max(v, 1)), dtype=H.dtype, device=dev) for v in self.valid]
                       if save_logits else None)
        flags = B.VP_SAVE_LOGITS if save_logits else 0
        fwd_call = B.VP_CALL_OUTPUT_FWD if algorithm == 1 else B.VP_CALL_OUTPUT_FWD_ALG2
        nbytes = 256
        for v in self.valid:
            if v > 0:
                nbytes = max(nbytes, B.vp_workspace_bytes(fwd_call, N, h, v, self.dt, flags),
                             B.vp_workspace_bytes(B.VP_CALL_OUTPUT_BWD, N, h, v, self.dt, flags))
        # Algorithm 2 keeps A = softmax' W_r and B = G W_r of every shard until the barrier
        self.A = [torch.empty((N, h), **f32) for _ in range(p)] if algorithm == 2 else None
        self.Bm = [torch.empty((N, h), dtype=H.dtype, device=dev) for _ in range(p)] if algorithm == 2 else None
        self.workspace = torch.empty((nbytes,), dtype=torch.uint8, device=dev)

    def _on(self, stream):
        """Context in which torch-side fills run on the same stream as the library's kernels."""
        if stream is None:
            return contextlib.nullcontext()
        if not isinstance(stream, torch.cuda.Stream):
            stream = torch.cuda.ExternalStream(int(stream))
        return torch.cuda.stream(stream)

    def forward(self, stream=None) -> None:
        for r in range(self.p):
            v = self.valid[r]
            if v == 0:     # all padding: the neutral element of the combine (exp(-inf) = 0)
                with self._on(stream):
                    self.local_max[r].fill_(float("-inf"))
                    self.local_sumexp[r].zero_()
                    self.local_target[r].zero_()
                continue
            lg = self.logits[r] if self.logits is not None else None
            if self.algorithm == 1:
                B.vp_output_fwd(self.H, self.W[r][:v], self.labels, self.offsets[r],
                                self.local_max[r], self.local_sumexp[r], self.local_target[r],
                                lg, self.workspace, stream)
            else:
                B.vp_output_fwd_alg2(self.H, self.W[r][:v], self.labels, self.offsets[r],
                                     self.local_max[r], self.local_sumexp[r], self.local_target[r],
                                     self.A[r], self.Bm[r], lg, self.workspace, stream)
        B.vp_combine_stats(self.local_max, self.local_sumexp, self.local_target,
                           self.global_max, self.global_sumexp, self.loss_rows, self.loss, stream)
        if self.algorithm == 2:
            # still inside the one barrier of Algorithm 2: the input gradient leaves here; the first shard
            # that contributes overwrites dH, so nothing is zero-filled
            first = True
            for r in range(self.p):
                if self.valid[r] > 0:
                    B.vp_output_dx_alg2(self.A[r], self.Bm[r], self.local_max[r], self.local_sumexp[r],
                                        self.global_max, self.global_sumexp, self.grad_scale, self.dH, stream,
                                        dh_overwrite=first)
                    first = False
            if first:      # no shard holds a real vocabulary row (cannot happen: vocab_size > 0)
                with self._on(stream):
                    self.dH.zero_()

    def backward(self, stream=None) -> None:
        first = True      # the first shard that contributes overwrites dH (Algorithm 1): no zero-fill
        for r in range(self.p):
            v = self.valid[r]
            if v < self.rows[r]:
                with self._on(stream):
                    self.dW[r][v:].zero_()
            if v == 0:
                continue
            B.vp_output_bwd(self.H, self.W[r][:v], self.labels, self.offsets[r], self.global_max, self.global_sumexp,
                            self.logits[r] if self.logits is not None else None, self.grad_scale,
                            self.dH if self.algorithm == 1 else None, self.dW[r][:v], self.workspace, stream,
                            dh_overwrite=first)
            first = False

    def step(self, stream=None) -> None:
        self.forward(stream)
        self.backward(stream)

    def result(self) -> OutputLayerResult:
        return OutputLayerResult(self.loss, self.loss_rows, self.global_max, self.global_sumexp,
                                 self.local_max, self.local_sumexp, self.local_target,
                                 self.dH, self.dW, self.logits)


def output_layer_step(H, W_shards, labels, save_logits=True, grad_scale=None, vocab_size=None) -> OutputLayerResult:
    """One forward + backward of the sharded output layer; returns all outputs."""
    plan = OutputLayerPlan(H, W_shards, labels, save_logits, grad_scale, vocab_size)
    plan.step()
    return plan.result()


class EmbeddingPlan:
    """Buffers and launch order for the sharded input layer (appendix C)."""

    def __init__(self, table_shards: List[torch.Tensor], ids: torch.Tensor, grad_out: Optional[torch.Tensor]):
        self.tables, self.ids, self.grad_out = table_shards, ids, grad_out
        self.p = len(table_shards)
        self.Vs, self.h = table_shards[0].shape
        self.N = ids.shape[0]
        dev = ids.device
        self.dt = B.VP_F32 if table_shards[0].dtype == torch.float32 else B.VP_BF16
        self.out = [torch.empty((self.N, self.h), dtype=table_shards[0].dtype, device=dev) for _ in range(self.p)]
        self.dtable = [torch.zeros((self.Vs, self.h), dtype=torch.float32, device=dev) for _ in range(self.p)]
        nbytes = max(B.vp_workspace_bytes(B.VP_CALL_EMBED_BWD, self.N, self.h, self.Vs, self.dt, 0), 256)
        self.workspace = torch.empty((nbytes,), dtype=torch.uint8, device=dev)

    def forward(self, stream=None) -> None:
        for r in range(self.p):
            B.vp_embed_fwd(self.tables[r], self.ids, r * self.Vs, self.out[r], stream)

    def backward(self, stream=None) -> None:
        for r in range(self.p):
            B.vp_embed_bwd(self.grad_out, self.ids, r * self.Vs, self.dtable[r], self.workspace, stream)


def embedding_forward(table_shards, ids):
    plan = EmbeddingPlan(table_shards, ids, None)
    plan.forward()
    return plan.out


def embedding_backward(grad_out, ids, Vs: int, p: int, dtable: Optional[List[torch.Tensor]] = None):
    """Scatter-add into (optionally supplied, accumulate-into) fp32 shard gradients."""
    N, h = grad_out.shape
    dev = grad_out.device
    if dtable is None:
        dtable = [torch.zeros((Vs, h), dtype=torch.float32, device=dev) for _ in range(p)]
    dt = B.VP_F32 if grad_out.dtype == torch.float32 else B.VP_BF16
    nbytes = max(B.vp_workspace_bytes(B.VP_CALL_EMBED_BWD, N, h, Vs, dt, 0), 256)
    ws = torch.empty((nbytes,), dtype=torch.uint8, device=dev)
    for r in range(p):
        B.vp_embed_bwd(grad_out, ids, r * Vs, dtable[r], ws)
    return dtable
