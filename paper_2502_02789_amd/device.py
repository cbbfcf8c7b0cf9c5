"""Device-memory plumbing around the binding: allocate outputs and workspaces with torch,
fill the argument structs, call the C entry points.  No arithmetic of the method happens here."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as sp


def bf16_from_bits(bits: np.ndarray, device="cuda") -> torch.Tensor:
    """numpy uint16 bit patterns -> torch.bfloat16 tensor on the device (bit-exact)."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.to(device).view(torch.bfloat16)


def bits_from_bf16(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


# The three configurations the paper compares (Sec. 4, list of evaluated variants), as settings
# of the same three calls: the plain variant scores with the last prompt token only and keeps
# single tokens by their un-smoothed scores; "full" adds pooling and chunk selection; "full_lah"
# adds the look-ahead queries.  (Window and chunk size are the synthetic workloads' choices.)
VARIANTS = {
    "raw": dict(n_queries=1, chunk=1, pool_window=1),
    "full": dict(n_queries=1, chunk=32, pool_window=13),
    "full_lah": dict(n_queries=8, chunk=32, pool_window=13),
}


class Scorer:
    """Holds the argument struct, outputs and workspace of one sp_score problem."""

    def __init__(self, q: torch.Tensor, k_layers: Sequence[torch.Tensor], cu_seqlens: torch.Tensor, *,
                 H_kv: int, scale: float, layer_reduce: int = sp.SP_LAYER_MAX,
                 n_valid: Optional[torch.Tensor] = None, want_lse: bool = False,
                 rope_theta: float = 0.0, q_pos: Optional[torch.Tensor] = None,
                 block_table: Optional[torch.Tensor] = None, page_size: int = 0, total_tokens: Optional[int] = None,
                 exclusive_device: bool = True, keep_workspace: bool = False, max_seqlen: int = 0,
                 k_scale: Optional[torch.Tensor] = None):
        """exclusive_device: promise that nothing else runs on the GPU during the call
        (SP_SCORE_EXCLUSIVE_DEVICE), which lets sp_score take its single-pass kernels.
        keep_workspace: from the second run() on, pass SP_SCORE_WORKSPACE_KEPT (this object owns
        its workspace, so the promise holds as long as run() is the only thing that writes it;
        anything else that does -- run(general=True), score_pool_select, a failed check() --
        makes the next run() start from a fresh workspace again)."""
        L, B, N, H, d = q.shape
        T = int(k_layers[0].shape[0]) if block_table is None else int(total_tokens)
        self.block_table = block_table
        dev = q.device
        self.q, self.k_layers, self.cu, self.n_valid, self.q_pos = q, list(k_layers), cu_seqlens, n_valid, q_pos
        self.scores = torch.empty(T, dtype=torch.float32, device=dev)
        self.lse = torch.empty((L, B, N, H), dtype=torch.float32, device=dev) if want_lse else None
        flags = sp.SP_SCORE_EXCLUSIVE_DEVICE if exclusive_device else 0
        probe = sp.make_score_args(q, self.k_layers, cu_seqlens, self.scores, H_kv=H_kv, scale=scale,
                                   layer_reduce=layer_reduce, n_valid=n_valid, lse=self.lse,
                                   rope_theta=rope_theta, q_pos=q_pos, T=T, block_table=block_table,
                                   page_size=page_size, flags=flags, max_seqlen=max_seqlen, k_scale=k_scale)
        need = sp.sp_score_workspace_bytes(probe)
        if need == 0:
            raise sp.SpError("sp_score_workspace_bytes", sp.SP_EINVAL)
        self.workspace = torch.empty(need, dtype=torch.uint8, device=dev)
        self.args = sp.make_score_args(q, self.k_layers, cu_seqlens, self.scores, H_kv=H_kv, scale=scale,
                                       layer_reduce=layer_reduce, n_valid=n_valid, lse=self.lse,
                                       workspace=self.workspace, rope_theta=rope_theta, q_pos=q_pos, T=T,
                                       block_table=block_table, page_size=page_size, flags=flags, max_seqlen=max_seqlen, k_scale=k_scale)

        self._base_flags, self._keep, self._kept = flags, keep_workspace, False

    def forget_workspace(self):
        """The workspace has been written by something other than sp_score."""
        self._kept = False

    def run(self, stream=None, general: bool = False) -> torch.Tensor:
        if general:
            self._kept = False
            sp.sp_score_general(self.args, stream)
            return self.scores
        self.args.flags = self._base_flags | (sp.SP_SCORE_WORKSPACE_KEPT if self._keep and self._kept else 0)
        sp.sp_score(self.args, stream)
        self._kept = True
        return self.scores

    def check(self, stream=None):
        """sp_score_check; raises SpError(SP_ETIMEOUT) if a bounded wait of the last run expired."""
        try:
            sp.sp_score_check(self.args, stream)
        except sp.SpError:
            self._kept = False
            raise


class Selector:
    """Outputs and workspace of one sp_pool_select (+ optional sp_gather) problem."""

    def __init__(self, scores: torch.Tensor, cu_seqlens: torch.Tensor, *, chunk: int, pool_window: int,
                 keep_rate: float, capacity: Optional[int] = None, want_chunk_scores: bool = False):
        dev = scores.device
        T = int(scores.numel())
        B = int(cu_seqlens.numel()) - 1
        cap = T if capacity is None else int(capacity)
        self.scores, self.cu = scores, cu_seqlens
        self.kept_idx = torch.full((max(cap, 1),), -1, dtype=torch.int32, device=dev)
        self.cu_keep = torch.zeros(B + 1, dtype=torch.int32, device=dev)
        self.chunk_scores = (torch.zeros(T // chunk + B, dtype=torch.float32, device=dev)
                             if want_chunk_scores else None)
        probe = sp.make_pool_select_args(scores, cu_seqlens, self.kept_idx, self.cu_keep, chunk=chunk,
                                         pool_window=pool_window, keep_rate=keep_rate, kept_capacity=cap)
        need = sp.sp_pool_select_workspace_bytes(probe)
        if need == 0:
            raise sp.SpError("sp_pool_select_workspace_bytes", sp.SP_EINVAL)
        self.workspace = torch.empty(need, dtype=torch.uint8, device=dev)
        self.args = sp.make_pool_select_args(scores, cu_seqlens, self.kept_idx, self.cu_keep, chunk=chunk,
                                             pool_window=pool_window, keep_rate=keep_rate,
                                             chunk_scores=self.chunk_scores, workspace=self.workspace,
                                             kept_capacity=cap)
        self.capacity = cap

    def run(self, stream=None):
        sp.sp_pool_select(self.args, stream)
        return self.kept_idx, self.cu_keep


def score_pool_select(scorer: Scorer, selector: Selector, stream=None):
    """One short prompt scored and selected in a single launch (sp_score_pool_select); the selector
    must have been built on scorer.scores and the same cu_seqlens."""
    scorer.forget_workspace()  # the logits pass through it
    sp.sp_score_pool_select(scorer.args, selector.args, stream)
    return scorer.scores, selector.kept_idx, selector.cu_keep


class Gatherer:
    def __init__(self, sel: Selector, *, token_ids: Optional[torch.Tensor] = None,
                 embed: Optional[torch.Tensor] = None):
        dev = sel.kept_idx.device
        cap = sel.capacity
        B = int(sel.cu.numel()) - 1
        self.kept_pos = torch.full((max(cap, 1),), -1, dtype=torch.int32, device=dev)
        self.kept_ids = torch.full((max(cap, 1),), -1, dtype=torch.int32, device=dev) if token_ids is not None else None
        self.decode_pos = torch.zeros(B, dtype=torch.int32, device=dev)
        self.out_embed = (torch.zeros((max(cap, 1), embed.shape[1]), dtype=torch.bfloat16, device=dev)
                          if embed is not None else None)
        self.token_ids, self.embed = token_ids, embed
        self.args = sp.make_gather_args(sel.cu, sel.cu_keep, sel.kept_idx, self.kept_pos, self.decode_pos,
                                        token_ids=token_ids, kept_ids=self.kept_ids, embed=embed,
                                        out_embed=self.out_embed, kept_capacity=cap)

    def run(self, stream=None):
        sp.sp_gather(self.args, stream)
        return self.kept_ids, self.kept_pos, self.decode_pos, self.out_embed
