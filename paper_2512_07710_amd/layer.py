"""Buffer management around the C-ABI calls: one MoE layer shape on one GPU.

`MoELayer` owns the output and intermediate device buffers (torch tensors used
as plain device memory) and issues the five library calls in order.  All
arithmetic happens inside libmoe355.
"""
from __future__ import annotations

from typing import Dict, Optional

import torch

from . import binding as B


class MoELayer:
    def __init__(self, T: int, d: int, E: int, k: int, F: int, device="cuda:0",
                 stream: Optional[torch.cuda.Stream] = None):
        self.T, self.d, self.E, self.k, self.F = T, d, E, k, F
        self.N = T * k
        self.device = torch.device(device)
        with torch.cuda.device(self.device):
            self.stream = stream if stream is not None else torch.cuda.current_stream()
            self.ctx = B.moe_create(T, d, E, k, F, self.stream)
            # a second stream (default priority) and an empty-batch context bound to it: the per-token quantisation does
            # not depend on the routing decision, so the whole-layer calls below run it beside the routing kernels
            self.side_stream = torch.cuda.Stream(device=self.device)
            self.side_ctx = B.moe_create(0, d, E, k, F, self.side_stream)
        # worth it only for large batches (measured: 0.2 ms off the 13.8 ms step at T = 32768, d = 7168; at T = 4096 and
        # below the two stream hand-overs cost more than the 0.03 ms the quantisation takes)
        self.overlap_quantize = T * d >= (1 << 26)
        dev, N = self.device, max(self.N, 1)
        self.topk_idx = torch.empty((T, k), dtype=torch.int32, device=dev)
        self.topk_w = torch.empty((T, k), dtype=torch.float32, device=dev)
        self.offsets = torch.empty((E + 1,), dtype=torch.int32, device=dev)
        self.perm = torch.empty((N,), dtype=torch.int32, device=dev)
        self.inv_perm = torch.empty((N,), dtype=torch.int32, device=dev)
        self.xq = torch.empty((N, d), dtype=torch.uint8, device=dev)
        self.xs = torch.empty((d // 128, N), dtype=torch.float32, device=dev)   # group-major scale planes
        self.xq_tok = torch.empty((max(T, 1), d), dtype=torch.uint8, device=dev)       # token order, quantised once
        self.xs_tok = torch.empty((d // 128, max(T, 1)), dtype=torch.float32, device=dev)
        self.y_perm = torch.empty((N, d), dtype=torch.float32, device=dev)
        self.y = torch.empty((T, d), dtype=torch.bfloat16, device=dev)

    def close(self):
        if getattr(self, "side_ctx", None):
            B.moe_destroy(self.side_ctx)
            self.side_ctx = None
        if getattr(self, "ctx", None):
            B.moe_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the five stages ------------------------------------------------------------
    def route(self, x, W_r, sel_bias=None):
        B.moe_route(self.ctx, x, W_r, sel_bias, self.k, self.topk_idx, self.topk_w, self.offsets, self.perm,
                    self.inv_perm)

    def route_replay(self, x, logged_idx, logged_w):
        B.moe_route_replay(self.ctx, x, logged_idx, logged_w, self.topk_idx, self.topk_w, self.offsets,
                           self.perm, self.inv_perm)

    def route_replay_ids(self, x, W_r, logged_idx):
        B.moe_route_replay_ids(self.ctx, x, W_r, logged_idx, self.topk_idx, self.topk_w, self.offsets, self.perm,
                               self.inv_perm)

    def quantize(self, x):
        B.moe_quantize_fp8(self.ctx, x, self.T, self.d, 128, self.inv_perm, self.k, self.xq, self.xs)

    def quantize_tokens(self, x):
        B.moe_quantize_fp8(self.ctx, x, self.T, self.d, 128, None, 1, self.xq_tok, self.xs_tok)

    def expert_ffn_gather(self, w: Dict[str, torch.Tensor]):
        B.moe_expert_ffn_fp8_gather(self.ctx, self.xq_tok, self.xs_tok, self.perm, self.offsets, w["W1q"], w["W3q"], w["W2q"],
                                    w["s1"], w["s3"], w["s2"], self.y_perm)

    def expert_ffn(self, w: Dict[str, torch.Tensor]):
        B.moe_expert_ffn_fp8(self.ctx, self.xq, self.xs, self.offsets, w["W1q"], w["W3q"], w["W2q"], w["s1"],
                             w["s3"], w["s2"], self.y_perm)

    def combine(self, y_f32=None):
        """y_f32 [T,d] f32 (optional): also receives the sums before the bf16 rounding."""
        B.moe_combine(self.ctx, self.y_perm, self.inv_perm, self.topk_w, self.y, y_f32)

    # ---- whole layer ----------------------------------------------------------------
    # `fused` = True: activations quantised once per token, gathered inside the gate/up GEMM;
    # False: the expert-ordered copy xq/xs is materialised first (same results bit for bit)
    def _ffn(self, x, w, fused):
        if fused:
            self.quantize_tokens(x)
            self.expert_ffn_gather(w)
        else:
            self.quantize(x)
            self.expert_ffn(w)
        self.combine()
        return self.y

    def _quantize_tokens_beside(self, x):
        """Token-order quantisation on the side stream; the caller's stream waits for it before the expert FFN."""
        self.side_stream.wait_stream(self.stream)           # x, and the previous step's readers of xq_tok / xs_tok
        B.moe_quantize_fp8(self.side_ctx, x, self.T, self.d, 128, None, 1, self.xq_tok, self.xs_tok)

    def _ffn_after_side(self, w):
        self.stream.wait_stream(self.side_stream)
        self.expert_ffn_gather(w)
        self.combine()
        return self.y

    def forward_routed(self, x, W_r, sel_bias, w, fused=True):
        if fused is True and self.overlap_quantize:
            self._quantize_tokens_beside(x)
            self.route(x, W_r, sel_bias)
            return self._ffn_after_side(w)
        self.route(x, W_r, sel_bias)
        return self._ffn(x, w, fused)

    def forward_replay(self, x, logged_idx, logged_w, w, fused=True):
        if fused is True and self.overlap_quantize:
            self._quantize_tokens_beside(x)
            self.route_replay(x, logged_idx, logged_w)
            return self._ffn_after_side(w)
        self.route_replay(x, logged_idx, logged_w)
        return self._ffn(x, w, fused)

    def hidden(self):
        """Copies of (hq [N,F] u8, hs [F/128,N] f32, group-major) written by the last expert_ffn call."""
        N, F = max(self.N, 1), self.F
        hq = torch.empty((N, F), dtype=torch.uint8, device=self.device)
        hs = torch.empty((F // 128, N), dtype=torch.float32, device=self.device)
        B.moe_debug_copy_hidden(self.ctx, hq, hs)
        torch.cuda.synchronize(self.device)
        return hq, hs
