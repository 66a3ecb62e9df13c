"""Sequencing of the three C-ABI calls over the layers of a model and over successive
verification steps (argument marshalling only; no arithmetic of the method lives here).

One step, for every layer: ems_verify_attention over the layer's caches; then once:
ems_greedy_accept on the step's logits; then ems_kv_append of the accepted rows into all
layers' caches, advancing the per-sample lengths in place on the device.  Nothing is copied
to the host between steps.
"""
from __future__ import annotations

import torch

from . import (ems_accept_workspace_bytes, ems_attention_workspace_bytes, ems_greedy_accept,
               ems_kv_append, ems_verify_attention, kv_cache)


class VerifyLoopRunner:
    def __init__(self, *, k_caches, v_caches, row_stride, head_stride, rows, kv_start, kv_len,
                 H, D, V, dtype, scale, max_k, max_kv_len, max_rows):
        dev = kv_start.device
        self.n_layers = len(k_caches)
        self.caches = [kv_cache(k, v, row_stride, head_stride, rows) for k, v in zip(k_caches, v_caches)]
        self._keep = (k_caches, v_caches)
        self.kv_start = kv_start
        self.kv_len = kv_len                      # advanced in place by every step
        self.B = kv_start.numel()
        self.H, self.D, self.V, self.scale = H, D, V, scale
        self.max_k, self.max_kv_len = max_k, max_kv_len
        self.out = [torch.empty((max_rows, H, D), dtype=dtype, device=dev) for _ in range(self.n_layers)]
        self.ws_attn = torch.empty(ems_attention_workspace_bytes(self.B, max_rows, H, D, max_kv_len),
                                   dtype=torch.uint8, device=dev)
        self.ws_acc = torch.empty(max(8, ems_accept_workspace_bytes(max_rows, V)), dtype=torch.uint8, device=dev)
        self.target = torch.empty(max_rows, dtype=torch.int32, device=dev)
        self.accepted = torch.empty(self.B, dtype=torch.int32, device=dev)
        self.accepted_cu = torch.empty(self.B + 1, dtype=torch.int32, device=dev)
        self.out_tokens = torch.empty(max_rows, dtype=torch.int32, device=dev)

    def step(self, q, k_new, v_new, cu_seqlens, logits, input_ids, target_ids=None):
        """q, k_new, v_new: per-layer lists of packed [T,H,D] tensors."""
        T = q[0].shape[0]
        for l in range(self.n_layers):
            ems_verify_attention(q[l], k_new[l], v_new[l], self.caches[l], cu_seqlens, self.kv_start,
                                 self.kv_len, self.out[l][:T], max_k=self.max_k,
                                 max_kv_len=self.max_kv_len, scale=self.scale, workspace=self.ws_attn)
        target = self.target[:T] if logits is not None else target_ids
        ems_greedy_accept(logits, target, input_ids, cu_seqlens, self.accepted, self.accepted_cu,
                          self.out_tokens[:max(T, 1)], workspace=self.ws_acc)
        ems_kv_append(k_new, v_new, self.caches, cu_seqlens, self.accepted, self.kv_start, self.kv_len,
                      self.kv_len)
