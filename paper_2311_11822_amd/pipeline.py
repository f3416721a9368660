"""Whole Book-Keeping path on one micro-batch: enqueues the library calls in order
(paper section 3: output gradient -> clipping factor -> parameter gradient -> noising).
Holds the buffers between calls; does no arithmetic of its own."""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import torch

from . import binding as dp


class BkPipeline:
    """layers: sequence of (a, g) device tensors, a [B,T,d_in], g [B,T,d_out]; bf16 tensors may be
    given as torch.bfloat16 or as int16/uint16 bit patterns, fp16 as torch.float16, fp32 as
    torch.float32."""

    def __init__(self, layers: Sequence[Tuple[torch.Tensor, torch.Tensor]], paths: Optional[List[int]] = None,
                 keep_instantiated: bool = True):
        a0 = layers[0][0]
        self.device = a0.device
        self.dt = {torch.float32: dp.DP_F32, torch.float16: dp.DP_F16}.get(a0.dtype, dp.DP_BF16)
        self.B = a0.shape[0]
        self.layers = list(layers)
        self.dims = [(a.shape[1], a.shape[2], g.shape[2]) for a, g in layers]
        self.paths = paths if paths is not None else [dp.dp_choose_path(T, d, p) for T, d, p in self.dims]
        self.desc = dp.layer_array([(a, g, T, d, p, path) for (a, g), (T, d, p), path
                                    in zip(self.layers, self.dims, self.paths)])
        L = len(layers)
        self.L = L
        self.psi = sum(d * p for _, d, p in self.dims)
        self.sqnorm = torch.zeros((L, self.B), dtype=torch.float32, device=self.device)
        self.C = torch.zeros(self.B, dtype=torch.float32, device=self.device)
        self.norm = torch.zeros(self.B, dtype=torch.float32, device=self.device)
        self.flat = torch.zeros(self.psi, dtype=torch.float32, device=self.device)
        self.grads, off = [], 0
        for _, d, p in self.dims:
            self.grads.append(self.flat[off:off + d * p].view(d, p))
            off += d * p
        self.grad_ptrs = (dp.C.c_void_p * L)(*[x.data_ptr() for x in self.grads])
        offs, acc = [], 0
        for _, d, p in self.dims:
            offs.append(acc)
            acc += d * p
        self.grad_offsets = (dp.C.c_uint64 * L)(*offs)
        ws_bytes = dp.dp_norms_multi_workspace_bytes(self.desc, self.dt, self.B)
        if ws_bytes == 0:
            raise dp.DpError(dp.DP_ERR_INVALID_ARG, "dp_norms_multi_workspace_bytes")
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=self.device)
        # Layers on the instantiated path keep their per-sample gradients [B, d, p] between the norm
        # pass and the gradient pass (smaller than the layer's Gram matrices by the path rule).
        self.kept = [None] * L
        if keep_instantiated and self.dt != dp.DP_F32:
            self.kept = [torch.empty((self.B, d, p), dtype=torch.float32, device=self.device)
                         if path == dp.DP_PATH_PEREX else None for (_, d, p), path in zip(self.dims, self.paths)]
        self.any_kept = any(k is not None for k in self.kept)
        self.kept_ptrs = (dp.C.c_void_p * L)(*[None if k is None else k.data_ptr() for k in self.kept])

    def norms(self, stream=None):
        if self.any_kept:
            dp.dp_norms_multi_keep(self.desc, self.dt, self.B, self.sqnorm, self.kept_ptrs, self.ws, stream)
        else:
            dp.dp_norms_multi(self.desc, self.dt, self.B, self.sqnorm, self.ws, stream)

    def clip(self, mode, R, stability=0.01, stream=None):
        dp.dp_clip_factors(self.sqnorm, self.L, self.B, mode, R, stability, self.C, self.norm, stream)

    def grad(self, accumulate=0, stream=None):
        if self.any_kept:
            dp.dp_clipped_grad_kept_multi(self.desc, self.dt, self.B, self.C, self.kept_ptrs, self.grad_ptrs, None,
                                          accumulate, 0, 0, 0.0, 1.0, 0, 0, stream)
        else:
            dp.dp_clipped_grad_multi(self.desc, self.dt, self.B, self.C, self.grad_ptrs, accumulate, stream)

    def grad_noise(self, sigma, R, seed, step, offset, count, accumulate=0, stream=None):
        """Gradients with the noise added in the same pass (elements [offset, offset + count) of
        the flattened gradient)."""
        if self.any_kept:
            dp.dp_clipped_grad_kept_multi(self.desc, self.dt, self.B, self.C, self.kept_ptrs, self.grad_ptrs,
                                          self.grad_offsets, accumulate, offset, count, sigma, R, seed, step, stream)
            return
        dp.dp_clipped_grad_noise_multi(self.desc, self.dt, self.B, self.C, self.grad_ptrs, self.grad_offsets,
                                       accumulate, offset, count, sigma, R, seed, step, stream)

    def noise(self, sigma, R, seed, step, offset, count, stream=None):
        dp.dp_add_noise(self.flat.data_ptr() + 4 * offset, offset, count, sigma, R, seed, step, stream)

    # group-wise clipping (eq. (1) of the paper with M groups; layer-wise = one group per layer)
    def set_groups(self, group_of_layer: Sequence[int], R: Sequence[float]):
        """Layers must be listed group by group (group_of_layer non-decreasing)."""
        M = len(R)
        assert list(group_of_layer) == sorted(group_of_layer) and max(group_of_layer) < M
        self.group_of_layer = list(group_of_layer)
        self.group_begin = [sum(1 for x in group_of_layer if x < m) for m in range(M + 1)]
        self.group_R = list(R)
        self.C_groups = torch.zeros((M, self.B), dtype=torch.float32, device=self.device)
        self.norm_groups = torch.zeros((M, self.B), dtype=torch.float32, device=self.device)

    def clip_grouped(self, mode, stability=0.01, stream=None):
        dp.dp_clip_factors_grouped(self.sqnorm, self.L, self.B, self.group_begin, self.group_R, mode, stability,
                                   self.C_groups, self.norm_groups, stream)

    def grad_grouped(self, accumulate=0, stream=None):
        dp.dp_clipped_grad_grouped(self.desc, self.dt, self.B, self.C_groups, self.group_of_layer,
                                   len(self.group_R), self.grad_ptrs, accumulate, stream)

    def noise_grouped(self, sigma, seed, step, offset, count, stream=None):
        self.noise(sigma, dp.dp_group_noise_threshold(self.group_R), seed, step, offset, count, stream)

    def layerwise_step(self, mode, stability, sigma, seed, step, offset, count, layers_per_pass=0,
                       accumulate=0, stream=None):
        """Layer-wise clipping (groups set with set_groups: one group per layer) without
        book-keeping: pass by pass norms -> factors -> gradients (+ noise), small layers in one kernel."""
        assert self.group_of_layer == list(range(self.L))
        if getattr(self, "ws_layerwise", None) is None:
            n = dp.dp_layerwise_workspace_bytes(self.desc, self.dt, self.B)
            if n == 0:
                raise dp.DpError(dp.DP_ERR_INVALID_ARG, "dp_layerwise_workspace_bytes")
            self.ws_layerwise = torch.empty(n, dtype=torch.uint8, device=self.device)
        dp.dp_layerwise_clipped_grad(self.desc, self.dt, self.B, self.group_R, mode, stability, self.grad_ptrs,
                                     self.grad_offsets, accumulate, offset, count, sigma, seed, step,
                                     self.sqnorm, self.C_groups, self.ws_layerwise, layers_per_pass, stream)

    def step(self, mode, R, sigma, stability, seed, step, offset, count, stream=None, fused=True):
        self.norms(stream)
        self.clip(mode, R, stability, stream)
        if fused:
            self.grad_noise(sigma, R, seed, step, offset, count, 0, stream)
        else:
            self.grad(0, stream)
            self.noise(sigma, R, seed, step, offset, count, stream)
