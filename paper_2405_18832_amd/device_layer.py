"""Device-side buffers of one MoE FFN layer: allocation, host->HBM upload, one-time weight
packing, and calls into the C ABI.  No arithmetic happens here.

Used by the tests, the smoke check and the bench.  Inputs arrive as numpy float32 arrays whose
values are already representable in the layer's storage dtype.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import Callable, Iterable, Optional

import numpy as np
import torch

from . import (make_shape, moe_combine, moe_expert_ffn, moe_expert_ffn_biased, moe_layer_forward,
               moe_layer_forward_biased, moe_pack_weights,
               moe_permute, moe_route, moe_workspace_bytes)


def torch_dtype(dtype: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


def to_device(a: np.ndarray, dtype: str, device) -> torch.Tensor:
    """Exact conversion: the values are representable in `dtype` already."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch_dtype(dtype)).to(device)


class DeviceLayer:
    def __init__(self, cfg, x: np.ndarray, w_gate: np.ndarray, b_gate: Optional[np.ndarray],
                 expert: Callable[[int], tuple], experts: Optional[Iterable[int]] = None,
                 device: str = "cuda:0", workers: int = 8, biases: Optional[tuple] = None):
        """cfg needs T, d_model, d_ff, E, k, dtype ("f32"|"bf16"), renormalize.
        `expert(e)` returns (W1_e [d_ff, d_model], W2_e [d_model, d_ff]).  If `experts` is
        given, only those experts get their real weights; the others are filled with
        device-generated normal noise of the same scale (used when only a known subset can
        receive tokens and generating all weights on the host would take minutes).
        `biases` = (b1 [E, d_ff], b2 [E, d_model]) float32 arrays for experts with biases."""
        self.cfg = cfg
        self.device = torch.device(device)
        act = {"relu": 0, "gelu": 1}[getattr(cfg, "activation", "relu")]
        self.shape = make_shape(cfg.T, cfg.d_model, cfg.d_ff, cfg.E, cfg.k, cfg.dtype, cfg.renormalize, act)
        td = torch_dtype(cfg.dtype)
        self.dtype = td
        T, d, f, E, k = cfg.T, cfg.d_model, cfg.d_ff, cfg.E, cfg.k
        A = T * k
        dev = self.device
        self.x = to_device(x, cfg.dtype, dev)
        self.w_gate = to_device(w_gate, cfg.dtype, dev)
        self.b_gate = None if b_gate is None else torch.from_numpy(
            np.ascontiguousarray(b_gate, dtype=np.float32)).to(dev)

        # packed expert weights [E, f*d]; `copies` > 1 keeps identical clones that a timing loop can
        # rotate through so that no step finds its weights in the last-level cache
        self.w1 = torch.empty((E, f * d), dtype=td, device=dev)
        self.w2 = torch.empty((E, d * f), dtype=td, device=dev)
        self._one = make_shape(cfg.T, cfg.d_model, cfg.d_ff, 1, 1, cfg.dtype, cfg.renormalize)
        want = list(range(E)) if experts is None else sorted(set(int(e) for e in experts))
        if len(want) < E:
            gen = torch.Generator(device=dev).manual_seed(12345)
            for e in range(E):      # per expert: keeps the fp32 temporary small
                self.w1[e] = (torch.randn((f * d,), device=dev, generator=gen) / d ** 0.5).to(td)
                self.w2[e] = (torch.randn((d * f,), device=dev, generator=gen) / f ** 0.5).to(td)
        self.upload_experts(expert, want, workers)
        self.weight_copies = [(self.w1, self.w2)]
        self.b1 = self.b2 = None
        if biases is not None:
            self.b1 = torch.from_numpy(np.ascontiguousarray(biases[0], dtype=np.float32)).to(dev)
            self.b2 = torch.from_numpy(np.ascontiguousarray(biases[1], dtype=np.float32)).to(dev)

        self.ws = torch.empty(max(256, moe_workspace_bytes(self.shape)), dtype=torch.uint8, device=dev)
        i32, f32 = torch.int32, torch.float32
        self.topk_idx = torch.empty((T, k), dtype=i32, device=dev)
        self.topk_w = torch.empty((T, k), dtype=f32, device=dev)
        self.margin = torch.empty((T,), dtype=f32, device=dev)
        self.counts = torch.empty((E,), dtype=i32, device=dev)
        self.offsets = torch.empty((E + 1,), dtype=i32, device=dev)
        self.hot_mask = torch.empty((E,), dtype=torch.uint8, device=dev)
        self.perm = torch.empty((A,), dtype=i32, device=dev)
        self.inv_perm = torch.empty((A,), dtype=i32, device=dev)
        self.x_perm = torch.empty((A, d), dtype=td, device=dev)
        self.y_perm = torch.empty((A, d), dtype=f32, device=dev)
        self.out = torch.empty((T, d), dtype=td, device=dev)

    def upload_experts(self, expert, experts, workers: int = 8) -> None:
        """Host -> HBM copy and packing of the given experts' weights (one expert at a time)."""
        cfg, dev, td = self.cfg, self.device, self.dtype
        experts = list(experts)
        if not experts:
            return
        s1 = torch.empty((cfg.d_ff, cfg.d_model), dtype=td, device=dev)
        s2 = torch.empty((cfg.d_model, cfg.d_ff), dtype=td, device=dev)
        with ThreadPoolExecutor(max_workers=max(1, workers)) as pool:
            for i in range(0, len(experts), workers):
                es = experts[i:i + workers]
                for e, (w1, w2) in zip(es, pool.map(expert, es)):
                    s1.copy_(torch.from_numpy(w1).to(td))
                    s2.copy_(torch.from_numpy(w2).to(td))
                    moe_pack_weights(self._one, 1, s1, self.w1[e])
                    moe_pack_weights(self._one, 2, s2, self.w2[e])
        torch.cuda.synchronize(dev)

    def make_copies(self, n: int) -> None:
        """Keep n identical copies of the packed weights (n >= 1)."""
        self.weight_copies = [(self.w1, self.w2)] + [(self.w1.clone(), self.w2.clone())
                                                     for _ in range(max(1, n) - 1)]

    # ---- the five entry points on this layer's buffers --------------------------------
    def route(self, H: int = -1):
        moe_route(self.shape, self.x, self.w_gate, self.b_gate, self.topk_idx, self.topk_w, self.margin,
                  self.counts, self.offsets, H, self.hot_mask if H >= 0 else None, self.ws)

    def permute(self, topk_idx=None, offsets=None):
        moe_permute(self.shape, self.x, self.topk_idx if topk_idx is None else topk_idx,
                    self.offsets if offsets is None else offsets, self.perm, self.inv_perm, self.x_perm,
                    self.ws)

    def expert_ffn(self, mask=None, x_perm=None, offsets=None, copy: int = 0):
        w1, w2 = self.weight_copies[copy % len(self.weight_copies)]
        xp = self.x_perm if x_perm is None else x_perm
        off = self.offsets if offsets is None else offsets
        if self.b1 is None and self.b2 is None:
            moe_expert_ffn(self.shape, xp, w1, w2, off, mask, self.y_perm, self.ws)
        else:
            moe_expert_ffn_biased(self.shape, xp, w1, self.b1, w2, self.b2, off, mask, self.y_perm, self.ws)

    def combine(self, mask=None, y_perm=None, inv_perm=None, topk_idx=None, topk_w=None):
        moe_combine(self.shape, self.y_perm if y_perm is None else y_perm,
                    self.inv_perm if inv_perm is None else inv_perm,
                    self.topk_idx if topk_idx is None else topk_idx,
                    self.topk_w if topk_w is None else topk_w, mask, self.out)

    def forward(self, mask=None, H: int = -1, debug: bool = False, copy: int = 0):
        w1, w2 = self.weight_copies[copy % len(self.weight_copies)]
        dbg = (self.topk_idx, self.topk_w, self.counts, self.perm, self.hot_mask) if debug else (None,) * 5
        if self.b1 is None and self.b2 is None:
            moe_layer_forward(self.shape, self.x, self.w_gate, self.b_gate, w1, w2, mask, H, self.out, *dbg,
                              ws=self.ws)
        else:
            moe_layer_forward_biased(self.shape, self.x, self.w_gate, self.b_gate, w1, self.b1, w2, self.b2, mask, H,
                                     self.out, *dbg, ws=self.ws)
        return self.out

    def out_numpy(self) -> np.ndarray:
        return self.out.float().cpu().numpy()
