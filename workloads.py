"""Seeded synthetic MoE-FFN layer inputs.

This module only *draws and rounds inputs*; it holds none of the layer's
arithmetic.  Both the CPU oracle's tests and the GPU tests/bench take their
inputs from here so that the two sides see bit-identical numbers.

The five presets mirror the shapes of the paper's workloads (Table 2:
Switch-style top-1 and NLLB-MoE-style top-2 layers with 128 experts, bf16),
plus a tiny fp32 layer and a Switch-base-like layer.  The datasets and
checkpoints the paper uses are not available; the skewed token-per-expert
histogram of its Fig. 3 is imitated by a per-expert gate bias equal to the
log of Zipf weights under a seeded rank permutation.

Memory layout handed to both sides (row-major, last index contiguous):
  x       [T, d_model]
  w_gate  [E, d_model]          (row e = gate weights of expert e)
  b_gate  [E] float32 or None
  W1[e]   [d_ff, d_model]       (row n = weights of hidden unit n)
  W2[e]   [d_model, d_ff]       (row n = weights of output feature n)
i.e. every weight matrix is "out-features x in-features", contraction index
contiguous.

Random streams: numpy PCG64 via default_rng, one independent stream per
tensor (and per expert for W1/W2) keyed by (seed, tag[, expert]), so a single
expert's weights can be regenerated without drawing the others.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Callable, Optional

import numpy as np

_TAG_X, _TAG_WG, _TAG_RANK, _TAG_W1, _TAG_W2 = 1, 2, 3, 4, 5


# ---------------------------------------------------------------------------
# bf16 storage helpers (input preparation only: round once, widen exactly)
# ---------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 -> bfloat16 (nearest, ties to even); returns uint16 bits."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + (np.uint32(0x7FFF) + lsb)
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bits (uint16) to the float32 holding the same value."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """float32 array whose values are exactly representable in `dtype`."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return a
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(a))
    raise ValueError(dtype)


# ---------------------------------------------------------------------------
# configs
# ---------------------------------------------------------------------------
@dataclass(frozen=True)
class MoEConfig:
    name: str
    T: int
    d_model: int
    d_ff: int
    E: int
    k: int
    dtype: str            # "f32" | "bf16"  (storage of x, w_gate, W1, W2, out)
    renormalize: bool     # gate weights renormalised over the chosen k
    seed: int
    zipf_s: Optional[float] = None   # gate bias = ln Zipf(s) weights; None = no bias
    H: Optional[int] = None          # hot mask = top-H experts by token count
    gate_std: float = 0.02
    activation: str = "relu"        # trailing activation of the first linear layer: "relu" | "gelu"
    expert_bias: bool = False       # experts carry biases b1 [d_ff], b2 [d_model] (fp32, N(0, 0.25^2))

    @property
    def A(self) -> int:
        return self.T * self.k


CONFIGS = {
    "tiny_f32": MoEConfig("tiny_f32", T=64, d_model=64, d_ff=256, E=8, k=2,
                          dtype="f32", renormalize=True, seed=0),
    "switch_base": MoEConfig("switch_base", T=2048, d_model=768, d_ff=3072, E=64, k=1,
                             dtype="bf16", renormalize=False, seed=1),
    "switch_large_skew": MoEConfig("switch_large_skew", T=4096, d_model=1024, d_ff=4096,
                                   E=128, k=1, dtype="bf16", renormalize=False, seed=2,
                                   zipf_s=1.1, H=16),
    "nllb_decode": MoEConfig("nllb_decode", T=32, d_model=2048, d_ff=8192, E=128, k=2,
                             dtype="bf16", renormalize=True, seed=3),
    "nllb_prefill_skew": MoEConfig("nllb_prefill_skew", T=16384, d_model=2048, d_ff=8192,
                                   E=128, k=2, dtype="bf16", renormalize=True, seed=4,
                                   zipf_s=1.2, H=32),
}
CONFIG_ORDER = ["tiny_f32", "switch_base", "switch_large_skew", "nllb_decode",
                "nllb_prefill_skew"]

# Further shapes the paper evaluates (Section 5): NLLB-MoE decoder steps at batch sizes 1, 4 and 16
# (one token per sequence and step), and two Switch variants around the base preset for its
# sensitivity study (the study's exact d_model / E are only in a figure; these take the base width
# with 8 and 128 experts).  Same recipe as the presets above.
EXTRA_CONFIGS = {
    "nllb_decode_b1": MoEConfig("nllb_decode_b1", T=1, d_model=2048, d_ff=8192, E=128, k=2,
                                dtype="bf16", renormalize=True, seed=5),
    "nllb_decode_b4": MoEConfig("nllb_decode_b4", T=4, d_model=2048, d_ff=8192, E=128, k=2,
                                dtype="bf16", renormalize=True, seed=6),
    "nllb_decode_b16": MoEConfig("nllb_decode_b16", T=16, d_model=2048, d_ff=8192, E=128, k=2,
                                 dtype="bf16", renormalize=True, seed=7),
    "switch_base_8": MoEConfig("switch_base_8", T=2048, d_model=768, d_ff=3072, E=8, k=1,
                               dtype="bf16", renormalize=False, seed=8),
    "switch_base_128": MoEConfig("switch_base_128", T=2048, d_model=768, d_ff=3072, E=128, k=1,
                                 dtype="bf16", renormalize=False, seed=9),
}


def matched_noise(cfg: MoEConfig) -> MoEConfig:
    """Secondary variant of a skewed preset: gate std = 1.28/sqrt(d_model), so the
    logit noise has roughly unit-Gumbel spread and token counts follow the Zipf
    weights (many cold experts with 1-7 tokens next to a few hot ones)."""
    return replace(cfg, name=cfg.name + "_matched",
                   gate_std=1.28 / float(np.sqrt(cfg.d_model)))


# ---------------------------------------------------------------------------
# generators
# ---------------------------------------------------------------------------
def _rng(seed: int, tag: int, sub: int = 0) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(tag), int(sub)])


def zipf_log_bias(E: int, s: float, seed: int) -> np.ndarray:
    """ln of Zipf(s) weights w_r = r^-s / sum r^-s, r=1..E, ranks assigned to
    experts by a seeded permutation.  float32."""
    r = np.arange(1, E + 1, dtype=np.float64)
    w = r ** (-float(s))
    w /= w.sum()
    rank_of_expert = _rng(seed, _TAG_RANK).permutation(E)
    return np.log(w[rank_of_expert]).astype(np.float32)


def make_activations(cfg: MoEConfig) -> np.ndarray:
    x = _rng(cfg.seed, _TAG_X).standard_normal((cfg.T, cfg.d_model), dtype=np.float32)
    return round_to_storage(x, cfg.dtype)


def make_gate(cfg: MoEConfig):
    wg = _rng(cfg.seed, _TAG_WG).standard_normal((cfg.E, cfg.d_model), dtype=np.float32)
    wg *= np.float32(cfg.gate_std)
    wg = round_to_storage(wg, cfg.dtype)
    bias = None if cfg.zipf_s is None else zipf_log_bias(cfg.E, cfg.zipf_s, cfg.seed)
    return wg, bias


def make_expert(cfg: MoEConfig, e: int):
    """(W1_e [d_ff, d_model], W2_e [d_model, d_ff]) as storage-rounded float32."""
    w1 = _rng(cfg.seed, _TAG_W1, e).standard_normal((cfg.d_ff, cfg.d_model), dtype=np.float32)
    w1 *= np.float32(1.0 / np.sqrt(cfg.d_model))
    w2 = _rng(cfg.seed, _TAG_W2, e).standard_normal((cfg.d_model, cfg.d_ff), dtype=np.float32)
    w2 *= np.float32(1.0 / np.sqrt(cfg.d_ff))
    return round_to_storage(w1, cfg.dtype), round_to_storage(w2, cfg.dtype)


_TAG_B1, _TAG_B2 = 101, 102


def make_expert_bias(cfg: MoEConfig, e: int):
    """(b1_e [d_ff], b2_e [d_model]) as float32, for configs with expert_bias."""
    b1 = _rng(cfg.seed, _TAG_B1, e).standard_normal(cfg.d_ff, dtype=np.float32) * np.float32(0.25)
    b2 = _rng(cfg.seed, _TAG_B2, e).standard_normal(cfg.d_model, dtype=np.float32) * np.float32(0.25)
    return b1, b2


@dataclass
class LayerInputs:
    cfg: MoEConfig
    x: np.ndarray
    w_gate: np.ndarray
    b_gate: Optional[np.ndarray]
    expert: Callable[[int], tuple]     # e -> (W1_e, W2_e), regenerated on demand

    def all_experts(self):
        """Stacked (W1 [E,d_ff,d_model], W2 [E,d_model,d_ff]); small configs only."""
        ws = [self.expert(e) for e in range(self.cfg.E)]
        return np.stack([w[0] for w in ws]), np.stack([w[1] for w in ws])


def make_layer(cfg: MoEConfig) -> LayerInputs:
    x = make_activations(cfg)
    wg, b = make_gate(cfg)
    return LayerInputs(cfg, x, wg, b, lambda e: make_expert(cfg, e))


def for_each_expert(cfg: MoEConfig, sink: Callable[[int, np.ndarray, np.ndarray], None],
                    workers: int = 8) -> None:
    """Generate every expert's weights (threaded) and hand them to `sink(e, W1_e, W2_e)`
    one expert at a time, so no more than `workers` experts live on the host at once."""
    with ThreadPoolExecutor(max_workers=max(1, workers)) as pool:
        for e0 in range(0, cfg.E, workers):
            es = list(range(e0, min(cfg.E, e0 + workers)))
            for e, (w1, w2) in zip(es, pool.map(lambda q: make_expert(cfg, q), es)):
                sink(e, w1, w2)
