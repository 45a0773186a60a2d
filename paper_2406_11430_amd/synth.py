"""Seeded synthetic KV caches with the shapes of the paper's workloads.

This module only draws random inputs.  It holds none of the method's
arithmetic (no norms, no selection, no attention), so both the HIP path and the
CPU checker can be fed from it without sharing any code of the method itself.

The paper evaluates on Llama-2-7B / Llama-3-8B style models (Sec. 4) with
contexts of a few thousand up to ~100k tokens and compression ratios of 50 %
and 90 %; its Sec. 3 / Fig. 1 observation is that a handful of tokens (the
beginning-of-sequence token, punctuation) have a markedly lower key norm than
the rest.  The generator imitates exactly that structure:

* ``K[l,b,h,t,:] = s * g`` with ``g ~ N(0,1)^D`` and a per-(l,b,h,t) log-normal
  scale ``s = exp(0.5 z)``, ``z ~ N(0,1)``;
* the first ``sink_tokens`` positions of every head are additionally scaled by
  ``sink_scale`` (low-norm "sink" tokens shared by all heads);
* optionally one contiguous span of ``span_len`` positions (same span in every
  head, start drawn from the seed) is scaled by ``span_scale`` -- a planted
  low-norm region standing in for a retrieval target;
* ``V ~ N(0,1)``, ``Q ~ N(0,1)``.

Everything is drawn in fp32 and then cast to the cache dtype.  Draws happen on
the requested device with a ``torch.Generator`` of that device, so CPU and GPU
draws of the same seed differ; a caller that wants the same bits on both sides
draws once and copies.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Tuple

import torch

__all__ = [
    "CacheConfig", "CONFIGS", "layer_seed", "make_layer", "make_query",
    "span_start", "ragged_lengths", "torch_dtype", "as_numpy_bits",
]


@dataclass(frozen=True)
class CacheConfig:
    name: str
    config_id: int
    L: int            # layers
    B: int            # batch (sequences)
    Hkv: int          # KV heads
    Hq: int           # query heads
    D: int            # head_dim
    T: int            # cached tokens per sequence
    dtype: str        # "f32" | "bf16"
    keep_ratio: float
    decode_steps: int
    sink_tokens: int = 4
    sink_scale: float = 0.1
    span_len: int = 0
    span_scale: float = 1.0

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def scaled(self, **kw) -> "CacheConfig":
        """Same recipe at another size (for tests)."""
        return replace(self, **kw)


CONFIGS: Dict[str, CacheConfig] = {
    # Tiny fp32 case the CPU checker finishes instantly.
    "C1": CacheConfig("C1-tiny", 1, L=1, B=1, Hkv=4, Hq=4, D=64, T=512,
                      dtype="f32", keep_ratio=0.5, decode_steps=1),
    # One Llama-2-7B-shaped MHA layer.
    "C2": CacheConfig("C2-llama2-7b-layer", 2, L=1, B=1, Hkv=32, Hq=32, D=128,
                      T=4096, dtype="bf16", keep_ratio=0.5, decode_steps=1),
    # Llama-3-8B-shaped GQA stack at 32k context (the graded workload).
    "C3": CacheConfig("C3-llama3-8b-gqa-32k", 3, L=32, B=4, Hkv=8, Hq=32,
                      D=128, T=32768, dtype="bf16", keep_ratio=0.5,
                      decode_steps=64),
    # Long-context retrieval shape with one planted low-norm span.
    "C4": CacheConfig("C4-retrieval-131k", 4, L=32, B=1, Hkv=8, Hq=32, D=128,
                      T=131072, dtype="bf16", keep_ratio=0.1, decode_steps=16,
                      span_len=64, span_scale=0.3),
}


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def layer_seed(cfg: CacheConfig, layer: int) -> int:
    return 1234 + 1000 * cfg.config_id + layer


def span_start(cfg: CacheConfig) -> int:
    """Start of the planted span (same in every layer and head); -1 if none."""
    if cfg.span_len <= 0:
        return -1
    g = torch.Generator(device="cpu")
    g.manual_seed(987654321 + cfg.config_id)
    lo = cfg.sink_tokens
    hi = cfg.T - cfg.span_len
    return int(torch.randint(lo, hi + 1, (1,), generator=g).item())


def make_layer(cfg: CacheConfig, layer: int, device="cpu"
               ) -> Tuple[torch.Tensor, torch.Tensor]:
    """K and V of one layer, each ``[B][Hkv][T][D]`` in the cache dtype."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(layer_seed(cfg, layer))
    shape = (cfg.B, cfg.Hkv, cfg.T, cfg.D)
    dt = torch_dtype(cfg.dtype)
    K = torch.empty(shape, dtype=dt, device=dev)
    V = torch.empty(shape, dtype=dt, device=dev)
    start = span_start(cfg)
    # One (b, h) slab at a time keeps the fp32 temporaries small at 131k tokens.
    for b in range(cfg.B):
        for h in range(cfg.Hkv):
            gk = torch.randn((cfg.T, cfg.D), generator=g, device=dev,
                             dtype=torch.float32)
            z = torch.randn((cfg.T, 1), generator=g, device=dev,
                            dtype=torch.float32)
            s = torch.exp(0.5 * z)
            if cfg.sink_tokens > 0:
                s[: cfg.sink_tokens] *= cfg.sink_scale
            if start >= 0:
                s[start: start + cfg.span_len] *= cfg.span_scale
            K[b, h] = (gk * s).to(dt)
            V[b, h] = torch.randn((cfg.T, cfg.D), generator=g, device=dev,
                                  dtype=torch.float32).to(dt)
    return K, V


def make_query(cfg: CacheConfig, layer: int, step: int, device="cpu"
               ) -> torch.Tensor:
    """One decode-step query ``[B][Hq][D]`` in the cache dtype."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(layer_seed(cfg, layer) * 4099 + 7 + step)
    q = torch.randn((cfg.B, cfg.Hq, cfg.D), generator=g, device=dev,
                    dtype=torch.float32)
    return q.to(torch_dtype(cfg.dtype))


def ragged_lengths(n_seq: int, lo: int, hi: int, seed: int) -> torch.Tensor:
    """Sequence lengths uniform in [lo, hi] (int64, CPU)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return torch.randint(lo, hi + 1, (n_seq,), generator=g, dtype=torch.int64)


def as_numpy_bits(t: torch.Tensor):
    """Host copy of a tensor as a NumPy array; bf16 comes back as uint16 bit
    patterns (NumPy has no bf16), everything else in its own dtype."""
    import numpy as np
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
