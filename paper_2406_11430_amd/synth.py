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
    "StreamConfig", "STREAM_CONFIGS", "stream_lengths", "make_ragged_layer", "make_stream_step",
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
    # Gemma-7B-shaped MHA stack (16 heads of 256 elements) at its 8k context: an extra
    # shape for the 512-byte bf16 rows, not one of the contract's workloads.
    "C6": CacheConfig("C6-gemma-7b-mha-8k", 6, L=28, B=4, Hkv=16, Hq=16, D=256,
                      T=8192, dtype="bf16", keep_ratio=0.5, decode_steps=64),
}


@dataclass(frozen=True)
class StreamConfig:
    """Ragged streaming batch: sequences of different prompt lengths, compressed to
    keep_ratio, then decoded step by step with the ratio enforced incrementally."""
    name: str
    config_id: int
    L: int
    n_seq: int
    len_lo: int
    len_hi: int
    Hkv: int
    Hq: int
    D: int
    dtype: str
    keep_ratio: float
    decode_steps: int
    sink_tokens: int = 4
    sink_scale: float = 0.1

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def scaled(self, **kw) -> "StreamConfig":
        return replace(self, **kw)


STREAM_CONFIGS: Dict[str, StreamConfig] = {
    # Batched streaming decode: 64 sequences, prompt lengths uniform in [1024, 8192].
    "C5": StreamConfig("C5-streaming-ragged", 5, L=32, n_seq=64, len_lo=1024, len_hi=8192, Hkv=8, Hq=32,
                       D=128, dtype="bf16", keep_ratio=0.5, decode_steps=256),
}


def stream_lengths(cfg: StreamConfig) -> torch.Tensor:
    """Prompt lengths of the batch (int64, CPU), seeded."""
    return ragged_lengths(cfg.n_seq, cfg.len_lo, cfg.len_hi, 424242 + cfg.config_id)


def _scaled_rows(shape, g, dev, dt, sink_rows=None, sink_scale=1.0):
    x = torch.randn(shape, generator=g, device=dev, dtype=torch.float32)
    z = torch.randn(shape[:-1] + (1,), generator=g, device=dev, dtype=torch.float32)
    s = torch.exp(0.5 * z)
    if sink_rows is not None:
        s[..., sink_rows, :] *= sink_scale
    return (x * s).to(dt)


def make_ragged_layer(cfg: StreamConfig, layer: int, device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """Prompt K and V of one layer, ``[Hkv][total_tokens][D]``: the sequences of the
    batch back to back in every head plane; the first tokens of every sequence
    are low-norm sinks."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(1234 + 1000 * cfg.config_id + layer)
    dt = torch_dtype(cfg.dtype)
    lens = stream_lengths(cfg)
    total = int(lens.sum())
    starts = torch.cumsum(lens, 0) - lens
    sink = torch.cat([torch.arange(int(a), int(a) + min(cfg.sink_tokens, int(n))) for a, n in zip(starts, lens)]).to(dev)
    K = _scaled_rows((cfg.Hkv, total, cfg.D), g, dev, dt, sink, cfg.sink_scale)
    V = torch.randn((cfg.Hkv, total, cfg.D), generator=g, device=dev, dtype=torch.float32).to(dt)
    return K, V


def make_stream_step(cfg: StreamConfig, step: int, device="cpu"):
    """New tokens and queries of one decode step: Knew, Vnew ``[L][n_seq][Hkv][D]``,
    Q ``[L][n_seq][Hq][D]``."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed((1234 + 1000 * cfg.config_id) * 7919 + step)
    dt = torch_dtype(cfg.dtype)
    Knew = _scaled_rows((cfg.L, cfg.n_seq, cfg.Hkv, cfg.D), g, dev, dt)
    Vnew = torch.randn((cfg.L, cfg.n_seq, cfg.Hkv, cfg.D), generator=g, device=dev, dtype=torch.float32).to(dt)
    Q = torch.randn((cfg.L, cfg.n_seq, cfg.Hq, cfg.D), generator=g, device=dev, dtype=torch.float32).to(dt)
    return Knew, Vnew, Q


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
