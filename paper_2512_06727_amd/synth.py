"""Seeded synthetic workloads with the shapes of the paper's GPT-2 / TinyLlama runs.

This module only *produces inputs* (activations, autoencoder weights, reuse
maps, workload shapes).  It holds none of the method's arithmetic (no encode,
decode, attention, rounding of results or source resolution) and is the one
module both the CPU oracle's tests and the HIP path's harness draw from.

Random numbers come from a counter-based generator so that any slice of any
tensor can be produced on its own, on the CPU or on the GPU, with identical
bits: value(key, i) = NORMAL_TABLE[ mix64(key ^ (i+1)*GOLDEN) >> 48 ] where
NORMAL_TABLE holds the 65536 mid-point quantiles of N(0,1).  Only integer
arithmetic and a table gather are involved, so torch's CPU and ROCm back ends
agree bit for bit.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB


def _s64(x: int) -> int:
    """Python int (mod 2^64) -> the same bits as a signed 64-bit value."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _mix_py(x: int) -> int:
    x &= _M64
    x = ((x ^ (x >> 30)) * _C1) & _M64
    x = ((x ^ (x >> 27)) * _C2) & _M64
    return x ^ (x >> 31)


def stream_key(seed: int, *parts: int) -> int:
    """64-bit key of an independent random stream named by integers."""
    k = _mix_py(seed + _GOLDEN)
    for p in parts:
        k = _mix_py(k ^ ((int(p) + 1) * _GOLDEN))
    return k


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of int64 bit patterns."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix_t(x: torch.Tensor) -> torch.Tensor:
    x = (x ^ _lsr(x, 30)) * _s64(_C1)
    x = (x ^ _lsr(x, 27)) * _s64(_C2)
    return x ^ _lsr(x, 31)


_TABLE_CACHE: Dict[str, torch.Tensor] = {}


def normal_table(device="cpu") -> torch.Tensor:
    """65536 mid-point quantiles of N(0,1), fp32, computed once on the CPU."""
    dev = str(device)
    if "cpu" not in _TABLE_CACHE:
        from scipy.special import ndtri
        u = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
        _TABLE_CACHE["cpu"] = torch.from_numpy(ndtri(u).astype(np.float32))
    if dev not in _TABLE_CACHE:
        _TABLE_CACHE[dev] = _TABLE_CACHE["cpu"].to(device)
    return _TABLE_CACHE[dev]


def normal_at(key: int, index: torch.Tensor) -> torch.Tensor:
    """N(0,1) samples (fp32) of stream `key` at the int64 positions `index`."""
    x = index.to(torch.int64)
    h = _mix_t(((x + 1) * _s64(_GOLDEN)) ^ _s64(key))
    return normal_table(index.device)[_lsr(h, 48)]


def normal(key: int, shape: Sequence[int], device="cpu", offset: int = 0) -> torch.Tensor:
    n = int(np.prod(shape)) if len(shape) else 1
    idx = torch.arange(offset, offset + n, dtype=torch.int64, device=device)
    return normal_at(key, idx).reshape(tuple(shape))


TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
DTYPE_BYTES = {"f32": 4, "f16": 2, "bf16": 2}

# stream purposes
_P_WEIGHT, _P_KV, _P_Q, _P_REUSE, _P_BIAS, _P_LATENT, _P_PROMPT_Q = 1, 2, 3, 4, 5, 6, 7


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape of one decode workload (all sizes per GPU)."""
    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    d_head: int
    batch: int
    n_cached: int            # tokens in the cache before the first decode step
    n_steps: int             # decode steps
    dtype: str               # 'f32' | 'f16' | 'bf16' (activations, weights, cache)
    latent: int              # r of a layer that stores all its heads
    hidden: int = 0          # 0: linear autoencoder; else width of the FC before/after the latent
    act: str = "none"        # 'none' | 'gelu' | 'leaky_relu'
    reuse: str = "none"      # 'none' | 'odd:3' | 'from2:1' | 'bernoulli:0.3' | 'kvbernoulli:0.3'
    policy: str = "P1"       # P1: latent shrinks with the stored heads; P2: full-width latent
    weight_std: float = 0.02
    seed: int = 0
    # test knobs (inputs only): multipliers on the decoder's first- and last-layer weights (to drive a two-layer
    # decoder's pre-activations over a chosen range), and a constant added to every latent column by the encoder's
    # last bias, for keys and for values (latent rows with a large common offset)
    dec_gain: Tuple[float, float] = (1.0, 1.0)
    latent_offset: Optional[Tuple[float, float]] = None

    @property
    def d_kv(self) -> int:
        return self.n_kv_heads * self.d_head

    @property
    def max_seq(self) -> int:
        return self.n_cached + self.n_steps

    def scaled(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# The five benchmark configurations: GPT-2-small and TinyLlama-1.1B shapes at growing batch and context.
CONFIGS: Tuple[Workload, ...] = (
    Workload("gpt2-1layer-f32", 1, 12, 12, 64, batch=1, n_cached=128, n_steps=1, dtype="f32", latent=384),
    Workload("gpt2-12layer-f16", 12, 12, 12, 64, batch=8, n_cached=1024, n_steps=64, dtype="f16", latent=384,
             reuse="odd:3"),
    Workload("tinyllama-bf16", 22, 32, 4, 64, batch=32, n_cached=2048, n_steps=128, dtype="bf16", latent=128,
             reuse="from2:1"),
    Workload("tinyllama-bf16-mlp-prefill", 22, 32, 4, 64, batch=16, n_cached=4096, n_steps=32, dtype="bf16",
             latent=128, hidden=256, act="gelu"),
    Workload("tinyllama-bf16-long", 22, 32, 4, 64, batch=256, n_cached=8192, n_steps=16, dtype="bf16",
             latent=128, reuse="bernoulli:0.3"),
)


def reuse_map(w: Workload) -> np.ndarray:
    """bool [n_layers, 2 (K,V), n_kv_heads]; true = the head takes the previous
    layer's tensor.  The same mask is used for K and V.  Layers are 0-indexed."""
    m = np.zeros((w.n_layers, 2, w.n_kv_heads), dtype=bool)
    if w.reuse == "none":
        return m
    kind, arg = w.reuse.split(":")
    for layer in range(1, w.n_layers):
        rng = np.random.default_rng([w.seed, _P_REUSE, layer])
        if kind == "odd" and layer % 2 == 1:
            m[layer, :, rng.choice(w.n_kv_heads, size=int(arg), replace=False)] = True
        elif kind == "from2" and layer >= 2:
            m[layer, :, rng.choice(w.n_kv_heads, size=int(arg), replace=False)] = True
        elif kind == "bernoulli":
            m[layer, :, :] = rng.random(w.n_kv_heads) < float(arg)
        elif kind == "kvbernoulli":                       # keys and values drawn independently
            m[layer] = rng.random((2, w.n_kv_heads)) < float(arg)
        elif kind == "all" and layer >= 1:
            m[layer, :, :] = True
    return m


def _round(x: torch.Tensor, dtype: str) -> torch.Tensor:
    """Make an input tensor exactly representable in the workload dtype."""
    return x.to(TORCH_DTYPE[dtype]).to(torch.float32)


@dataclasses.dataclass
class AEWeights:
    """Autoencoder of one (layer, K|V): fp32 tensors holding dtype-representable
    values; row-major [in_features, out_features]."""
    heads: List[int]               # KV heads whose columns the autoencoder covers, in order
    latent: int
    hidden: int
    act: str
    slope: float
    enc: List[Tuple[torch.Tensor, Optional[torch.Tensor]]]
    dec: List[Tuple[torch.Tensor, Optional[torch.Tensor]]]

    @property
    def width(self) -> int:
        return self.enc[0][0].shape[0]


def autoencoder(w: Workload, layer: int, which: int, reuse: Optional[np.ndarray] = None,
                with_bias: bool = False) -> AEWeights:
    """Seeded N(0, weight_std) autoencoder of one layer's K (which=0) or V (which=1).

    Full-size matrices are drawn for the D_kv -> r -> D_kv shape; under policy P1 a
    layer that stores only the head set S uses the leading sub-blocks
    W_enc[cols(S), :r_S], W_dec[:r_S, cols(S)] with r_S = r * |S| / H_kv.
    """
    reuse = reuse_map(w) if reuse is None else reuse
    stored = [g for g in range(w.n_kv_heads) if not reuse[layer, which, g]]
    if w.policy == "P1":
        heads = stored
        latent = w.latent * len(stored) // w.n_kv_heads
    else:
        heads = list(range(w.n_kv_heads))
        latent = w.latent
    cols = torch.tensor([g * w.d_head + i for g in heads for i in range(w.d_head)], dtype=torch.int64)
    d = w.d_kv

    def mat(tag: int, rows: int, cs: int) -> torch.Tensor:
        key = stream_key(w.seed, _P_WEIGHT, layer, which, tag)
        return _round(normal(key, (rows, cs)) * w.weight_std, w.dtype)

    def bias(tag: int, n: int) -> Optional[torch.Tensor]:
        if not with_bias:
            return None
        key = stream_key(w.seed, _P_BIAS, layer, which, tag)
        return _round(normal(key, (n,)) * w.weight_std, w.dtype)

    if w.hidden == 0:
        enc = [(mat(0, d, w.latent)[cols][:, :latent].contiguous(), None if not with_bias else bias(0, w.latent)[:latent].contiguous())]
        dec = [(mat(1, w.latent, d)[:latent][:, cols].contiguous(), None if not with_bias else bias(1, d)[cols].contiguous())]
    else:
        h = w.hidden
        enc = [(mat(0, d, h)[cols].contiguous(), bias(0, h)),
               (mat(2, h, w.latent)[:, :latent].contiguous(), None if not with_bias else bias(2, w.latent)[:latent].contiguous())]
        dec = [(mat(3, w.latent, h)[:latent].contiguous(), bias(3, h)),
               (mat(1, h, d)[:, cols].contiguous(), None if not with_bias else bias(1, d)[cols].contiguous())]
    if w.dec_gain != (1.0, 1.0):
        dec[0] = (_round(dec[0][0] * w.dec_gain[0], w.dtype), dec[0][1])
        dec[-1] = (_round(dec[-1][0] * w.dec_gain[1], w.dtype), dec[-1][1])
    if w.latent_offset is not None and latent > 0:
        b_last = enc[-1][1] if enc[-1][1] is not None else torch.zeros(latent)
        enc[-1] = (enc[-1][0], _round(b_last + float(w.latent_offset[which]), w.dtype))
    return AEWeights(heads=heads, latent=latent, hidden=w.hidden, act=w.act, slope=0.01, enc=enc, dec=dec)


def kv_tokens(w: Workload, layer: int, which: int, b0: int, b1: int, t0: int, t1: int,
              device="cpu") -> torch.Tensor:
    """New-token K (which=0) or V (which=1) activations ~ N(0,1) for sequences
    [b0,b1) and positions [t0,t1): fp32 [b1-b0, t1-t0, D_kv], dtype-representable.
    Any slice can be generated on its own."""
    key = stream_key(w.seed, _P_KV, layer, which)
    d = w.d_kv
    b = torch.arange(b0, b1, dtype=torch.int64, device=device).view(-1, 1, 1)
    t = torch.arange(t0, t1, dtype=torch.int64, device=device).view(1, -1, 1)
    c = torch.arange(d, dtype=torch.int64, device=device).view(1, 1, -1)
    idx = (b * w.max_seq + t) * d + c
    return _round(normal_at(key, idx), w.dtype)


def queries(w: Workload, layer: int, step: int, device="cpu", gain: float = 1.0) -> torch.Tensor:
    """q ~ N(0,1) * gain for one decode step: fp32 [batch, H_q, d_head]."""
    key = stream_key(w.seed, _P_Q, layer, step)
    return _round(normal(key, (w.batch, w.n_q_heads, w.d_head), device=device) * gain, w.dtype)


def prompt_queries(w: Workload, layer: int, b0: int, b1: int, t0: int, t1: int, device="cpu",
                   gain: float = 1.0) -> torch.Tensor:
    """q ~ N(0,1) * gain of the prompt tokens at positions [t0,t1) of sequences [b0,b1):
    fp32 [b1-b0, t1-t0, H_q, d_head], dtype-representable.  Any slice can be generated on its own."""
    key = stream_key(w.seed, _P_PROMPT_Q, layer)
    d = w.n_q_heads * w.d_head
    b = torch.arange(b0, b1, dtype=torch.int64, device=device).view(-1, 1, 1)
    t = torch.arange(t0, t1, dtype=torch.int64, device=device).view(1, -1, 1)
    c = torch.arange(d, dtype=torch.int64, device=device).view(1, 1, -1)
    idx = (b * w.max_seq + t) * d + c
    return _round(normal_at(key, idx) * gain, w.dtype).view(b1 - b0, t1 - t0, w.n_q_heads, w.d_head)


def latent_rows(w: Workload, layer: int, which: int, latent: int, b0: int, b1: int, t0: int, t1: int,
                device="cpu", std: float = 0.32) -> torch.Tensor:
    """Synthetic latent rows ~ N(0, std) for tests that fill a cache directly
    (std 0.32 is what a N(0,0.02) encoder gives a 256-wide N(0,1) input)."""
    key = stream_key(w.seed, _P_LATENT, layer, which)
    b = torch.arange(b0, b1, dtype=torch.int64, device=device).view(-1, 1, 1)
    t = torch.arange(t0, t1, dtype=torch.int64, device=device).view(1, -1, 1)
    c = torch.arange(latent, dtype=torch.int64, device=device).view(1, 1, -1)
    idx = (b * w.max_seq + t) * latent + c
    return _round(normal_at(key, idx) * std, w.dtype)
