"""Plain, slow, fp64 CPU oracle of KV-CAR's decode-time path.

TEST INFRASTRUCTURE ONLY: used by tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py.  It shares no code with the HIP kernels and
never reads anything they produced.

What it computes, in the paper's order (Methodology, "Network Architecture";
attention is Eq. 1 of the Background section):

  1. encode   z = enc(x)            the encoder placed after K/V generation maps
                                    a 1 x D vector to 1 x d (here: D_kv -> r)
  2. store    Z[layer][K|V][b,t] =  round(z -> cache dtype); one latent row is
                                    appended per token, for K and for V
  3. resolve  a reused head of layer N takes the K (or V) of the same head in
                                    layer N-1 (inter-layer head reuse); chains are
                                    followed back to the nearest layer that stores
                                    the head itself
  4. decode   x^ = dec(Z rows)      applied to every cached row at every step
  5. attend   softmax(q K^T / sqrt(d_k)) V   per query head (Eq. 1)

All arithmetic is float64.  The only rounding that belongs to the method is the
one at the store (the cache holds P-byte elements, Eq. 3); it is done as
fp64 -> fp32 -> cache dtype, round-to-nearest-even.

Optional int8 latents (Methodology, "Quantization", Eq. "quant"): step 2 then
quantises each latent row to int8 codes with a per-row scale and zero point, and
step 4 dequantises the row before the decoder.  The quantiser's decisions (min,
max, scale, zero point, codes) are integer-valued results of floating point, so
they are taken in fp32, one IEEE operation at a time, as the kernels take them.

Pins (tests/test_oracle_*.py): pure-Python brute force on tiny shapes, a library
SDPA on the decoded K/V, r = D with an orthogonal autoencoder == uncompressed
attention, all-false reuse map == per-layer attention, softmax rows sum to 1,
q = 0 closed form, peaked q, chained reuse vs explicit copies, rounding vs hand
cases and a library cast, GELU vs erf; the quantiser vs a hand-worked row, exact
rational arithmetic, an arithmetic progression (codes -128..127), the half-step
error bound, and invariance under positive dyadic scaling and shifts; the prefill form vs scalar
brute force, a library causal SDPA, token-by-token decode steps, and causality.  The numerical values a *trained*
autoencoder would produce are "parity unpinned": the paper ships no weights.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

K, V = 0, 1

ACT_NONE = "none"          # linear autoencoder
ACT_LEAKY_RELU = "leaky_relu"
ACT_GELU = "gelu"          # exact erf form


# --------------------------------------------------------------------------
# rounding to the cache dtype (step 2)
# --------------------------------------------------------------------------
def _round_f32_to_bf16(x32: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 round-to-nearest-even, result returned as fp32 values."""
    bits = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    bits = bits + np.uint64(0x7FFF) + lsb
    bits = (bits >> np.uint64(16)) << np.uint64(16)
    return bits.astype(np.uint32).view(np.float32)


def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64 values to `dtype` ('f32' | 'f16' | 'bf16'); returns fp64 holding
    exactly-representable values.  Path: fp64 -> fp32 (RNE) -> dtype (RNE)."""
    x32 = np.asarray(x, dtype=np.float64).astype(np.float32)
    if dtype == "f32":
        return x32.astype(np.float64)
    if dtype == "f16":
        return x32.astype(np.float16).astype(np.float64)
    if dtype == "bf16":
        return _round_f32_to_bf16(x32).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


def dtype_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """Raw storage bits of already-rounded values (for byte-exact cache checks)."""
    if dtype == "f32":
        return np.asarray(x, dtype=np.float32).view(np.uint32)
    if dtype == "f16":
        return np.asarray(x, dtype=np.float16).view(np.uint16)
    if dtype == "bf16":
        b = np.ascontiguousarray(np.asarray(x, dtype=np.float32)).view(np.uint32)
        return (b >> np.uint32(16)).astype(np.uint16)
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# autoencoder (steps 1 and 4)
# --------------------------------------------------------------------------
def activation(x: np.ndarray, kind: str, slope: float = 0.01) -> np.ndarray:
    if kind == ACT_NONE:
        return x
    if kind == ACT_LEAKY_RELU:
        return np.where(x >= 0.0, x, slope * x)
    if kind == ACT_GELU:
        erf = np.vectorize(math.erf, otypes=[np.float64])
        return 0.5 * x * (1.0 + erf(x / math.sqrt(2.0)))
    raise ValueError(kind)


class Autoencoder:
    """One layer's autoencoder for K or for V.

    heads   KV-head indices whose d_head-wide column blocks, concatenated in
            this order, form the encoder input / decoder output.
    enc,dec lists of (W [in,out], b [out] or None): one pair = linear map,
            two pairs = FC -> act -> FC (batch-norm, if any, folded by the
            caller into the first pair).
    """

    def __init__(self, heads: Sequence[int], enc, dec, act: str = ACT_NONE, slope: float = 0.01):
        self.heads = [int(h) for h in heads]
        self.enc = [(np.asarray(w, np.float64), None if b is None else np.asarray(b, np.float64)) for w, b in enc]
        self.dec = [(np.asarray(w, np.float64), None if b is None else np.asarray(b, np.float64)) for w, b in dec]
        self.act = act
        self.slope = float(slope)
        assert len(self.enc) in (1, 2) and len(self.dec) == len(self.enc)
        if len(self.enc) == 1:
            assert act == ACT_NONE
        self.latent = self.enc[-1][0].shape[1]
        self.width = self.enc[0][0].shape[0]
        assert self.dec[0][0].shape[0] == self.latent and self.dec[-1][0].shape[1] == self.width

    def _mlp(self, x, layers):
        h = x
        for i, (w, b) in enumerate(layers):
            h = h @ w
            if b is not None:
                h = h + b
            if i + 1 < len(layers):
                h = activation(h, self.act, self.slope)
        return h

    def encode(self, x: np.ndarray) -> np.ndarray:
        """x [..., width] -> z [..., latent]  (encoder after K/V generation)."""
        return self._mlp(np.asarray(x, np.float64), self.enc)

    def decode(self, z: np.ndarray) -> np.ndarray:
        """z [..., latent] -> x^ [..., width]  (decoder at cache retrieval)."""
        return self._mlp(np.asarray(z, np.float64), self.dec)


# --------------------------------------------------------------------------
# int8 quantisation of latent rows ("Quantization", Eq. "quant")
# --------------------------------------------------------------------------
def quantize_rows(z: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Eq. "quant" applied to each row (last axis) of z:

        scale     = 255 / (max(x) - min(x))
        zeropoint = -round(scale * min(x)) - 128
        Xquant    = round(scale * x + zeropoint)

    Returns (codes int8 [..., r], scale fp32 [...], zeropoint int32 [...]).
    Readings where the paper is silent: x is one token's latent row; round is
    round-half-to-even; codes saturate to [-128, 127] (the two roundings can
    push max(x) to 128); a constant row uses |x| in place of the zero range
    (then it is reproduced up to the rounding of the scale), an all-zero row uses 1.  Every operation is
    a single fp32 operation (the input is rounded to fp32 first)."""
    f32 = np.float32
    x = np.asarray(z, dtype=np.float64).astype(f32)
    mx = x.max(axis=-1)
    mn = x.min(axis=-1)
    rng = (mx - mn).astype(f32)
    rng = np.where(rng == 0, np.abs(mx), rng).astype(f32)
    rng = np.where(rng == 0, f32(1), rng).astype(f32)
    scale = (f32(255) / rng).astype(f32)
    zp = (-np.rint((scale * mn).astype(f32)) - f32(128)).astype(f32)
    t = (scale[..., None] * x).astype(f32)
    q = np.rint((t + zp[..., None]).astype(f32))
    codes = np.clip(q, -128, 127).astype(np.int8)
    return codes, scale, zp.astype(np.int64).clip(-2**31, 2**31 - 1).astype(np.int32)


def dequantize_rows(codes: np.ndarray, scale: np.ndarray, zeropoint: np.ndarray) -> np.ndarray:
    """Eq. "quant", last line: Xdequant = (Xquant - zeropoint) / scale, in fp64."""
    c = np.asarray(codes, dtype=np.float64)
    return (c - np.asarray(zeropoint, np.float64)[..., None]) / np.asarray(scale, np.float64)[..., None]


# --------------------------------------------------------------------------
# head reuse (step 3)
# --------------------------------------------------------------------------
def resolve_source(reuse: np.ndarray, layer: int, which: int, head: int) -> int:
    """Layer whose cache supplies `head` of `layer`.

    reuse[N][which][g] true means head g of layer N takes the previous layer's
    K (which=0) or V (which=1).  "The previous layer's KV" is whatever layer
    N-1 itself uses, so chains are followed to the nearest layer M <= N whose
    bit is clear.  Layer 0 has no predecessor.
    """
    m = layer
    while reuse[m][which][head]:
        if m == 0:
            raise ValueError("layer 0 cannot reuse")
        m -= 1
    return m


# --------------------------------------------------------------------------
# the path
# --------------------------------------------------------------------------
class KVCAROracle:
    def __init__(self, n_layers: int, n_q_heads: int, n_kv_heads: int, d_head: int,
                 max_batch: int, max_seq: int, dtype: str, softmax_scale: Optional[float] = None,
                 latent_format: str = "dtype"):
        assert n_q_heads % n_kv_heads == 0
        self.n_layers, self.hq, self.hkv, self.dh = n_layers, n_q_heads, n_kv_heads, d_head
        self.max_batch, self.max_seq, self.dtype = max_batch, max_seq, dtype
        self.scale = 1.0 / math.sqrt(d_head) if not softmax_scale else float(softmax_scale)
        self.reuse = np.zeros((n_layers, 2, n_kv_heads), dtype=bool)
        self.ae: Dict[Tuple[int, int], Autoencoder] = {}
        self.Z: Dict[Tuple[int, int], np.ndarray] = {}   # latent caches, values already rounded
        # "int8": rows are stored as codes + (scale, zeropoint) per row; Z then holds their dequantised values
        assert latent_format in ("dtype", "int8")
        self.latent_format = latent_format
        self.Q: Dict[Tuple[int, int], np.ndarray] = {}         # int8 codes [B, L, r]
        self.Qscale: Dict[Tuple[int, int], np.ndarray] = {}    # fp32 [B, L]
        self.Qzero: Dict[Tuple[int, int], np.ndarray] = {}     # int32 [B, L]

    # -- configuration ------------------------------------------------------
    def set_reuse_map(self, layer: int, k_reuse, v_reuse) -> None:
        k_reuse = np.asarray(k_reuse, dtype=bool)
        v_reuse = np.asarray(v_reuse, dtype=bool)
        if layer == 0 and (k_reuse.any() or v_reuse.any()):
            raise ValueError("layer 0 cannot reuse")
        self.reuse[layer, K] = k_reuse
        self.reuse[layer, V] = v_reuse

    def set_autoencoder(self, layer: int, which: int, ae: Autoencoder) -> None:
        assert ae.width == len(ae.heads) * self.dh
        self.ae[(layer, which)] = ae
        self.Z[(layer, which)] = np.full((self.max_batch, self.max_seq, ae.latent), np.nan)
        if self.latent_format == "int8":
            self.Q[(layer, which)] = np.zeros((self.max_batch, self.max_seq, ae.latent), np.int8)
            self.Qscale[(layer, which)] = np.zeros((self.max_batch, self.max_seq), np.float32)
            self.Qzero[(layer, which)] = np.zeros((self.max_batch, self.max_seq), np.int32)

    # -- steps 1+2 ----------------------------------------------------------
    def encode_append(self, layer: int, k_new: np.ndarray, v_new: np.ndarray, pos0) -> None:
        """k_new, v_new [B, T_new, H_kv*d_head]; rows land at [pos0, pos0+T_new).  pos0 may be a
        sequence of per-sequence positions (ragged batch)."""
        if not np.isscalar(pos0):
            for b, pb in enumerate(pos0):
                self._encode_append_rows(layer, k_new[b:b + 1], v_new[b:b + 1], int(pb), b)
            return
        self._encode_append_rows(layer, k_new, v_new, int(pos0), 0)

    def _encode_append_rows(self, layer: int, k_new: np.ndarray, v_new: np.ndarray, pos0: int, b0: int) -> None:
        for which, x in ((K, k_new), (V, v_new)):
            ae = self.ae[(layer, which)]
            if ae.latent == 0 or not ae.heads:
                continue
            x = np.asarray(x, np.float64)
            b, t, _ = x.shape
            assert b0 + b <= self.max_batch and pos0 + t <= self.max_seq
            cols = np.concatenate([np.arange(g * self.dh, (g + 1) * self.dh) for g in ae.heads])
            z = ae.encode(x[:, :, cols])
            if self.latent_format == "int8":
                codes, scale, zp = quantize_rows(z)
                self.Q[(layer, which)][b0:b0 + b, pos0:pos0 + t, :] = codes
                self.Qscale[(layer, which)][b0:b0 + b, pos0:pos0 + t] = scale
                self.Qzero[(layer, which)][b0:b0 + b, pos0:pos0 + t] = zp
                self.Z[(layer, which)][b0:b0 + b, pos0:pos0 + t, :] = dequantize_rows(codes, scale, zp)
            else:
                self.Z[(layer, which)][b0:b0 + b, pos0:pos0 + t, :] = round_to_dtype(z, self.dtype)

    # -- steps 3+4 ----------------------------------------------------------
    def decoded_head(self, layer: int, which: int, head: int, b: int, n_ctx: int,
                     _memo: Optional[dict] = None) -> np.ndarray:
        """[n_ctx, d_head] reconstruction of one KV head as seen by `layer`."""
        src = resolve_source(self.reuse, layer, which, head)
        ae = self.ae[(src, which)]
        if head not in ae.heads:
            raise ValueError(f"layer {src} does not store head {head}")
        key = (src, which, b)
        if _memo is not None and key in _memo:
            full = _memo[key]
        else:
            full = ae.decode(self.Z[(src, which)][b, :n_ctx, :])
            if _memo is not None:
                _memo[key] = full
        i = ae.heads.index(head)
        return full[:, i * self.dh:(i + 1) * self.dh]

    # -- step 5 -------------------------------------------------------------
    def decode_attention(self, layer: int, q: np.ndarray, n_ctx: int, return_probs: bool = False,
                         seq_lens: Optional[Sequence[int]] = None,
                         k_cur: Optional[np.ndarray] = None, v_cur: Optional[np.ndarray] = None):
        """q [B, H_q, d_head] -> out [B, H_q, d_head] (fp64), attending over cached
        tokens 0..n_ctx-1 of every sequence.

        seq_lens: per-sequence context lengths (ragged batch) instead of the common n_ctx.
        k_cur, v_cur [B, H_kv*d_head]: the paper's form of the decode step ("Network
        Architecture", 2nd paragraph): the decoded rows of the cached tokens are
        concatenated with the current token's exact key and value vectors, so the
        attention runs over n cached rows plus one row that never went through the
        autoencoder.  Column block g of k_cur / v_cur is the vector KV head g of this
        layer uses (for a reused head: the source layer's)."""
        q = np.asarray(q, np.float64)
        bsz = q.shape[0]
        group = self.hq // self.hkv
        out = np.zeros((bsz, self.hq, self.dh))
        assert (k_cur is None) == (v_cur is None)
        exact = k_cur is not None
        if exact:
            k_cur = np.asarray(k_cur, np.float64)
            v_cur = np.asarray(v_cur, np.float64)
        probs = np.zeros((bsz, self.hq, n_ctx + (1 if exact else 0))) if return_probs else None
        for b in range(bsz):
            memo: dict = {}
            n = n_ctx if seq_lens is None else int(seq_lens[b])
            assert 0 <= n <= n_ctx and (n > 0 or exact)
            for j in range(self.hq):
                g = j // group
                k_hat = self.decoded_head(layer, K, g, b, n, memo)
                v_hat = self.decoded_head(layer, V, g, b, n, memo)
                if exact:
                    k_hat = np.concatenate([k_hat, k_cur[b, None, g * self.dh:(g + 1) * self.dh]], axis=0)
                    v_hat = np.concatenate([v_hat, v_cur[b, None, g * self.dh:(g + 1) * self.dh]], axis=0)
                s = (k_hat @ q[b, j]) * self.scale
                p = np.exp(s - s.max())
                p = p / p.sum()
                out[b, j] = p @ v_hat
                if return_probs:
                    probs[b, j, :p.shape[0]] = p
        return (out, probs) if return_probs else out

    # -- step 5 for a whole prompt chunk (prefill) ---------------------------
    def prefill_attention(self, layer: int, q: np.ndarray, pos0: int) -> np.ndarray:
        """Causal attention of a chunk of T query tokens over the latent cache (Introduction: the
        prefill phase processes the prompt and produces the keys and values of all its tokens,
        which are stored - here as latent rows - and read back through the decoder; Eq. 1 per
        token, each token seeing the rows up to and including its own).

        q [B, T, H_q, d_head]; query token i of a sequence sits at position pos0 + i and its own
        latent row (like every earlier one) is already in the cache.  Returns [B, T, H_q, d_head]
        (fp64):  out[b, i, j] = sum_{t <= pos0 + i} softmax_t(scale q[b,i,j] . K^_g[t]) V^_g[t]."""
        q = np.asarray(q, np.float64)
        bsz, t_new = q.shape[0], q.shape[1]
        n = pos0 + t_new
        assert pos0 >= 0 and n <= self.max_seq
        group = self.hq // self.hkv
        out = np.zeros((bsz, t_new, self.hq, self.dh))
        visible = np.arange(n)[None, :] <= (pos0 + np.arange(t_new))[:, None]      # [T, n]
        for b in range(bsz):
            memo: dict = {}
            for j in range(self.hq):
                g = j // group
                k_hat = self.decoded_head(layer, K, g, b, n, memo)
                v_hat = self.decoded_head(layer, V, g, b, n, memo)
                s = (q[b, :, j, :] @ k_hat.T) * self.scale
                s = np.where(visible, s, -np.inf)
                p = np.exp(s - s.max(axis=1, keepdims=True))
                p = p / p.sum(axis=1, keepdims=True)
                out[b, :, j, :] = p @ v_hat
        return out


# --------------------------------------------------------------------------
# reuse-map selection statistic (Algorithm 2, steps 1-2)
# --------------------------------------------------------------------------
def head_l1_distance(x_prev: np.ndarray, x_cur: np.ndarray, n_kv_heads: int, d_head: int) -> np.ndarray:
    """Mean L1 distance between the same head of adjacent layers over a batch of tokens:
    x_prev, x_cur [n_tokens, H_kv*d_head] are the keys (or the values) of layer N-1 and
    layer N; returns [H_kv].  The paper averages this over mini-batches and applies an
    empirical threshold to pick the heads that reuse the previous layer's tensor."""
    a = np.asarray(x_prev, np.float64).reshape(-1, n_kv_heads, d_head)
    b = np.asarray(x_cur, np.float64).reshape(-1, n_kv_heads, d_head)
    return np.abs(b - a).mean(axis=(0, 2))


# --------------------------------------------------------------------------
# memory accounting (Eq. 3 and the savings columns of Tables 2-4)
# --------------------------------------------------------------------------
def kv_cache_bytes(bytes_per_elem: int, n_layers: int, d_model: int, seq_len: int, batch: int) -> int:
    """Eq. 3: 2 x P x N_layers x d_model x L_seq x B."""
    return 2 * bytes_per_elem * n_layers * d_model * seq_len * batch


def latent_cache_bytes(bytes_per_elem: int, latent_widths: np.ndarray, seq_len: int, batch: int) -> int:
    """Eq. 3 with each layer's K and V width replaced by what that layer stores:
    latent_widths[N][which] elements per token."""
    return int(bytes_per_elem * int(np.asarray(latent_widths).sum()) * seq_len * batch)


def quantized_latent_cache_bytes(latent_widths: np.ndarray, seq_len: int, batch: int) -> int:
    """int8 latents: one byte per latent element plus, per stored row, the fp32 scale and
    the int32 zero point that the dequantisation of Eq. "quant" needs (8 bytes)."""
    w = np.asarray(latent_widths)
    return int((int(w.sum()) + 8 * int((w > 0).sum())) * seq_len * batch)


def savings_autoencoder(n_compressed_layers: int, n_layers: int, ratio: float) -> float:
    """Table 2: compressing n of N layers to `ratio` of their width."""
    return n_compressed_layers / n_layers * (1.0 - ratio)


def savings_reuse(n_head_tensors: int, n_layers: int, n_heads: int) -> float:
    """Table 3: reused K-or-V head tensors out of 2 x N_layers x H."""
    return n_head_tensors / (2 * n_layers * n_heads)
