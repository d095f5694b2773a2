"""Plumbing between a synthetic workload and the library: allocates caches, weights and
workspace as PyTorch tensors on the GPU and drives the C ABI.  No arithmetic of the method
lives here."""
from __future__ import annotations

from typing import List, Optional

import numpy as np
import torch

from . import binding, synth


# Most query heads per attention workgroup that a Session asks for when its caller names none (0 = the library chooses;
# tests set 32 to reach the widest form of the kernels with the small batches they run).
default_group_slots = 0


class Session:
    def __init__(self, w: synth.Workload, reuse: Optional[np.ndarray] = None, with_bias: bool = False,
                 device: str = "cuda:0", n_splits: int = 0, force_generic: bool = False, tile_order: int = 0, no_fuse: bool = False, poison: bool = False,
                 max_batch: Optional[int] = None, latent_format: str = "dtype", wg_waves: int = 0, no_bulk_encode: bool = False, no_arrive: bool = False,
                 per_head: bool = False, group_slots: Optional[int] = None, no_colocate: bool = False):
        """per_head: every KV head has an autoencoder d_head -> latent / H_kv -> d_head of its own (the library's
        per_head descriptor flag); head g's weights and activations are those of per_head_workloads(w)[g]."""
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: libkvcar has no CPU path")
        self.w = w
        self.per_head = per_head
        self.poison = poison
        self.dev = torch.device(device)
        self.tdt = synth.TORCH_DTYPE[w.dtype]
        self.reuse = synth.reuse_map(w) if reuse is None else reuse
        self.latent_format = latent_format
        self.ctx = binding.Context(w.n_layers, w.n_q_heads, w.n_kv_heads, w.d_head, max_batch or w.batch, w.max_seq, w.dtype,
                                   latent_format=latent_format)
        self.ctx.set_tuning(n_splits=n_splits, force_generic=force_generic, tile_order=tile_order, no_fuse=no_fuse, wg_waves=wg_waves, no_bulk_encode=no_bulk_encode, no_arrive=no_arrive,
                            group_slots=default_group_slots if group_slots is None else group_slots, no_colocate=no_colocate)
        self.ae: List[List[synth.AEWeights]] = []
        self.caches: List[List[Optional[torch.Tensor]]] = []
        for layer in range(w.n_layers):
            self.ctx.set_reuse_map(layer, self.reuse[layer, 0], self.reuse[layer, 1])
        self.parts = per_head_workloads(w, self.reuse) if per_head else None
        for layer in range(w.n_layers):
            row, crow = [], []
            for which in (0, 1):
                ae = self.stacked_autoencoder(layer, which, with_bias) if per_head else synth.autoencoder(w, layer, which, self.reuse, with_bias)
                up = lambda pairs: [(wt.to(self.dev, self.tdt).contiguous(), None if b is None else b.to(self.dev, self.tdt).contiguous())
                                    for wt, b in pairs]
                enc, dec = up(ae.enc), up(ae.dec)
                self.ctx.set_autoencoder(layer, which, len(ae.heads) * w.d_head if per_head else ae.width, ae.hidden if ae.heads else 0, ae.latent,
                                         ae.act if ae.heads else "none", enc, dec, ae.slope, per_head=per_head and bool(ae.heads))
                nbytes = self.ctx.cache_bytes(layer, which)
                cache = None
                if nbytes and latent_format == "int8":
                    cache = torch.empty(nbytes, dtype=torch.uint8, device=self.dev)
                    if poison:
                        cache.fill_(0x7F)
                    self.ctx.bind_cache(layer, which, cache)
                elif nbytes:
                    n = nbytes // synth.DTYPE_BYTES[w.dtype]
                    cache = torch.empty(n, dtype=self.tdt, device=self.dev)
                    if poison:
                        cache.fill_(float("nan"))
                    self.ctx.bind_cache(layer, which, cache)
                row.append(ae)
                crow.append(cache)
            self.ae.append(row)
            self.caches.append(crow)
        self.workspace = None
        self._ws_key = None

    # ------------------------------------------------------------------
    def stacked_autoencoder(self, layer: int, which: int, with_bias: bool) -> synth.AEWeights:
        """Per-head autoencoders of one layer-tensor in the library's layout: the stored heads' matrices one after the
        other, enc [n][d_head][r_h], dec [n][r_h][d_head], biases concatenated (pure data movement)."""
        stored = [g for g in range(self.w.n_kv_heads) if not self.reuse[layer, which, g]]
        aes = [synth.autoencoder(self.parts[g][0], layer, which, self.parts[g][1], with_bias) for g in stored]
        if not stored:
            empty = torch.zeros(0, 0)
            return synth.AEWeights([], 0, 0, "none", 0.01, [(empty, None)], [(empty, None)])
        cat = lambda vs: torch.cat(list(vs)) if with_bias else None
        enc = [(torch.stack([a.enc[0][0] for a in aes]), cat(a.enc[0][1] for a in aes))]
        dec = [(torch.stack([a.dec[0][0] for a in aes]), cat(a.dec[0][1] for a in aes))]
        return synth.AEWeights(stored, sum(a.latent for a in aes), 0, "none", 0.01, enc, dec)

    def kv(self, layer: int, which: int, t0: int, t1: int) -> torch.Tensor:
        """Synthetic keys (which = 0) or values [batch, t1 - t0, D_kv] of positions [t0, t1); per-head sessions: head g's
        columns are the stream of per_head_workloads(w)[g]."""
        w = self.w
        if not self.per_head:
            return synth.kv_tokens(w, layer, which, 0, w.batch, t0, t1, device=self.dev).to(self.tdt)
        return torch.cat([synth.kv_tokens(wg, layer, which, 0, w.batch, t0, t1, device=self.dev) for wg, _ in self.parts], dim=2).to(self.tdt)

    def queries(self, layer: int, step: int, gain: float = 1.0) -> torch.Tensor:
        """Synthetic decode queries [batch, H_q, d_head] (per-head sessions: head g's query heads from its own stream)."""
        if not self.per_head:
            return synth.queries(self.w, layer, step, device=self.dev, gain=gain).to(self.tdt)
        return torch.cat([synth.queries(wg, layer, step, device=self.dev, gain=gain) for wg, _ in self.parts], dim=1).to(self.tdt)

    def cache_view(self, layer: int, which: int) -> Optional[torch.Tensor]:
        """[max_batch, max_seq, r] view of a latent cache (the documented layout); per-head autoencoders: the heads'
        blocks [n_stored_heads][max_batch][max_seq][r_h] gathered side by side into rows of the same shape (a copy)."""
        c = self.caches[layer][which]
        if c is None:
            return None
        if self.latent_format == "int8":
            raise RuntimeError("int8 latents: use quantized_view")
        ae = self.ae[layer][which]
        if self.per_head:
            n, mb, ms = len(ae.heads), self.ctx.cfg.max_batch, self.w.max_seq
            return c.view(n, mb, ms, ae.latent // n).permute(1, 2, 0, 3).reshape(mb, ms, ae.latent)
        return c.view(self.ctx.cfg.max_batch, self.w.max_seq, ae.latent)

    def quantized_view(self, layer: int, which: int):
        """int8 latents: (codes int8 [max_batch, max_seq, r], scale fp32 [max_batch, max_seq],
        zeropoint int32 [max_batch, max_seq]) views of one cache buffer (the documented layout)."""
        c = self.caches[layer][which]
        if c is None:
            return None
        mb, ms, r = self.ctx.cfg.max_batch, self.w.max_seq, self.ae[layer][which].latent
        n = mb * ms * r
        off = (n + 255) // 256 * 256
        codes = c[:n].view(torch.int8).view(mb, ms, r)
        meta = c[off:off + mb * ms * 8]
        return codes, meta.view(torch.float32).view(mb, ms, 2)[..., 0], meta.view(torch.int32).view(mb, ms, 2)[..., 1]

    def ensure_workspace(self, batch: int, n_ctx: int):
        need = self.ctx.workspace_bytes(batch, n_ctx)
        if self.workspace is None or self.workspace.numel() < need:
            self.workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=self.dev)
            if self.poison:                      # the library must not rely on anything a workspace holds
                self.workspace.random_(0, 256)

    def encode_append(self, layer: int, k_new: torch.Tensor, v_new: torch.Tensor, pos0: int):
        b, t, _ = k_new.shape
        self.ctx.encode_append(layer, k_new, v_new, b, pos0, t)

    def prefill(self, t0: int, t1: int, chunk: int = 512, layers=None):
        """Encode+append synthetic K/V for positions [t0, t1) of every sequence."""
        w = self.w
        for layer in (range(w.n_layers) if layers is None else layers):
            for c0 in range(t0, t1, chunk):
                c1 = min(t1, c0 + chunk)
                self.encode_append(layer, self.kv(layer, 0, c0, c1), self.kv(layer, 1, c0, c1), c0)

    def decode_attention(self, layer: int, q: torch.Tensor, n_ctx: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        b = q.shape[0]
        self.ensure_workspace(b, n_ctx)
        if out is None:
            out = torch.empty_like(q)
        self.ctx.decode_attention(layer, q, out, b, n_ctx, self.workspace)
        return out

    def append_attend(self, layer: int, k_new: torch.Tensor, v_new: torch.Tensor, q: torch.Tensor, pos: int,
                      out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """One decode step of a layer: k_new, v_new [batch, 1, D_kv] are encoded and appended at `pos`, q attends over rows 0 .. pos."""
        b = q.shape[0]
        self.ensure_workspace(b, pos + 1)
        if out is None:
            out = torch.empty_like(q)
        self.ctx.append_attend(layer, k_new, v_new, q, out, b, pos, self.workspace)
        return out

    def prefill_attention(self, layer: int, q: torch.Tensor, pos0: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """q [batch, t_new, H_q, d_head]: causal attention of the chunk at positions pos0.. over the caches."""
        b, t = q.shape[0], q.shape[1]
        need = self.ctx.prefill_workspace_bytes(b, pos0 + t)
        if getattr(self, "prefill_ws", None) is None or self.prefill_ws.numel() < need:
            self.prefill_ws = torch.empty(need, dtype=torch.uint8, device=self.dev)
        if out is None:
            out = torch.empty_like(q)
        self.ctx.prefill_attention(layer, q, out, b, pos0, t, self.prefill_ws)
        return out


def per_head_workloads(w: synth.Workload, reuse: Optional[np.ndarray] = None):
    """The per-head (block-diagonal) autoencoder variant of a workload: every KV head has its own autoencoder
    d_head -> latent / H_kv -> d_head and its own latent rows, so the model splits into H_kv independent
    single-KV-head models.  Returns [(workload of head g, its reuse map [n_layers, 2, 1])]; head g's weights
    and activations come from seed streams of their own."""
    reuse = synth.reuse_map(w) if reuse is None else reuse
    gq = w.n_q_heads // w.n_kv_heads
    return [(w.scaled(name=f"{w.name}-head{g}", n_q_heads=gq, n_kv_heads=1, latent=w.latent // w.n_kv_heads,
                      seed=w.seed + 7919 * (g + 1), reuse="none"), reuse[:, :, g:g + 1].copy())
            for g in range(w.n_kv_heads)]


class PerHeadSessions:
    """One library context per KV head (the per-head autoencoder variant): a head that reuses the previous
    layer's keys or values reads only that head's rows of the source layer, so reuse adds no cache traffic."""

    def __init__(self, w: synth.Workload, reuse: Optional[np.ndarray] = None, **session_kw):
        self.w = w
        self.parts = per_head_workloads(w, reuse)
        self.sessions = [Session(wg, reuse=rg, **session_kw) for wg, rg in self.parts]

    def prefill(self, t0: int, t1: int, **kw):
        for s in self.sessions:
            s.prefill(t0, t1, **kw)

    def decode_attention(self, layer: int, qs, n_ctx: int):
        """qs: one [batch, H_q / H_kv, d_head] tensor per KV head; returns [batch, H_q, d_head]."""
        return torch.cat([s.decode_attention(layer, q, n_ctx) for s, q in zip(self.sessions, qs)], dim=1)
