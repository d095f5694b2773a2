"""ctypes binding over libkvcar.so (C ABI in include/kvcar.h).

Argument marshalling only: every step of the path runs inside the library's HIP
kernels.  PyTorch supplies device memory and the stream.  A missing library is an
error; there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libkvcar.so")

OK = 0
ENC_NONE, ENC_PLAIN, ENC_MFMA, ENC_MFMA_TWO_LAYER, ENC_MFMA_STREAM = range(5)
ERR_ARG, ERR_SHAPE, ERR_CAPACITY, ERR_REUSE, ERR_UNSUPPORTED, ERR_STATE, ERR_HIP, ERR_WORKSPACE, ERR_NOMEM = range(-1, -10, -1)
F32, F16, BF16 = 0, 1, 2
STATIC_SCRATCH_BYTES = 32 << 20         # KVCAR_STATIC_SCRATCH_BYTES
ACT_NONE, ACT_LEAKY_RELU, ACT_GELU = 0, 1, 2
K, V = 0, 1

DTYPES = {"f32": F32, "f16": F16, "bf16": BF16}
ACTS = {"none": ACT_NONE, "leaky_relu": ACT_LEAKY_RELU, "gelu": ACT_GELU}
LATENT_FORMATS = {"dtype": 0, "int8": 1}


class Config(C.Structure):
    _fields_ = [("n_layers", C.c_int), ("n_q_heads", C.c_int), ("n_kv_heads", C.c_int), ("d_head", C.c_int),
                ("max_batch", C.c_int), ("max_seq", C.c_int), ("dtype", C.c_int), ("softmax_scale", C.c_float),
                ("latent_format", C.c_int)]


class AEDesc(C.Structure):
    _fields_ = [("in_width", C.c_int), ("hidden_width", C.c_int), ("latent_width", C.c_int), ("act", C.c_int),
                ("leaky_slope", C.c_float),
                ("enc_w1", C.c_void_p), ("enc_b1", C.c_void_p), ("enc_w2", C.c_void_p), ("enc_b2", C.c_void_p),
                ("dec_w1", C.c_void_p), ("dec_b1", C.c_void_p), ("dec_w2", C.c_void_p), ("dec_b2", C.c_void_p),
                ("per_head", C.c_int)]


class Tuning(C.Structure):
    _fields_ = [("n_splits", C.c_int), ("force_generic", C.c_int), ("tile_order", C.c_int), ("no_fuse", C.c_int), ("wg_waves", C.c_int), ("no_bulk_encode", C.c_int), ("no_arrive", C.c_int), ("no_colocate", C.c_int), ("group_slots", C.c_int)]


class StepExt(C.Structure):
    _fields_ = [("seq_lens", C.c_void_p), ("k_cur", C.c_void_p), ("v_cur", C.c_void_p)]


class PlanInfo(C.Structure):
    _fields_ = [("uses_mfma", C.c_int), ("n_groups", C.c_int), ("n_splits", C.c_int), ("n_launches", C.c_int), ("fused", C.c_int),
                ("workspace_bytes", C.c_size_t), ("latent_bytes", C.c_size_t), ("append_in_kernel", C.c_int)]


# every symbol include/kvcar.h declares: name -> (restype, argtypes)
SYMBOLS = {
    "kvcar_create": (C.c_int, [C.POINTER(Config), C.POINTER(C.c_void_p)]),
    "kvcar_destroy": (C.c_int, [C.c_void_p]),
    "kvcar_set_reuse_map": (C.c_int, [C.c_void_p, C.c_int, C.c_char_p, C.c_char_p]),
    "kvcar_resolve_source": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int)]),
    "kvcar_set_autoencoder": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.POINTER(AEDesc)]),
    "kvcar_cache_bytes": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_size_t)]),
    "kvcar_bind_cache": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_size_t]),
    "kvcar_set_tuning": (C.c_int, [C.c_void_p, C.POINTER(Tuning)]),
    "kvcar_workspace_bytes": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_size_t)]),
    "kvcar_encode_append": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]),
    "kvcar_decode_attention": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p,
                                         C.c_size_t, C.c_void_p]),
    "kvcar_decode_attention_ex": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.POINTER(StepExt), C.c_void_p,
                                            C.c_size_t, C.c_void_p]),
    "kvcar_decode_attention_static": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]),
    "kvcar_append_attend": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_size_t,
                                      C.c_void_p]),
    "kvcar_encode_append_at": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p]),
    "kvcar_describe_encode": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int)]),
    "kvcar_prefill_workspace_bytes": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_size_t)]),
    "kvcar_prefill_attention": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_size_t,
                                          C.c_void_p]),
    "kvcar_describe_plan": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.POINTER(PlanInfo)]),
    "kvcar_profile_enable": (C.c_int, [C.c_void_p, C.c_int]),
    "kvcar_profile_read": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_long)]),
    "kvcar_head_l1_workspace_bytes": (C.c_int, [C.c_size_t, C.c_int, C.POINTER(C.c_size_t)]),
    "kvcar_head_l1_distance": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, C.c_size_t, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                         C.c_size_t, C.c_void_p]),
    "kvcar_probe_read_bandwidth": (C.c_int, [C.c_void_p, C.c_size_t, C.c_int, C.c_void_p, C.POINTER(C.c_double)]),
    "kvcar_status_string": (C.c_char_p, [C.c_int]),
    "kvcar_last_error": (C.c_char_p, [C.c_void_p]),
}

_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    """Open libkvcar.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2512_06727_amd.build`")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(l, name)
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib


class KVCARError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{lib().kvcar_status_string(status).decode()}: {text}")
        self.status = status


def _ptr(t) -> Optional[int]:
    """Raw address of a tensor (None -> NULL)."""
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream() -> C.c_void_p:
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def head_l1_distance(x_prev, x_cur, n_kv_heads: int, d_head: int, dist=None, accumulate: bool = False, workspace=None):
    """kvcar_head_l1_distance on two [n_tokens, n_kv_heads * d_head] tensors; returns the fp32 tensor
    dist [n_kv_heads] (allocated here unless given).  Marshalling only."""
    import torch
    n_tokens = x_prev.numel() // (n_kv_heads * d_head)
    dt = {torch.float32: F32, torch.float16: F16, torch.bfloat16: BF16}[x_prev.dtype]
    need = C.c_size_t(0)
    st = lib().kvcar_head_l1_workspace_bytes(n_tokens, n_kv_heads, C.byref(need))
    if st != 0:
        raise KVCARError(st, "kvcar_head_l1_workspace_bytes")
    if workspace is None:
        workspace = torch.empty(max(need.value, 16), dtype=torch.uint8, device=x_prev.device)
    if dist is None:
        dist = torch.zeros(n_kv_heads, dtype=torch.float32, device=x_prev.device)
    st = lib().kvcar_head_l1_distance(_ptr(x_prev), _ptr(x_cur), dt, n_tokens, n_kv_heads, d_head, 1 if accumulate else 0, _ptr(dist),
                                      _ptr(workspace), workspace.numel(), _stream())
    if st != 0:
        raise KVCARError(st, "kvcar_head_l1_distance")
    return dist


def probe_read_bandwidth(buf, repeats: int = 8) -> float:
    """GB/s of a read-only sweep over the tensor `buf` (kvcar_probe_read_bandwidth)."""
    out = C.c_double(0.0)
    st = lib().kvcar_probe_read_bandwidth(_ptr(buf), buf.numel() * buf.element_size(), repeats, _stream(), C.byref(out))
    if st != 0:
        raise KVCARError(st, "kvcar_probe_read_bandwidth")
    return out.value


class Context:
    """Thin owner of a kvcar_ctx.  Methods mirror the C entry points one to one."""

    def __init__(self, n_layers: int, n_q_heads: int, n_kv_heads: int, d_head: int, max_batch: int, max_seq: int,
                 dtype: str, softmax_scale: float = 0.0, latent_format: str = "dtype"):
        self._h = C.c_void_p()
        cfg = Config(n_layers, n_q_heads, n_kv_heads, d_head, max_batch, max_seq, DTYPES[dtype], softmax_scale,
                     LATENT_FORMATS[latent_format])
        st = lib().kvcar_create(C.byref(cfg), C.byref(self._h))
        if st != OK:
            raise KVCARError(st, "kvcar_create")
        self.cfg = cfg
        self._keep = []          # tensors whose memory the context points at

    def close(self):
        if self._h:
            lib().kvcar_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != OK:
            raise KVCARError(st, lib().kvcar_last_error(self._h).decode())

    def set_reuse_map(self, layer: int, k_reuse: Sequence[bool], v_reuse: Sequence[bool]):
        kb = bytes(1 if x else 0 for x in k_reuse)
        vb = bytes(1 if x else 0 for x in v_reuse)
        self._check(lib().kvcar_set_reuse_map(self._h, layer, kb, vb))

    def resolve_source(self, layer: int, which: int, kv_head: int) -> int:
        out = C.c_int(-1)
        self._check(lib().kvcar_resolve_source(self._h, layer, which, kv_head, C.byref(out)))
        return out.value

    def set_autoencoder(self, layer: int, which: int, in_width: int, hidden_width: int, latent_width: int, act: str,
                        enc, dec, leaky_slope: float = 0.01, per_head: bool = False):
        """enc / dec: lists of (weight tensor, bias tensor or None) on the device."""
        d = AEDesc()
        d.per_head = 1 if per_head else 0
        d.in_width, d.hidden_width, d.latent_width, d.act, d.leaky_slope = in_width, hidden_width, latent_width, ACTS[act], leaky_slope
        names = [("enc_w1", "enc_b1"), ("enc_w2", "enc_b2")]
        for (wn, bn), (w, b) in zip(names, enc):
            setattr(d, wn, _ptr(w)); setattr(d, bn, _ptr(b))
        names = [("dec_w1", "dec_b1"), ("dec_w2", "dec_b2")]
        for (wn, bn), (w, b) in zip(names, dec):
            setattr(d, wn, _ptr(w)); setattr(d, bn, _ptr(b))
        self._keep.append((enc, dec))
        self._check(lib().kvcar_set_autoencoder(self._h, layer, which, C.byref(d)))

    def cache_bytes(self, layer: int, which: int) -> int:
        n = C.c_size_t(0)
        self._check(lib().kvcar_cache_bytes(self._h, layer, which, C.byref(n)))
        return n.value

    def bind_cache(self, layer: int, which: int, tensor):
        self._keep.append(tensor)
        nbytes = 0 if tensor is None else tensor.numel() * tensor.element_size()
        self._check(lib().kvcar_bind_cache(self._h, layer, which, _ptr(tensor), nbytes))

    def set_tuning(self, n_splits: int = 0, force_generic: bool = False, tile_order: int = 0, no_fuse: bool = False,
                   wg_waves: int = 0, no_bulk_encode: bool = False, no_arrive: bool = False, group_slots: int = 0,
                   no_colocate: bool = False):
        t = Tuning(n_splits, 1 if force_generic else 0, tile_order, 1 if no_fuse else 0, wg_waves, 1 if no_bulk_encode else 0, 1 if no_arrive else 0,
                   1 if no_colocate else 0, group_slots)
        self._check(lib().kvcar_set_tuning(self._h, C.byref(t)))

    def describe_encode(self, layer: int, batch: int, t_new: int) -> int:
        """The encoder kernel an encode_append call of this size takes (one of the ENC_* values)."""
        k = C.c_int(0)
        self._check(lib().kvcar_describe_encode(self._h, layer, batch, t_new, C.byref(k)))
        return k.value

    def workspace_bytes(self, batch: int, n_ctx: int) -> int:
        n = C.c_size_t(0)
        self._check(lib().kvcar_workspace_bytes(self._h, batch, n_ctx, C.byref(n)))
        return n.value

    def describe_plan(self, layer: int, batch: int, n_ctx: int) -> PlanInfo:
        info = PlanInfo()
        self._check(lib().kvcar_describe_plan(self._h, layer, batch, n_ctx, C.byref(info)))
        return info

    def profile_enable(self, enable: bool):
        self._check(lib().kvcar_profile_enable(self._h, 1 if enable else 0))

    def profile_read(self):
        """(summed attention-kernel milliseconds, launches) since the last read; blocks on the events."""
        ms, n = C.c_double(0.0), C.c_long(0)
        self._check(lib().kvcar_profile_read(self._h, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def encode_append(self, layer: int, k_new, v_new, batch: int, pos0: int, t_new: int):
        self._check(lib().kvcar_encode_append(self._h, layer, _ptr(k_new), _ptr(v_new), batch, pos0, t_new, _stream()))

    def encode_append_at(self, layer: int, k_new, v_new, batch: int, positions, t_new: int):
        """positions: int32 device tensor [batch]."""
        self._check(lib().kvcar_encode_append_at(self._h, layer, _ptr(k_new), _ptr(v_new), batch, _ptr(positions), t_new, _stream()))

    def decode_attention_ex(self, layer: int, q, out, batch: int, n_ctx: int, workspace, seq_lens=None, k_cur=None, v_cur=None):
        """seq_lens: int32 device tensor [batch] or None; k_cur, v_cur: [batch, D_kv] tensors or None."""
        nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        ext = StepExt(None if seq_lens is None else seq_lens.data_ptr(), None if k_cur is None else k_cur.data_ptr(),
                      None if v_cur is None else v_cur.data_ptr())
        self._check(lib().kvcar_decode_attention_ex(self._h, layer, _ptr(q), _ptr(out), batch, n_ctx, C.byref(ext), _ptr(workspace),
                                                    nbytes, _stream()))

    def decode_attention(self, layer: int, q, out, batch: int, n_ctx: int, workspace):
        nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        self._check(lib().kvcar_decode_attention(self._h, layer, _ptr(q), _ptr(out), batch, n_ctx, _ptr(workspace),
                                                 nbytes, _stream()))

    def append_attend(self, layer: int, k_new, v_new, q, out, batch: int, pos: int, workspace):
        """kvcar_append_attend: encode + append the new token at `pos`, then attend over rows 0 .. pos."""
        nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        self._check(lib().kvcar_append_attend(self._h, layer, _ptr(k_new), _ptr(v_new), _ptr(q), _ptr(out), batch, pos, _ptr(workspace), nbytes,
                                              _stream()))

    def decode_attention_static(self, layer: int, q, out, batch: int, n_ctx: int):
        """kvcar_decode_attention on the library's own static scratch buffer (no workspace, no allocation)."""
        self._check(lib().kvcar_decode_attention_static(self._h, layer, _ptr(q), _ptr(out), batch, n_ctx, _stream()))

    def prefill_workspace_bytes(self, batch: int, n_rows: int) -> int:
        n = C.c_size_t(0)
        self._check(lib().kvcar_prefill_workspace_bytes(self._h, batch, n_rows, C.byref(n)))
        return n.value

    def prefill_attention(self, layer: int, q, out, batch: int, pos0: int, t_new: int, workspace):
        """q, out: [batch, t_new, H_q, d_head] device tensors."""
        nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        self._check(lib().kvcar_prefill_attention(self._h, layer, _ptr(q), _ptr(out), batch, pos0, t_new, _ptr(workspace), nbytes, _stream()))
