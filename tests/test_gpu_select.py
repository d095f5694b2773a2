"""Reuse-map selection statistic on the GPU (Algorithm 2, steps 1-2) against the oracle."""
import numpy as np
import pytest
import torch

from oracle import kvcar_oracle as O
from paper_2512_06727_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = {"f32": 2e-6, "f16": 2e-6, "bf16": 2e-6}      # inputs are exact in their dtype; fp32 partial sums, fp64 final sum


def layer_pair(w, which, n_tokens, layer):
    per = -(-n_tokens // w.batch)
    a = synth.kv_tokens(w, layer - 1, which, 0, w.batch, 0, per).reshape(-1, w.d_kv)[:n_tokens]
    b = synth.kv_tokens(w, layer, which, 0, w.batch, 0, per).reshape(-1, w.d_kv)[:n_tokens]
    return a, b


@pytest.mark.parametrize("cfg,n_tokens", [(0, 1), (0, 37), (1, 1000), (2, 5), (2, 4099), (2, 70000), (4, 30001)])
def test_l1_distance_matches_oracle(cfg, n_tokens):
    w = synth.CONFIGS[cfg]
    tdt = synth.TORCH_DTYPE[w.dtype]
    for which in (0, 1):
        a, b = layer_pair(w, which, n_tokens, 1)
        a, b = a.to(tdt), b.to(tdt)
        want = O.head_l1_distance(a.double().numpy(), b.double().numpy(), w.n_kv_heads, w.d_head)
        got = binding.head_l1_distance(a.to(DEV), b.to(DEV), w.n_kv_heads, w.d_head).cpu().double().numpy()
        np.testing.assert_allclose(got, want, rtol=TOL[w.dtype], atol=0)


def test_l1_distance_special_cases_and_accumulation():
    w = synth.CONFIGS[2]
    a, b = layer_pair(w, 0, 3000, 3)
    a, b = a.to(torch.bfloat16).to(DEV), b.to(torch.bfloat16).to(DEV)
    assert (binding.head_l1_distance(a, a, w.n_kv_heads, w.d_head) == 0).all()
    c = a.clone()
    c[:, w.d_head:2 * w.d_head] = 0                      # head 1 of the second tensor zeroed: distance = mean |a| of head 1
    got = binding.head_l1_distance(a, c, w.n_kv_heads, w.d_head).cpu().numpy()
    assert got[0] == 0 and got[2] == 0 and got[3] == 0
    np.testing.assert_allclose(got[1], a[:, w.d_head:2 * w.d_head].float().abs().double().mean().item(), rtol=2e-6)
    # two mini-batches accumulated, then averaged = the statistic of the whole batch (equal sizes)
    dist = binding.head_l1_distance(a[:1500], b[:1500], w.n_kv_heads, w.d_head)
    binding.head_l1_distance(a[1500:], b[1500:], w.n_kv_heads, w.d_head, dist=dist, accumulate=True)
    whole = binding.head_l1_distance(a, b, w.n_kv_heads, w.d_head)
    np.testing.assert_allclose((dist / 2).cpu().numpy(), whole.cpu().numpy(), rtol=1e-6)
    # repeated calls give the same bits (fixed reduction order)
    again = binding.head_l1_distance(a, b, w.n_kv_heads, w.d_head)
    assert torch.equal(whole, again)


def test_l1_distance_argument_errors():
    lib = binding.lib()
    import ctypes as C
    x = torch.zeros(64, 256, dtype=torch.bfloat16, device=DEV)
    d = torch.zeros(4, dtype=torch.float32, device=DEV)
    ws = torch.zeros(1 << 16, dtype=torch.uint8, device=DEV)
    call = lambda *a: lib.kvcar_head_l1_distance(*a)
    p = lambda t: C.c_void_p(t.data_ptr())
    assert call(None, p(x), binding.BF16, 64, 4, 64, 0, p(d), p(ws), ws.numel(), None) == binding.ERR_ARG
    assert call(p(x), p(x), binding.BF16, 0, 4, 64, 0, p(d), p(ws), ws.numel(), None) == binding.ERR_ARG
    assert call(p(x), p(x), 7, 64, 4, 64, 0, p(d), p(ws), ws.numel(), None) == binding.ERR_UNSUPPORTED
    assert call(p(x), p(x), binding.BF16, 64, 64, 4, 0, p(d), p(ws), ws.numel(), None) == binding.ERR_SHAPE
    assert call(p(x), p(x), binding.BF16, 64, 4, 64, 0, p(d), p(ws), 8, None) == binding.ERR_WORKSPACE
    torch.cuda.synchronize()
