"""GPU parity over a seeded sweep of shapes: head counts, head widths, latent and hidden widths, dtypes, latent
formats, reuse maps and context lengths drawn at random (fixed seed), most of them off the paths the benchmark
configurations take (latent widths that are no multiple of 32, three KV heads, sixteen query heads per KV head,
head width 96, ...).  Whatever kernel the library picks for a shape, caches and outputs must match the oracle."""
import numpy as np
import pytest

from paper_2512_06727_amd import synth
from tests.helpers import (ABS_TOL, REL_TOL, elementwise_bound, assert_cache_close, assert_outputs_close, assert_quantized_cache_close, build_oracle, oracle_prefill,
                           run_gpu, run_oracle)

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("both_groupings")]


def draw_cases(n, seed=20251206, matrix_core=False):
    rng = np.random.default_rng(seed)
    pick = lambda xs: xs[int(rng.integers(len(xs)))]
    cases = []
    for i in range(n):
        n_kv = pick([1, 2, 3, 4, 8])
        d_head = pick([32, 64, 64, 96, 128])
        group = pick([1, 2, 4, 8, 16]) if n_kv * d_head <= 512 else pick([1, 2, 4])
        dtype, fmt = pick(["bf16", "f16", "bf16", "f32"]), pick(["dtype", "dtype", "int8"])
        # a latent row (per stored head: per_head columns) must be a multiple of 16 bytes
        per_head = pick([16, 32, 48]) if fmt == "int8" else pick([8, 16, 24, 32, 40]) if dtype != "f32" else pick([4, 12, 16, 24, 32, 40])
        if matrix_core:
            # shapes the matrix-core kernels take: 16-bit dtypes, head width 64 or 128, 32 latent columns per stored head
            n_kv, d_head, per_head = pick([2, 4, 4, 8]), pick([64, 64, 128]), pick([32, 32, 16, 48])
            dtype, group = pick(["bf16", "f16"]), pick([1, 2, 4, 8])
        latent = n_kv * min(per_head, d_head)
        hidden = pick([0, 0, 128, 256]) if matrix_core else pick([0, 0, 0, 64, 96, 128])
        act = "none" if hidden == 0 else pick(["gelu", "leaky_relu"])
        w = synth.Workload(f"sweep{i}{'m' if matrix_core else ''}", n_layers=int(rng.integers(2, 4)), n_q_heads=n_kv * group, n_kv_heads=n_kv, d_head=d_head,
                           batch=int(rng.integers(1, 4)), n_cached=int(rng.integers(0, 261)), n_steps=int(rng.integers(1, 3)),
                           dtype=dtype, latent=latent, hidden=hidden, act=act,
                           reuse=pick(["none", "odd:1", "bernoulli:0.3", "bernoulli:0.6"]), policy=pick(["P1", "P1", "P2"]), seed=100 + i)
        kw = {"with_bias": bool(rng.integers(2)), "latent_format": fmt, "gain": pick([1.0, 8.0, 40.0])}
        cases.append((w, kw))
    return cases


CASES = draw_cases(36) + draw_cases(28, seed=6727, matrix_core=True)


@pytest.mark.parametrize("i", range(len(CASES)))
def test_shape_sweep(i):
    w, kw = CASES[i]
    print(f"case {i}: {w} {kw}", flush=True)
    orc, want = run_oracle(w, **kw)
    ses, got = run_gpu(w, **kw)
    n_rows = w.n_cached + w.n_steps
    if kw["latent_format"] == "int8":
        assert_quantized_cache_close(w, ses, orc, n_rows)
    else:
        assert_cache_close(w, ses, orc, n_rows)
    assert_outputs_close(w, got, want, f"sweep {i}")


def check(w, got, want, label):
    """Absolute tolerance plus half a unit in the last place of the reference (outputs of O(1) where the exact current
    row or a single value row dominates carry the rounding of the result to the dtype)."""
    assert got.shape == want.shape and np.isfinite(got).all(), label
    err = np.abs(got - want)
    worst = (err - elementwise_bound(want, w.dtype)).max()
    assert worst <= 0, f"{label}: error exceeds abs tol + half an ulp by {worst:.3e}"
    assert err.max() <= REL_TOL[w.dtype] * np.abs(want).max(), f"{label}: err {err.max():.3e} vs max |ref| {np.abs(want).max():.3e}"


def oracle_side(w, kw):
    """Oracle with the prompt cached; expected outputs of the last layer for (a) a decode step with ragged context
    lengths (one sequence empty when there are several) and the exact current row, (b) prefill attention over the prompt."""
    okw = {"with_bias": kw["with_bias"], "latent_format": kw["latent_format"]}
    orc = build_oracle(w, **okw)
    for n in range(w.n_layers):
        oracle_prefill(orc, w, n, 0, w.n_cached)
    layer = w.n_layers - 1
    rng = np.random.default_rng(w.seed)
    lens = rng.integers(0, w.n_cached + 1, size=w.batch)
    lens[0] = w.n_cached
    if w.batch > 1:
        lens[-1] = 0
    q = synth.queries(w, layer, 0, gain=kw["gain"])
    kc = synth.kv_tokens(w, layer, 0, 0, w.batch, w.n_cached, w.n_cached + 1)[:, 0]
    vc = synth.kv_tokens(w, layer, 1, 0, w.batch, w.n_cached, w.n_cached + 1)[:, 0]
    want_step = orc.decode_attention(layer, q.double().numpy(), w.n_cached, seq_lens=lens, k_cur=kc.double().numpy(), v_cur=vc.double().numpy())
    qp = want_pre = None
    if w.n_cached >= 1:
        qp = synth.prompt_queries(w, layer, 0, w.batch, 0, w.n_cached, gain=kw["gain"])
        want_pre = orc.prefill_attention(layer, qp.double().numpy(), 0)
    return okw, layer, lens, q, kc, vc, want_step, qp, want_pre


@pytest.mark.parametrize("i", range(len(CASES)))
def test_shape_sweep_variants_and_prefill(i):
    import torch
    from paper_2512_06727_amd.harness import Session
    w, kw = CASES[i]
    print(f"case {i}: {w} {kw}", flush=True)
    okw, layer, lens, q, kc, vc, want_step, qp, want_pre = oracle_side(w, kw)
    ses = Session(w, poison=True, **okw)
    ses.prefill(0, w.n_cached, chunk=256)
    dev = lambda t: t.to(ses.dev, ses.tdt).contiguous()
    qd = dev(q)
    out = torch.empty_like(qd)
    ses.ensure_workspace(w.batch, max(1, w.n_cached))
    ses.ctx.decode_attention_ex(layer, qd, out, w.batch, w.n_cached, ses.workspace, k_cur=dev(kc), v_cur=dev(vc),
                                seq_lens=torch.tensor(lens, dtype=torch.int32, device=ses.dev))
    check(w, out.float().cpu().double().numpy(), want_step, f"sweep {i} ragged + exact row, lens {lens.tolist()}")
    if qp is not None:
        cut = w.n_cached // 3
        parts = [ses.prefill_attention(layer, dev(qp[:, a:b]), a) for a, b in ((0, cut), (cut, w.n_cached)) if b > a]
        got = torch.cat(parts, dim=1).float().cpu().double().numpy()
        check(w, got, want_pre, f"sweep {i} prefill")
