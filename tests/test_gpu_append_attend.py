"""kvcar_append_attend: the layer's whole decode step (encode the new token, append, attend over the cache including the
new row) in one call - where the shapes allow, in one kernel - against the oracle's encode_append + decode_attention, step
after step, caches included."""
import numpy as np
import pytest
import torch

from paper_2512_06727_amd import synth
from paper_2512_06727_amd.harness import Session
from tests.helpers import assert_cache_close, assert_outputs_close, assert_quantized_cache_close, run_oracle

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("both_groupings")]

C = synth.CONFIGS
ALL_K_REUSED = np.zeros((3, 2, 4), dtype=bool)
ALL_K_REUSED[1, 0, 1] = ALL_K_REUSED[1, 1, 2] = True
ALL_K_REUSED[2, 0, :] = True
CASES = {
    # name: (workload, oracle / session keywords, session-only keywords, in-kernel encoder expected)
    # TinyLlama shape with a reuse chain: several splits, the last workgroup to arrive merges
    "tinyllama-splits": (C[2].scaled(n_layers=5, batch=3, n_cached=301, n_steps=3), {}, {}, True),
    # context ending exactly on a tile boundary / one token into a tile / a single cached token
    "tile-boundary": (C[2].scaled(n_layers=3, batch=2, n_cached=255, n_steps=3), {}, {}, True),
    "nothing-cached": (C[2].scaled(n_layers=3, batch=2, n_cached=0, n_steps=3), {}, {}, True),
    # Bernoulli map: layers storing 0 .. 4 heads (a layer may store nothing), groups of mixed widths, biases
    "bernoulli-bias": (C[4].scaled(n_layers=8, batch=2, n_cached=333, n_steps=2), {"with_bias": True}, {}, True),
    "bernoulli-p2": (C[4].scaled(n_layers=6, batch=2, n_cached=150, n_steps=2, policy="P2"), {}, {}, True),
    # one split: the fused kernel, four and eight waves
    "one-split-w4": (C[4].scaled(n_layers=6, batch=2, n_cached=200, n_steps=2), {}, {"n_splits": 1, "wg_waves": 4}, True),
    "one-split-w8": (C[4].scaled(n_layers=6, batch=2, n_cached=200, n_steps=2), {}, {"n_splits": 1, "wg_waves": 8}, True),
    # several splits in one launch with eight waves per workgroup, against the same with four; five splits of 602 tokens
    # leave two eight-wave splits without a tile
    "splits-w8": (C[4].scaled(n_layers=6, batch=2, n_cached=700, n_steps=2), {"with_bias": True}, {"n_splits": 3, "wg_waves": 8}, True),
    "splits-w4": (C[4].scaled(n_layers=6, batch=2, n_cached=700, n_steps=2), {"with_bias": True}, {"n_splits": 3, "wg_waves": 4}, True),
    "tinyllama-empty-splits-w8": (C[2].scaled(n_layers=5, batch=3, n_cached=601, n_steps=3), {}, {"n_splits": 5, "wg_waves": 8}, True),
    # head width 128, fp16
    "dh128-f16": (C[2].scaled(n_layers=3, batch=2, n_cached=300, n_steps=2, n_q_heads=16, n_kv_heads=2, d_head=128, latent=64, policy="P2",
                              reuse="odd:1", dtype="f16"), {"with_bias": True}, {}, True),
    # shapes the in-kernel encoder does not take: the call falls back to the two launches
    "gpt2-f16": (C[1].scaled(n_layers=3, batch=2, n_cached=150, n_steps=2), {}, {}, False),
    "two-layer": (C[3].scaled(n_layers=2, batch=2, n_cached=90, n_steps=2), {}, {}, False),
    # int8 rows: the workgroup quantises the row it encodes (several splits; one split with four and eight waves; biases
    # and the Bernoulli map with layers that store nothing); plain-ALU plans keep the two launches
    "int8": (C[2].scaled(n_layers=3, batch=2, n_cached=200, n_steps=2), {"latent_format": "int8"}, {}, True),
    "int8-tile-boundary": (C[2].scaled(n_layers=3, batch=3, n_cached=255, n_steps=3), {"latent_format": "int8"}, {}, True),
    "int8-one-split-w4": (C[4].scaled(n_layers=6, batch=2, n_cached=200, n_steps=2), {"latent_format": "int8", "with_bias": True},
                          {"n_splits": 1, "wg_waves": 4}, True),
    "int8-one-split-w8": (C[4].scaled(n_layers=6, batch=2, n_cached=200, n_steps=2), {"latent_format": "int8"}, {"n_splits": 1, "wg_waves": 8}, True),
    "int8-splits-w8": (C[4].scaled(n_layers=6, batch=2, n_cached=700, n_steps=2), {"latent_format": "int8", "with_bias": True},
                       {"n_splits": 3, "wg_waves": 8}, True),
    "int8-bernoulli-splits": (C[4].scaled(n_layers=8, batch=2, n_cached=333, n_steps=2), {"latent_format": "int8", "with_bias": True}, {}, True),
    "int8-plain-alu": (C[2].scaled(n_layers=3, batch=2, n_cached=100, n_steps=2), {"latent_format": "int8"}, {"force_generic": True}, False),
    "f32": (C[0].scaled(n_layers=2, batch=2, n_cached=60, n_steps=2, reuse="odd:5"), {"with_bias": True}, {}, False),
    "separate-kernels": (C[2].scaled(n_layers=3, batch=2, n_cached=200, n_steps=2), {}, {"no_fuse": True}, False),
    # full-width autoencoders, and a last layer whose key heads are ALL reused: it still stores key rows (nobody reads
    # them), which no workgroup of the attention launch would write: that layer keeps the encoder launch
    "p2-all-key-heads-reused": (C[2].scaled(n_layers=3, batch=2, n_cached=140, n_steps=2, policy="P2"), {"reuse": ALL_K_REUSED}, {}, False),
}


@pytest.mark.parametrize("name", list(CASES))
def test_append_attend_steps(name):
    w, kw, skw, in_kernel = CASES[name]
    print(f"case {name}: {w} {kw} {skw}", flush=True)
    orc, want = run_oracle(w, gain=20.0, **kw)
    ses = Session(w, poison=True, **kw, **skw)
    ses.prefill(0, w.n_cached, chunk=256)
    assert ses.ctx.describe_plan(w.n_layers - 1, w.batch, w.n_cached + 1).append_in_kernel == (1 if in_kernel else 0)
    got = []
    for step in range(w.n_steps):
        pos = w.n_cached + step
        row = {}
        for n in range(w.n_layers):
            k = synth.kv_tokens(w, n, 0, 0, w.batch, pos, pos + 1, device=ses.dev).to(ses.tdt)
            v = synth.kv_tokens(w, n, 1, 0, w.batch, pos, pos + 1, device=ses.dev).to(ses.tdt)
            q = synth.queries(w, n, step, gain=20.0).to(ses.dev, ses.tdt)
            row[n] = ses.append_attend(n, k, v, q, pos).float().cpu().double().numpy()
        got.append(row)
    torch.cuda.synchronize()
    assert_outputs_close(w, got, want, name)
    if kw.get("latent_format") == "int8":
        assert_quantized_cache_close(w, ses, orc, w.n_cached + w.n_steps)
    else:
        assert_cache_close(w, ses, orc, w.n_cached + w.n_steps)


GRAPH_CASES = {
    # the one-kernel step; the step whose encoder shares a launch with the absorbed-query projection (linear, two-layer)
    "one-kernel": (C[4].scaled(n_layers=4, batch=4, n_cached=600, n_steps=2), 1),
    "gpt2-folded": (C[1].scaled(n_layers=3, batch=3, n_cached=300, n_steps=2), 0),
    "two-layer-folded": (C[3].scaled(n_layers=2, batch=3, n_cached=200, n_steps=2), 0),
}


@pytest.mark.parametrize("name", list(GRAPH_CASES))
def test_append_attend_in_a_replayed_graph(name):
    """The step captured as a HIP graph: replays rewrite the same cache row and give the eager result."""
    w, in_kernel = GRAPH_CASES[name]
    ses = Session(w, poison=True)
    ses.prefill(0, w.n_cached, chunk=256)
    dev, tdt, pos = ses.dev, ses.tdt, w.n_cached
    ks = [synth.kv_tokens(w, n, 0, 0, w.batch, pos, pos + 1, device=dev).to(tdt) for n in range(w.n_layers)]
    vs = [synth.kv_tokens(w, n, 1, 0, w.batch, pos, pos + 1, device=dev).to(tdt) for n in range(w.n_layers)]
    qs = [synth.queries(w, n, 0, device=dev, gain=10.0).to(tdt) for n in range(w.n_layers)]
    outs = [torch.empty_like(q) for q in qs]
    ses.ensure_workspace(w.batch, w.max_seq)
    assert ses.ctx.describe_plan(w.n_layers - 1, w.batch, pos + 1).append_in_kernel == in_kernel

    def step():
        for n in range(w.n_layers):
            ses.ctx.append_attend(n, ks[n], vs[n], qs[n], outs[n], w.batch, pos, ses.workspace)

    step()
    torch.cuda.synchronize()
    want = [o.clone() for o in outs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for replay in range(3):
        for o in outs:
            o.fill_(float("nan"))
        scratch = torch.randn(1 << 16, device=dev).sum().item()       # eager work and a host synchronisation between replays
        assert scratch == scratch
        graph.replay()
        torch.cuda.synchronize()
        for n in range(w.n_layers):
            assert torch.equal(outs[n], want[n]), f"replay {replay}, layer {n}"
