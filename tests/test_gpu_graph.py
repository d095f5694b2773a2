"""A decode step captured as a HIP graph gives the eager result on every replay, with eager work and
synchronisations of the program's own between the replays (the library records no memset nodes and
allocates nothing, so its calls may be captured)."""
import pytest
import torch

from paper_2512_06727_amd import synth
from paper_2512_06727_amd.harness import Session

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("both_groupings")]


@pytest.mark.parametrize("fmt,splits", [("dtype", 1), ("dtype", 3), ("int8", 1)])
def test_graph_replays_match_eager(fmt, splits):
    w = synth.CONFIGS[4].scaled(n_layers=3, batch=4, n_cached=200, n_steps=4)
    ses = Session(w, latent_format=fmt, n_splits=splits)
    ses.prefill(0, w.n_cached, chunk=128)
    dev, tdt = ses.dev, ses.tdt
    pos = w.n_cached
    ks = [synth.kv_tokens(w, n, 0, 0, w.batch, pos, pos + 1, device=dev).to(tdt) for n in range(w.n_layers)]
    vs = [synth.kv_tokens(w, n, 1, 0, w.batch, pos, pos + 1, device=dev).to(tdt) for n in range(w.n_layers)]
    qs = [synth.queries(w, n, 0, device=dev, gain=10.0).to(tdt) for n in range(w.n_layers)]
    outs = [torch.empty_like(q) for q in qs]
    ses.ensure_workspace(w.batch, w.max_seq)

    def step():
        for n in range(w.n_layers):
            ses.ctx.encode_append(n, ks[n], vs[n], w.batch, pos, 1)
            ses.ctx.decode_attention(n, qs[n], outs[n], w.batch, pos + 1, ses.workspace)

    step()                                        # eager reference (and first-call set-up of every kernel)
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
    for replay in range(4):
        for o in outs:
            o.fill_(float("nan"))                 # eager work between replays: a replay must rewrite every output
        scratch = torch.randn(1 << 16, device=dev).sum().item()      # and a library reduction with a host sync
        assert scratch == scratch
        graph.replay()
        torch.cuda.synchronize()
        for n in range(w.n_layers):
            assert torch.equal(outs[n], want[n]), f"replay {replay}, layer {n}"


@pytest.mark.parametrize("hidden", [0, 256])
def test_prefill_graph_replays_match_eager(hidden):
    """The prompt phase (encode of the chunk + prefill attention, every layer) captured and replayed."""
    base = synth.CONFIGS[3] if hidden else synth.CONFIGS[2]
    w = base.scaled(n_layers=3, batch=2, n_cached=300, n_steps=0)
    ses = Session(w)
    dev, tdt = ses.dev, ses.tdt
    T = w.n_cached
    ks = [synth.kv_tokens(w, n, 0, 0, w.batch, 0, T, device=dev).to(tdt) for n in range(w.n_layers)]
    vs = [synth.kv_tokens(w, n, 1, 0, w.batch, 0, T, device=dev).to(tdt) for n in range(w.n_layers)]
    qs = [synth.prompt_queries(w, n, 0, w.batch, 0, T, device=dev, gain=10.0).to(tdt) for n in range(w.n_layers)]
    outs = [torch.empty_like(q) for q in qs]
    ws = torch.empty(ses.ctx.prefill_workspace_bytes(w.batch, T), dtype=torch.uint8, device=dev)

    def step():
        for n in range(w.n_layers):
            ses.ctx.encode_append(n, ks[n], vs[n], w.batch, 0, T)
            ses.ctx.prefill_attention(n, qs[n], outs[n], w.batch, 0, T, ws)

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
        ws.fill_(0xFF)                            # the decoded rows of the last call are not relied on
        scratch = torch.randn(1 << 16, device=dev).sum().item()      # a library reduction with a host sync between replays
        assert scratch == scratch
        graph.replay()
        torch.cuda.synchronize()
        for n in range(w.n_layers):
            assert torch.equal(outs[n], want[n]), f"replay {replay}, layer {n}"


def test_two_contexts_on_two_streams_at_once():
    """Two library contexts (own caches, own workspaces) driven from two streams of default priority at the same
    time: the library keeps no device state of its own, so each gives the bytes it gives when run alone."""
    wa = synth.CONFIGS[4].scaled(n_layers=3, batch=8, n_cached=3000, n_steps=1)
    wb = synth.CONFIGS[2].scaled(n_layers=3, batch=6, n_cached=2500, n_steps=1, seed=5)
    sessions = [Session(wa), Session(wb, latent_format="int8")]
    work = []
    for ses in sessions:
        w = ses.w
        ses.prefill(0, w.n_cached, chunk=512)
        ses.ensure_workspace(w.batch, w.max_seq)
        qs = [synth.queries(w, n, 0, device=ses.dev, gain=10.0).to(ses.tdt) for n in range(w.n_layers)]
        work.append((qs, [torch.empty_like(q) for q in qs]))

    def run(i):
        ses, (qs, outs) = sessions[i], work[i]
        for rep in range(5):
            for n in range(ses.w.n_layers):
                ses.ctx.decode_attention(n, qs[n], outs[n], ses.w.batch, ses.w.n_cached, ses.workspace)

    want = []
    for i in range(2):                            # each alone, on the current stream
        run(i)
        torch.cuda.synchronize()
        want.append([o.clone() for o in work[i][1]])
        for o in work[i][1]:
            o.zero_()
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(3):                          # interleaved submissions, both streams busy
        for i in range(2):
            with torch.cuda.stream(streams[i]):
                run(i)
    torch.cuda.synchronize()
    for i in range(2):
        for got, ref in zip(work[i][1], want[i]):
            assert torch.equal(got.view(torch.int16), ref.view(torch.int16))
