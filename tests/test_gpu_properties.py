"""Properties of the attention kernels that hold at any size, checked on caches filled directly
with synthetic latent rows (the cache layout is part of the C ABI)."""
import numpy as np
import pytest
import torch

from oracle import kvcar_oracle as O
from paper_2512_06727_amd import synth
from paper_2512_06727_amd.harness import Session
from tests.helpers import ABS_TOL, REL_TOL, build_oracle

pytestmark = pytest.mark.gpu


def fill(ses, orc, w, n_rows, perm=None):
    """Same synthetic latent rows into the GPU caches and the oracle's (optionally permuted in time)."""
    for n in range(w.n_layers):
        for which in (0, 1):
            view = ses.cache_view(n, which)
            if view is None:
                continue
            r = view.shape[-1]
            z = synth.latent_rows(w, n, which, r, 0, w.batch, 0, n_rows)
            if perm is not None:
                z = z[:, perm]
            view[:, :n_rows] = z.to(ses.dev, ses.tdt)
            if orc is not None:
                orc.Z[(n, which)][:, :n_rows] = z.double().numpy()


def close(w, got, want):
    err = np.abs(got - want).max()
    assert err <= ABS_TOL[w.dtype] and err <= REL_TOL[w.dtype] * np.abs(want).max(), err


@pytest.mark.parametrize("cfg,n_rows", [(2, 1000), (1, 515), (4, 777)])
def test_attention_alone_on_direct_cache_fill(cfg, n_rows):
    w = synth.CONFIGS[cfg].scaled(n_layers=4, batch=3, n_cached=n_rows, n_steps=1)
    ses, orc = Session(w), build_oracle(w)
    fill(ses, orc, w, n_rows)
    for n in range(w.n_layers):
        q = synth.queries(w, n, 0, gain=25.0)
        got = ses.decode_attention(n, q.to(ses.dev, ses.tdt), n_rows).float().cpu().double().numpy()
        close(w, got, orc.decode_attention(n, q.double().numpy(), n_rows))


def test_token_permutation_invariance():
    """Attention does not depend on the order of the cached tokens; a permuted cache sends tokens to
    different tiles, waves and splits, so this exercises the online-softmax merge."""
    w = synth.CONFIGS[2].scaled(n_layers=2, batch=2, n_cached=900, n_steps=1, reuse="none")
    perm = torch.from_numpy(np.random.default_rng(3).permutation(900))
    outs = []
    for p in (None, perm):
        ses = Session(w, n_splits=5)
        fill(ses, None, w, 900, p)
        q = synth.queries(w, 1, 0, gain=25.0).to(ses.dev, ses.tdt)
        outs.append(ses.decode_attention(1, q, 900).float().cpu().double().numpy())
    assert np.abs(outs[0] - outs[1]).max() <= 4 * 2.0 ** -8 * np.abs(outs[0]).max()


def test_zero_query_gives_mean_of_decoded_values():
    w = synth.CONFIGS[2].scaled(n_layers=1, batch=2, n_cached=600, n_steps=1, reuse="none")
    ses, orc = Session(w), build_oracle(w)
    fill(ses, orc, w, 600)
    q = torch.zeros(2, w.n_q_heads, w.d_head)
    got = ses.decode_attention(0, q.to(ses.dev, ses.tdt), 600).float().cpu().double().numpy()
    ae = orc.ae[(0, 1)]
    mean_v = (orc.Z[(0, 1)][:, :600].mean(1) @ ae.dec[0][0]).reshape(2, w.n_kv_heads, 1, w.d_head)
    want = np.broadcast_to(mean_v, (2, w.n_kv_heads, w.n_q_heads // w.n_kv_heads, w.d_head)).reshape(2, w.n_q_heads, w.d_head)
    close(w, got, want)


def test_plain_alu_and_mfma_kernels_agree():
    w = synth.CONFIGS[4].scaled(n_layers=5, batch=2, n_cached=700, n_steps=1)
    outs = []
    for generic in (False, True):
        ses = Session(w, force_generic=generic)
        assert ses.ctx.describe_plan(4, 2, 700).uses_mfma == (0 if generic else 1)
        fill(ses, None, w, 700)
        q = synth.queries(w, 4, 0, gain=25.0).to(ses.dev, ses.tdt)
        outs.append(ses.decode_attention(4, q, 700).float().cpu().double().numpy())
    assert np.abs(outs[0] - outs[1]).max() <= REL_TOL[w.dtype] * np.abs(outs[1]).max()


def test_two_host_threads_with_their_own_contexts_and_streams():
    """Two host threads, each with its own context and stream, run decode steps at the same time (the launchers'
    once-per-process kernel attributes are set from whichever thread comes first): both must match the oracle."""
    import threading
    from paper_2512_06727_amd import synth
    from paper_2512_06727_amd.harness import Session
    from tests.helpers import assert_outputs_close, run_oracle
    ws = [synth.CONFIGS[2].scaled(n_layers=3, batch=2, n_cached=150, n_steps=1, seed=11),
          synth.CONFIGS[1].scaled(n_layers=2, batch=2, n_cached=120, n_steps=1, seed=12)]
    wants = [run_oracle(w, gain=8.0)[1] for w in ws]
    got, errors = [None, None], []

    def work(i):
        try:
            w = ws[i]
            with torch.cuda.stream(torch.cuda.Stream()):
                ses = Session(w)
                ses.prefill(0, w.n_cached + 1, chunk=64)
                row = {}
                for n in range(w.n_layers):
                    q = synth.queries(w, n, 0, gain=8.0).to(ses.dev, ses.tdt)
                    row[n] = ses.decode_attention(n, q, w.n_cached + 1).float().cpu().double().numpy()
                got[i] = [row]
        except Exception as e:          # surfaced below: an exception in a thread would otherwise be lost
            errors.append(e)

    threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for w, g, want in zip(ws, got, wants):
        assert_outputs_close(w, g, want, w.name)


@pytest.mark.parametrize("batch,n_rows,n_splits", [(11, 700, 3), (5, 300, 0), (37, 260, 1), (16, 1000, 0), (3, 2100, 7)])
@pytest.mark.parametrize("fmt", ["dtype", "int8"])
def test_where_a_workgroup_runs_does_not_change_what_it_computes(batch, n_rows, n_splits, fmt):
    """Small launches give every KV head a group and place the groups of a (split, sequence) on one XCD by renumbering the
    workgroups; the renumbering is a permutation of (split, sequence, group), so the outputs must equal, bit for bit,
    those of the same launch in launch order (kvcar_tuning.no_colocate) - for unit counts that are and are not multiples
    of eight - and match the oracle."""
    w = synth.CONFIGS[4].scaled(n_layers=6, batch=batch, n_cached=n_rows - 1, n_steps=1)
    orc = build_oracle(w, latent_format=fmt)
    outs = []
    for no_colocate in (False, True):
        ses = Session(w, poison=True, latent_format=fmt, n_splits=n_splits, no_colocate=no_colocate, group_slots=0)
        ses.prefill(0, n_rows, chunk=256)
        plan = ses.ctx.describe_plan(w.n_layers - 1, batch, n_rows)
        assert plan.n_groups == w.n_kv_heads and plan.n_launches == 1
        outs.append([ses.decode_attention(n, synth.queries(w, n, 0, gain=20.0).to(ses.dev, ses.tdt), n_rows) for n in range(w.n_layers)])
    for n in range(w.n_layers):
        assert torch.equal(outs[0][n], outs[1][n]), n
    for n in range(w.n_layers):
        k = synth.kv_tokens(w, n, 0, 0, batch, 0, n_rows).double().numpy()
        v = synth.kv_tokens(w, n, 1, 0, batch, 0, n_rows).double().numpy()
        orc.encode_append(n, k, v, 0)
    for n in range(w.n_layers):
        want = orc.decode_attention(n, synth.queries(w, n, 0, gain=20.0).double().numpy(), n_rows)
        err = np.abs(outs[0][n].float().cpu().double().numpy() - want).max()
        assert err <= ABS_TOL[w.dtype] and err <= REL_TOL[w.dtype] * np.abs(want).max(), (n, err)
