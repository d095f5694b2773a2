#!/usr/bin/env python3
"""Benchmark of the KV-CAR decode hot path on one MI355X.

A "step" is one decode step of the whole path over one batch: for every layer, the encoder and
append of the new token's K/V followed by decode attention over the latent cache (reuse map
applied) - kvcar_append_attend, which is the two calls kvcar_encode_append + kvcar_decode_attention
in one (and, where the shapes allow, in one kernel); --separate-encode makes the two calls.  The default workload is the TinyLlama-shaped long-context
configuration (batch 256, 8192 cached tokens, 22 layers, bf16, linear autoencoder r=128,
Bernoulli(0.3) head-reuse map).  Inputs are synthetic and resident in HBM before timing starts.

Prints ONE JSON line: tokens/s of the whole job, the HBM roofline of the dominant kernel (the
MFMA attention kernel, timed live with HIP events recorded around it on its stream in a second
pass over the same steps), the CPU oracle timed on a bounded sample of the same workload, and -
in the default run - a `workloads` block with the other four configurations at their full sizes
(ms per step, tokens/s, the attention kernel against the HBM peak; the two-layer configuration
also against the MFMA peak).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E bandwidth
MFMA_PEAK_TFLOPS = 2500.0    # MI355X published dense bf16 / fp16 matrix rate


def sources(reuse, layer, which):
    """Per KV head, the layer whose cache supplies it (nearest earlier layer whose bit is clear)."""
    out = []
    for g in range(reuse.shape[2]):
        m = layer
        while m > 0 and reuse[m, which, g]:
            m -= 1
        out.append(m)
    return out


def algorithmic_latent_bytes(w, reuse, widths, batch, n_ctx, elem, row_meta=0):
    """Bytes of latent rows one decode step must read, per layer: every distinct source
    layer's K rows and V rows once (P * B * n_ctx * sum of source widths; int8 latents: one byte
    per element plus the 8 bytes of scale and zero point per row)."""
    per_layer = []
    for layer in range(w.n_layers):
        tot = 0
        for which in (0, 1):
            tot += sum(widths[m][which] * elem + row_meta for m in set(sources(reuse, layer, which)) if widths[m][which])
        per_layer.append(batch * n_ctx * tot)
    return per_layer


def cpu_baseline(w, reuse, budget_s: float, n_steps: int = 1):
    """The CPU oracle timed on (layer, sequence, step) units of the same workload: full-length context, one
    sequence at a time.  Units are taken in an order that covers, first, the first and the last layer and one
    layer of every reuse-chain depth at the first and at the last decode step, then every layer of further sequences
    (up to 32 sequences, 720 units) until the budget of CPU time is spent - timed steps and the untimed filling of the
    oracle's caches together - but at least 64 units.  Returns tokens/s extrapolated to the whole job."""
    import numpy as np
    import torch
    from threadpoolctl import threadpool_info
    from oracle import kvcar_oracle as O
    from paper_2512_06727_amd import synth

    wo = w.scaled(batch=1)
    cv = lambda pairs: [(a.double().numpy(), None if b is None else b.double().numpy()) for a, b in pairs]
    aes = {(layer, which): synth.autoencoder(w, layer, which, reuse) for layer in range(w.n_layers) for which in (0, 1)}

    def new_oracle():
        orc = O.KVCAROracle(w.n_layers, w.n_q_heads, w.n_kv_heads, w.d_head, 1, w.max_seq, w.dtype)
        for layer in range(w.n_layers):
            orc.set_reuse_map(layer, reuse[layer, 0], reuse[layer, 1])
        for (layer, which), ae in aes.items():
            orc.set_autoencoder(layer, which, O.Autoencoder(ae.heads, cv(ae.enc), cv(ae.dec), act=ae.act, slope=ae.slope))
        return orc

    # chain depth of a layer: how far back its farthest source lies
    depth = [max(layer - m for which in (0, 1) for m in sources(reuse, layer, which)) for layer in range(w.n_layers)]
    by_depth = {}
    for layer, d in enumerate(depth):
        by_depth.setdefault(d, layer)
    first_layers = list(dict.fromkeys([0, w.n_layers - 1] + list(by_depth.values())))
    last_step = max(0, n_steps - 1)
    seqs = list(dict.fromkeys([0, w.batch - 1, w.batch // 2, w.batch // 3] + [(7 * i + 3) % w.batch for i in range(w.batch)]))[:32]
    units = [(layer, seqs[0], st) for layer in first_layers for st in dict.fromkeys([0, last_step])]
    for b in seqs:
        units += [(layer, b, 0 if (layer + b) % 2 == 0 else last_step) for layer in range(w.n_layers)]
    units = list(dict.fromkeys(units))[:720]

    t_begin = time.perf_counter()
    t_used, done, covered = 0.0, 0, set()
    orc, orc_b, filled = None, None, {}
    for layer, b, st in units:
        if orc_b != b:
            orc, orc_b, filled = new_oracle(), b, {}
        n_ctx = w.n_cached + st + 1
        need = {layer} | set(sources(reuse, layer, 0)) | set(sources(reuse, layer, 1))
        for m in sorted(need):                       # untimed: the sequence's cached rows up to this step (prefill is not part of the step)
            have = filled.get(m, 0)
            upto = n_ctx if m != layer else n_ctx - 1
            if have < upto:
                orc.encode_append(m, synth.kv_tokens(wo, m, 0, b, b + 1, have, upto).double().numpy(),
                                  synth.kv_tokens(wo, m, 1, b, b + 1, have, upto).double().numpy(), have)
                filled[m] = upto
        k1 = synth.kv_tokens(wo, layer, 0, b, b + 1, n_ctx - 1, n_ctx).double().numpy()
        v1 = synth.kv_tokens(wo, layer, 1, b, b + 1, n_ctx - 1, n_ctx).double().numpy()
        q = synth.queries(w, layer, st)[b:b + 1].double().numpy()
        t0 = time.perf_counter()
        orc.encode_append(layer, k1, v1, n_ctx - 1)           # timed: one decode step of one (layer, sequence)
        orc.decode_attention(layer, q, n_ctx)
        t_used += time.perf_counter() - t0
        filled[layer] = max(filled.get(layer, 0), n_ctx)
        done += 1
        covered.add((depth[layer], st))
        if time.perf_counter() - t_begin > budget_s and done >= 64:      # the budget covers the untimed filling of the oracle's caches too
            break
    per_unit = t_used / done
    step_s = per_unit * w.n_layers * w.batch                  # extrapolated to all layers and sequences
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [torch.get_num_threads(), 1])
    return {"value": w.batch / step_s, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{done} (layer, sequence, step) units of one decode step at n_ctx={w.n_cached + 1}..{w.n_cached + last_step + 1} "
                      f"(first and last layer, reuse-chain depths {sorted({d for d, _ in covered})}, decode steps {sorted({t for _, t in covered})}), "
                      f"{per_unit * 1e3:.1f} ms each, extrapolated to {w.n_layers} layers x {w.batch} sequences"}


def bench_l1_distance(args):
    """Secondary measurement: the reuse-map selection statistic (per-head mean L1 distance between the keys
    of two adjacent layers) over the tokens of the chosen workload; HBM-bound, both tensors read once."""
    import numpy as np
    import torch
    from oracle import kvcar_oracle as O
    from paper_2512_06727_amd import binding, synth

    w = synth.CONFIGS[args.workload]
    if args.batch:
        w = w.scaled(batch=args.batch)
    if args.cached:
        w = w.scaled(n_cached=args.cached)
    dev, tdt = torch.device("cuda:0"), synth.TORCH_DTYPE[w.dtype]
    n_tokens = w.batch * w.n_cached
    chunk = max(1, (1 << 25) // (w.batch * w.d_kv))
    xs = []
    for layer in (0, 1):
        parts = [synth.kv_tokens(w, layer, 0, 0, w.batch, c0, min(w.n_cached, c0 + chunk), device=dev).to(tdt) for c0 in range(0, w.n_cached, chunk)]
        xs.append(torch.cat(parts, dim=1).reshape(n_tokens, w.d_kv).contiguous())
    dist = torch.zeros(w.n_kv_heads, dtype=torch.float32, device=dev)
    need = binding.C.c_size_t(0)
    binding.lib().kvcar_head_l1_workspace_bytes(n_tokens, w.n_kv_heads, binding.C.byref(need))
    ws = torch.empty(max(16, need.value), dtype=torch.uint8, device=dev)
    run = lambda: binding.head_l1_distance(xs[0], xs[1], w.n_kv_heads, w.d_head, dist=dist, workspace=ws)
    for _ in range(args.warmup):
        run()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    nbytes = 2 * xs[0].numel() * xs[0].element_size()
    gbs = nbytes / (ms * 1e-3) / 1e9
    probe = torch.zeros(1 << 32, dtype=torch.uint8, device=dev)
    ceiling = binding.probe_read_bandwidth(probe, repeats=4)
    del probe
    # oracle on a bounded sample, and parity of the sample
    n_s = min(n_tokens, 1 << 18)
    a, b = xs[0][:n_s].float().cpu().double().numpy(), xs[1][:n_s].float().cpu().double().numpy()
    t0 = time.perf_counter()
    want = O.head_l1_distance(a, b, w.n_kv_heads, w.d_head)
    t_cpu = time.perf_counter() - t0
    got = binding.head_l1_distance(xs[0][:n_s], xs[1][:n_s], w.n_kv_heads, w.d_head).cpu().double().numpy()
    print(json.dumps({
        "metric": "reuse-selection L1 distance, tokens/s", "value": n_tokens / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "op": "head_l1_distance", "tokens": n_tokens, "kv_heads": w.n_kv_heads, "d_head": w.d_head},
        "roofline": {"bound": "hbm", "kernel": "head_l1_partial_kernel", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": gbs / HBM_PEAK_GBS, "traffic": None, "algorithmic_bytes_per_launch": nbytes, "avg_launch_ms": ms,
                     "read_ceiling_GBs": ceiling, "frac_of_read_ceiling": gbs / ceiling},
        "cpu_baseline": {"value": n_s / t_cpu, "unit": "tokens/s", "cores": 1, "kind": "oracle",
                         "sample": f"first {n_s} tokens, {t_cpu:.2f} s; max relative difference GPU vs oracle on the sample {np.abs(got / want - 1).max():.2e}"},
    }))




def bench_prefill(args):
    """Secondary measurement: the prompt phase.  A step = for every layer, kvcar_encode_append of the whole
    prompt chunk (T tokens per sequence) followed by kvcar_prefill_attention of the chunk over the latent
    caches.  Bound by the matrix units: the roofline object is the causal attention kernel against the dense
    16-bit MFMA peak, with 4 * H_q * d_head flops per (query, visible row) pair."""
    import numpy as np
    import torch
    from oracle import kvcar_oracle as O
    from paper_2512_06727_amd import synth
    from paper_2512_06727_amd.harness import Session

    base = synth.CONFIGS[args.workload]
    w = base.scaled(batch=args.batch or 16, n_cached=args.cached or 4096, n_steps=0)
    if args.policy:
        w = w.scaled(policy=args.policy)
    if args.no_reuse:
        w = w.scaled(reuse="none")
    reuse = synth.reuse_map(w)
    T = w.n_cached
    ses = Session(w, reuse=reuse, latent_format=args.latent)
    dev, tdt = ses.dev, ses.tdt
    chunk = max(1, (1 << 25) // (w.batch * w.d_kv))
    gen = lambda f: torch.cat([f(c0, min(T, c0 + chunk)) for c0 in range(0, T, chunk)], dim=1).contiguous()
    ks = [gen(lambda a, b: synth.kv_tokens(w, n, 0, 0, w.batch, a, b, device=dev).to(tdt)) for n in range(w.n_layers)]
    vs = [gen(lambda a, b: synth.kv_tokens(w, n, 1, 0, w.batch, a, b, device=dev).to(tdt)) for n in range(w.n_layers)]
    qs = [gen(lambda a, b: synth.prompt_queries(w, n, 0, w.batch, a, b, device=dev).to(tdt)) for n in range(w.n_layers)]
    out = torch.empty_like(qs[0])
    ws = torch.empty(ses.ctx.prefill_workspace_bytes(w.batch, T), dtype=torch.uint8, device=dev)
    ctx = ses.ctx

    def step_fn():
        for n in range(w.n_layers):
            ctx.encode_append(n, ks[n], vs[n], w.batch, 0, T)
            ctx.prefill_attention(n, qs[n], out, w.batch, 0, T, ws)

    for _ in range(args.warmup):
        step_fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step_fn()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    ctx.profile_enable(True)
    for _ in range(args.steps):
        step_fn()
    attend_ms, n_launch = ctx.profile_read()
    ctx.profile_enable(False)
    pairs = w.batch * T * (T + 1) // 2                                  # (query, visible row) pairs per layer
    flops = 4 * w.n_q_heads * w.d_head * pairs                          # per attention launch
    achieved = flops / (attend_ms / n_launch * 1e-3) / 1e12

    result = {
        "metric": "prefill tokens/s over latent KV cache (encode + causal attention, all layers)", "value": w.batch * T * args.steps / elapsed,
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "op": "prefill", "batch": w.batch, "prompt_tokens": T, "layers": w.n_layers, "q_heads": w.n_q_heads,
                   "kv_heads": w.n_kv_heads, "d_head": w.d_head, "latent": w.latent, "hidden": w.hidden, "latent_format": args.latent,
                   "reuse": w.reuse, "policy": w.policy},
        "roofline": {"bound": "mfma", "kernel": "prefill_mfma_kernel", "achieved": achieved, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_PEAK_TFLOPS, "traffic": None, "algorithmic_flops_per_launch": flops,
                     "avg_launch_ms": attend_ms / n_launch, "launches": n_launch,
                     "attention_share_of_step": attend_ms / args.steps / ms_per_step},
    }
    if args.cpu_seconds > 0:
        # the oracle on one (layer, sequence) unit of the same prompt (shortened if the budget asks for it)
        t_s = T if args.cpu_seconds >= 10 else min(T, 1024)
        wo = w.scaled(batch=1)
        orc = O.KVCAROracle(w.n_layers, w.n_q_heads, w.n_kv_heads, w.d_head, 1, T, w.dtype, latent_format=args.latent)
        cv = lambda pairs_: [(a.double().numpy(), None if b is None else b.double().numpy()) for a, b in pairs_]
        for which in (0, 1):
            ae = synth.autoencoder(w, 0, which, reuse)
            orc.set_autoencoder(0, which, O.Autoencoder(ae.heads, cv(ae.enc), cv(ae.dec), act=ae.act, slope=ae.slope))
        k = synth.kv_tokens(wo, 0, 0, 0, 1, 0, t_s).double().numpy()
        v = synth.kv_tokens(wo, 0, 1, 0, 1, 0, t_s).double().numpy()
        q = synth.prompt_queries(wo, 0, 0, 1, 0, t_s).double().numpy()
        from threadpoolctl import threadpool_info
        t0 = time.perf_counter()
        orc.encode_append(0, k, v, 0)
        want = orc.prefill_attention(0, q, 0)
        t_cpu = time.perf_counter() - t0
        got = ses.prefill_attention(0, qs[0][:1, :t_s].contiguous(), 0).float().cpu().double().numpy()
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [torch.get_num_threads(), 1])
        # cost grows with the square of the prompt: scale the unit to the full prompt before extrapolating
        unit_s = t_cpu * (T * (T + 1)) / (t_s * (t_s + 1))
        result["cpu_baseline"] = {"value": w.batch * T / (unit_s * w.n_layers * w.batch), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
                                  "sample": f"layer 0, sequence 0, first {t_s} prompt tokens: {t_cpu:.1f} s, scaled by visible pairs to {T} tokens "
                                            f"and to {w.n_layers} layers x {w.batch} sequences; max |GPU - oracle| on the sample {np.abs(got - want).max():.2e}"}
    print(json.dumps(result))


def bench_per_head(args):
    """Secondary measurement: the per-head (block-diagonal) autoencoder variant of the workload - the autoencoder
    descriptor's per_head flag: every KV head has a d_head -> latent / H_kv -> d_head autoencoder and a block of the
    cache of its own, a layer's attention is one launch with a group per KV head.  A reused head then reads only its
    own rows of the source layer, so the step moves the bytes of the map-free workload while storing what the map
    leaves.  A step = kvcar_append_attend for every layer (--separate-encode: kvcar_encode_append +
    kvcar_decode_attention)."""
    import torch
    from paper_2512_06727_amd import synth
    from paper_2512_06727_amd.harness import Session

    total_steps = args.steps + args.warmup
    w = synth.CONFIGS[args.workload].scaled(n_steps=total_steps)
    if args.batch:
        w = w.scaled(batch=args.batch)
    if args.cached:
        w = w.scaled(n_cached=args.cached)
    if args.reuse:
        w = w.scaled(reuse=args.reuse)
    reuse = synth.reuse_map(w)
    elem = synth.DTYPE_BYTES[w.dtype]
    ses = Session(w, reuse, per_head=True, n_splits=args.splits, wg_waves=args.wg_waves, no_arrive=args.no_arrive)
    t0 = time.perf_counter()
    ses.prefill(0, w.n_cached, chunk=max(1, (1 << 25) // (w.batch * w.d_kv)))
    torch.cuda.synchronize()
    t_fill = time.perf_counter() - t0
    H = w.n_kv_heads
    qs = [[ses.queries(n, step) for n in range(w.n_layers)] for step in range(total_steps)]
    ks = [[ses.kv(n, 0, w.n_cached + step, w.n_cached + step + 1) for n in range(w.n_layers)] for step in range(total_steps)]
    vs = [[ses.kv(n, 1, w.n_cached + step, w.n_cached + step + 1) for n in range(w.n_layers)] for step in range(total_steps)]
    outs = [torch.empty_like(qs[0][n]) for n in range(w.n_layers)]
    ses.ensure_workspace(w.batch, w.max_seq)
    ctx, ws = ses.ctx, ses.workspace

    def step_fn(step):
        pos = w.n_cached + step
        for n in range(w.n_layers):
            if args.separate_encode:
                ctx.encode_append(n, ks[step][n], vs[step][n], w.batch, pos, 1)
                ctx.decode_attention(n, qs[step][n], outs[n], w.batch, pos + 1, ws)
            else:
                ctx.append_attend(n, ks[step][n], vs[step][n], qs[step][n], outs[n], w.batch, pos, ws)

    for step in range(args.warmup):
        step_fn(step)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for step in range(args.warmup, total_steps):
        step_fn(step)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ctx.profile_enable(True)
    for step in range(args.warmup, total_steps):
        step_fn(step)
    attend_ms, n_launch = ctx.profile_read()
    ctx.profile_enable(False)
    plan = ctx.describe_plan(w.n_layers - 1, w.batch, w.n_cached + 1)
    r_h = w.latent // H
    alg = sum(2 * r_h * elem * H * w.batch * (w.n_cached + step + 1) * w.n_layers for step in range(args.warmup, total_steps))
    achieved = alg / (attend_ms * 1e-3) / 1e9
    stored = sum(int((~reuse[n, k]).sum()) * r_h * elem for n in range(w.n_layers) for k in (0, 1))
    print(json.dumps({
        "metric": "decode-attn tokens/s over latent KV cache, per-head autoencoders", "value": w.batch * args.steps / elapsed, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "variant": "per-head autoencoders (descriptor flag, one context)", "batch": w.batch, "cached_tokens": w.n_cached,
                   "layers": w.n_layers, "kv_heads": H, "latent_per_head": r_h, "reuse": w.reuse, "reused_head_fraction": float(reuse[1:].mean()),
                   "groups": plan.n_groups, "splits": plan.n_splits, "fused": plan.fused, "append_in_kernel": plan.append_in_kernel and not args.separate_encode,
                   "prefill_s": t_fill},
        "roofline": {"bound": "hbm", "kernel": "attend_mfma_r128_kernel (latent width 32 per head" + (", new token encoded inside)" if plan.append_in_kernel and not args.separate_encode else ")"),
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None, "algorithmic_bytes_per_launch": alg / max(1, n_launch),
                     "avg_launch_ms": attend_ms / max(1, n_launch), "launches": n_launch},
        "bytes_per_token_stored": stored, "bytes_per_token_read_per_step": 2 * r_h * elem * H * w.n_layers,
    }))


def capacity_check(args):
    """Capacity leg (the analogue of the paper's maximum-sequence-length-before-OOM measurement, Results,
    "System Evaluation"): allocate latent caches for as many cached tokens as fit in this GPU's free memory
    (batch of the workload, context grown), fill them, run one decode step over the full context and
    report what was allocated against what the uncompressed cache would need."""
    import torch
    from paper_2512_06727_amd import synth
    from paper_2512_06727_amd.harness import Session

    base = synth.CONFIGS[args.workload]
    if args.policy:
        base = base.scaled(policy=args.policy)
    if args.no_reuse:
        base = base.scaled(reuse="none")
    reuse = synth.reuse_map(base)
    elem = synth.DTYPE_BYTES[base.dtype]
    lat_elem, row_meta = (1, 8) if args.latent == "int8" else (elem, 0)
    probe = Session(base.scaled(batch=1, n_cached=1, n_steps=1), reuse=reuse, latent_format=args.latent)
    widths = [[probe.ae[n][k].latent for k in (0, 1)] for n in range(base.n_layers)]
    del probe
    lat_tok = sum(r * lat_elem + (row_meta if r else 0) for pair in widths for r in pair)
    full_tok = 2 * elem * base.n_layers * base.d_kv
    free, total = torch.cuda.mem_get_info()
    budget = int(free * args.capacity_fraction)
    max_seq = budget // (lat_tok * base.batch) // 128 * 128
    w = base.scaled(n_cached=max_seq - 1, n_steps=1)
    t0 = time.perf_counter()
    ses = Session(w, reuse=reuse, latent_format=args.latent)
    for n, row in enumerate(ses.caches):                    # every row holds valid data
        for which, c in enumerate(row):
            if c is None:
                continue
            if args.latent == "int8":
                codes, scale, zp = ses.quantized_view(n, which)
                flat = codes.view(-1).view(torch.uint8)
                for i in range(0, flat.numel(), 1 << 30):
                    flat[i:i + (1 << 30)].random_(0, 256)
                scale.fill_(127.5)
                zp.zero_()
            else:
                for i in range(0, c.numel(), 1 << 29):
                    c[i:i + (1 << 29)].normal_(0.0, 0.32)
    torch.cuda.synchronize()
    t_alloc = time.perf_counter() - t0
    dev, tdt = ses.dev, ses.tdt
    pos = w.n_cached
    q = [torch.randn(w.batch, w.n_q_heads, w.d_head, device=dev).to(tdt) for _ in range(w.n_layers)]
    k = [torch.randn(w.batch, 1, w.d_kv, device=dev).to(tdt) for _ in range(w.n_layers)]
    v = [torch.randn(w.batch, 1, w.d_kv, device=dev).to(tdt) for _ in range(w.n_layers)]
    outs = [torch.empty_like(x) for x in q]
    ses.ensure_workspace(w.batch, w.max_seq)

    def step():
        for n in range(w.n_layers):
            ses.ctx.encode_append(n, k[n], v[n], w.batch, pos, 1)
            ses.ctx.decode_attention(n, q[n], outs[n], w.batch, pos + 1, ses.workspace)

    step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3
    finite = all(bool(torch.isfinite(o.float()).all()) for o in outs)
    cache_bytes = sum(c.numel() * c.element_size() for row in ses.caches for c in row if c is not None)
    tokens = w.batch * w.max_seq
    print(json.dumps({
        "metric": "cached tokens resident in HBM (capacity check)", "value": tokens, "unit": "tokens", "n_gpus": 1,
        "higher_is_better": True, "dtype": w.dtype, "data": "synthetic (random latents)",
        "config": {"workload": w.name, "batch": w.batch, "context": w.max_seq, "latent_format": args.latent, "policy": w.policy, "reuse": w.reuse},
        "device_memory_bytes": total, "free_before_bytes": free, "latent_cache_bytes": cache_bytes,
        "bytes_per_token_latent": lat_tok, "bytes_per_token_uncompressed": full_tok,
        "uncompressed_cache_would_need_bytes": tokens * full_tok, "uncompressed_tokens_in_same_bytes": cache_bytes // full_tok,
        "decode_step_ms_at_full_context": ms, "outputs_finite": finite, "alloc_and_fill_s": t_alloc,
    }))


def kernel_source_hash() -> str:
    """sha256 over the library's sources (csrc/ and the public header): what a committed profile was taken with."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2512_06727_amd", "csrc")
    for name in sorted(os.listdir(csrc)) + ["../../include/kvcar.h"]:
        if name.endswith((".hip", ".hpp", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def attention_flops_per_token(w) -> int:
    """Algorithmic flops of the attention kernel per cached token and layer: scores and weighted sums over the
    contraction width (the latent, or the hidden width of a two-layer decoder), plus, for a two-layer decoder, the
    rebuild of the K and V hidden rows."""
    c = w.hidden if w.hidden else w.latent
    return 2 * 2 * w.n_q_heads * c + (2 * 2 * w.latent * w.hidden if w.hidden else 0)


def roofline_entry(w, m, latent_format):
    """Roofline object of the attention kernel of one measured workload: achieved = algorithmic latent bytes per
    launch / average launch time (HIP events around the kernel on its stream) against the HBM peak; two-layer
    decoders (matrix work per byte near the ridge) also against the dense 16-bit MFMA peak."""
    plan = m["plan"]
    achieved = m["alg_bytes"] / (m["attend_ms"] * 1e-3) / 1e9
    kernel = "attend_generic_kernel"
    if plan.uses_mfma:
        # the attention kernel's forms by row width and waves per workgroup: all launches of a step are averaged
        kernel = ("attend_mlp_mfma_kernel" if w.hidden else "attend_i8_mfma_r128_kernel / attend_i8_mfma_r128_w8_kernel" if latent_format == "int8"
                  else "attend_mfma_r384_kernel" if w.latent > 128 else "attend_mfma_r128_kernel / attend_mfma_r128_w8_kernel")
    r = {"bound": "hbm", "kernel": kernel, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
         "traffic": None, "algorithmic_bytes_per_launch": m["alg_bytes"] / max(1, m["n_launch"]),
         "avg_launch_ms": m["attend_ms"] / max(1, m["n_launch"]), "launches": m["n_launch"],
         "whole_step_GBs": m["alg_bytes"] / m["steps"] / (m["ms_per_step"] * 1e-3) / 1e9}
    if m.get("sep_attend_ms"):
        a2 = m["alg_bytes"] / (m["sep_attend_ms"] * 1e-3) / 1e9
        r["attention_launch_without_encoder"] = {"avg_launch_ms": m["sep_attend_ms"] / max(1, m["n_launch"]), "achieved": a2, "frac": a2 / HBM_PEAK_GBS,
                                                 "note": "same steps as kvcar_encode_append + kvcar_decode_attention: the attention kernel alone; the figures above "
                                                         "are for the one kernel per layer that also encodes and appends the new token"}
    if w.hidden and plan.uses_mfma:
        tf = m["alg_flops"] / (m["attend_ms"] * 1e-3) / 1e12
        r["mfma"] = {"achieved": tf, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tf / MFMA_PEAK_TFLOPS,
                     "algorithmic_flops_per_launch": m["alg_flops"] / max(1, m["n_launch"])}
    return r


def measure_decode(w, args, steps, warmup, graph=True, plain=False):
    """Times `steps` decode steps of workload `w` (after `warmup`), then the same steps again with HIP events around
    the attention kernel.  `plain`: library defaults, model-dtype latents and the cache-only variant whatever the
    command line says (the extra workloads of the default run)."""
    import torch
    from paper_2512_06727_amd import synth
    from paper_2512_06727_amd.harness import Session

    total_steps = steps + warmup
    latent = "dtype" if plain else args.latent
    variant = "cache" if plain else args.variant
    fill = "encode" if plain else args.fill
    reuse = synth.reuse_map(w)
    elem = synth.DTYPE_BYTES[w.dtype]
    separate = False if plain else args.separate_encode
    kw = {} if plain else dict(n_splits=args.splits, tile_order=args.tile_order, wg_waves=args.wg_waves, no_fuse=args.no_fuse, no_arrive=args.no_arrive, group_slots=args.group_slots, no_colocate=args.no_colocate)
    ses = Session(w, reuse=reuse, latent_format=latent, **kw)
    lat_elem, row_meta = (1, 8) if latent == "int8" else (elem, 0)
    dev, tdt = ses.dev, ses.tdt
    widths = [[ses.ae[n][which].latent for which in (0, 1)] for n in range(w.n_layers)]
    t_fill = time.perf_counter()
    if fill == "encode":
        ses.prefill(0, w.n_cached, chunk=max(1, (1 << 25) // (w.batch * w.d_kv)))
    else:
        torch.manual_seed(w.seed)
        for n, row in enumerate(ses.caches):
            for which, c in enumerate(row):
                if c is None:
                    continue
                if latent == "int8":
                    codes, scale, zp = ses.quantized_view(n, which)
                    codes.view(torch.uint8).random_(0, 256)
                    scale.fill_(127.5)
                    zp.random_(-8, 9)
                else:
                    c.normal_(0.0, 0.32)
    torch.cuda.synchronize()
    t_fill = time.perf_counter() - t_fill

    # inputs of every step, resident in HBM before timing
    qs, ks, vs = [], [], []
    for step in range(total_steps):
        pos = w.n_cached + step
        if fill == "encode":
            qs.append([synth.queries(w, n, step, device=dev).to(tdt) for n in range(w.n_layers)])
            ks.append([synth.kv_tokens(w, n, 0, 0, w.batch, pos, pos + 1, device=dev).to(tdt) for n in range(w.n_layers)])
            vs.append([synth.kv_tokens(w, n, 1, 0, w.batch, pos, pos + 1, device=dev).to(tdt) for n in range(w.n_layers)])
        else:
            qs.append([torch.randn(w.batch, w.n_q_heads, w.d_head, device=dev).to(tdt) for n in range(w.n_layers)])
            ks.append([torch.randn(w.batch, 1, w.d_kv, device=dev).to(tdt) for n in range(w.n_layers)])
            vs.append([torch.randn(w.batch, 1, w.d_kv, device=dev).to(tdt) for n in range(w.n_layers)])
    outs = [torch.empty_like(qs[0][n]) for n in range(w.n_layers)]
    ses.ensure_workspace(w.batch, w.max_seq)
    ctx, ws = ses.ctx, ses.workspace

    seq_lens = None
    if variant == "ragged":
        gen = torch.Generator(device="cpu").manual_seed(w.seed)
        seq_lens = torch.randint(w.n_cached // 2, w.n_cached + 1, (w.batch,), generator=gen, dtype=torch.int32).to(dev)

    def step_fn(step):
        pos = w.n_cached + step
        for n in range(w.n_layers):
            if variant == "exact":
                kc, vc = ks[step][n].view(w.batch, w.d_kv), vs[step][n].view(w.batch, w.d_kv)
                ctx.decode_attention_ex(n, qs[step][n], outs[n], w.batch, pos, ws, k_cur=kc, v_cur=vc)
                ctx.encode_append(n, ks[step][n], vs[step][n], w.batch, pos, 1)
            elif variant == "ragged":
                ctx.encode_append(n, ks[step][n], vs[step][n], w.batch, pos, 1)
                ctx.decode_attention_ex(n, qs[step][n], outs[n], w.batch, pos + 1, ws, seq_lens=seq_lens)
            elif separate:
                ctx.encode_append(n, ks[step][n], vs[step][n], w.batch, pos, 1)
                ctx.decode_attention(n, qs[step][n], outs[n], w.batch, pos + 1, ws)
            else:
                ctx.append_attend(n, ks[step][n], vs[step][n], qs[step][n], outs[n], w.batch, pos, ws)

    for step in range(warmup):
        step_fn(step)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for step in range(warmup, total_steps):
        step_fn(step)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / steps * 1e3
    tokens_per_s = w.batch * steps / elapsed

    # the same step as a HIP graph: captured once at the last step's positions, replayed `steps` times
    graph_ms = None
    if graph:
        last = total_steps - 1
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step_fn(last)                                  # every kernel has run once on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            step_fn(last)
        g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) / steps * 1e3
        del g

    # second pass over the same steps with HIP events around the attention kernel
    ctx.profile_enable(True)
    for step in range(warmup, total_steps):
        step_fn(step)
    attend_ms, n_launch = ctx.profile_read()
    ctx.profile_enable(False)
    # the same steps once more as two calls per layer (encoder launch + attention launch), for the attention kernel alone
    sep_ms = None
    if not separate and variant == "cache" and not plain and ctx.describe_plan(w.n_layers - 1, w.batch, w.max_seq).append_in_kernel:
        separate = True
        ctx.profile_enable(True)
        for step in range(warmup, total_steps):
            step_fn(step)
        sep_ms, _ = ctx.profile_read()
        ctx.profile_enable(False)
        separate = False
    alg, flops = 0, 0
    for step in range(warmup, total_steps):
        n_rows = w.n_cached + step + (0 if variant == "exact" else 1)
        if seq_lens is not None:                      # ragged: bytes of the rows each sequence really reads
            alg += sum(algorithmic_latent_bytes(w, reuse, widths, 1, int(seq_lens.sum().item()), lat_elem, row_meta))
        else:
            alg += sum(algorithmic_latent_bytes(w, reuse, widths, w.batch, n_rows, lat_elem, row_meta))
        flops += attention_flops_per_token(w) * w.batch * n_rows * w.n_layers
    return {"reuse": reuse, "widths": widths, "ms_per_step": ms_per_step, "tokens_per_s": tokens_per_s, "graph_ms": graph_ms,
            "attend_ms": attend_ms, "sep_attend_ms": sep_ms, "n_launch": n_launch, "alg_bytes": alg, "alg_flops": flops, "steps": steps, "prefill_s": t_fill,
            "plan": ctx.describe_plan(w.n_layers - 1, w.batch, w.max_seq), "one_call": not separate and variant == "cache"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=16)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", type=int, default=4, help="index into the configuration list (default: long-context TinyLlama)")
    ap.add_argument("--batch", type=int, default=0, help="override the batch (for quick runs)")
    ap.add_argument("--cached", type=int, default=0, help="override the cached tokens (for quick runs)")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--tile-order", type=int, default=0, help="0 library default, 1 contiguous token range per split, 2 tiles dealt round-robin")
    ap.add_argument("--policy", default="", help="P1 (latent shrinks with stored heads) or P2 (full width)")
    ap.add_argument("--no-reuse", action="store_true")
    ap.add_argument("--reuse", default="", help="override the reuse map, e.g. kvbernoulli:0.3 (keys and values drawn independently)")
    ap.add_argument("--act", default="", help="override the activation of a two-layer autoencoder (gelu | leaky_relu)")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="seconds of CPU work for the CPU-oracle leg (timed steps plus the untimed filling of its caches; at least 64 units, up to 720); 0 skips it")
    ap.add_argument("--no-workloads", action="store_true", help="default run only: skip the block with the other four configurations")
    ap.add_argument("--fill", default="encode", choices=["encode", "random"],
                    help="encode: caches filled by kvcar_encode_append of seeded K/V (default); random: torch.randn latents and "
                         "inputs (profiling runs only: same traffic, far fewer helper kernels)")
    ap.add_argument("--latent", default="dtype", choices=["dtype", "int8"],
                    help="latent rows in the model dtype (default, the headline) or as int8 codes with a scale and zero point per row")
    ap.add_argument("--variant", default="cache", choices=["cache", "exact", "ragged"],
                    help="cache: append the new token, attend over the cache (default, the headline); exact: attend over the cached "
                         "rows plus the current token's exact K/V row (kvcar_decode_attention_ex), then append; ragged: per-sequence "
                         "context lengths drawn uniformly from [n_cached/2, n_cached]")
    ap.add_argument("--op", default="decode", choices=["decode", "l1dist", "prefill"],
                    help="decode: the decode step (default, the headline); l1dist: the reuse-map selection statistic over the workload's tokens; "
                         "prefill: encode + causal attention of a whole prompt (default batch 16 x 4096 tokens of the chosen workload's shape)")
    ap.add_argument("--per-head", action="store_true",
                    help="the per-head (block-diagonal) autoencoder variant (the descriptor's per_head flag): reuse adds no cache traffic")
    ap.add_argument("--no-fuse", action="store_true", help="run prologue / attention / merge as separate kernels")
    ap.add_argument("--separate-encode", action="store_true",
                    help="a layer's step as kvcar_encode_append + kvcar_decode_attention (two calls) instead of kvcar_append_attend")
    ap.add_argument("--no-colocate", action="store_true", help="workgroups in launch order even where groups read the same rows")
    ap.add_argument("--group-slots", type=int, default=0, help="most query heads per attention workgroup: 0 automatic, 16 or 32")
    ap.add_argument("--no-arrive", action="store_true", help="several splits: partials to the separate merge kernel instead of the one-launch form")
    ap.add_argument("--capacity-check", action="store_true",
                    help="allocate latent caches for as many tokens as fit in free HBM, run one decode step over them, report")
    ap.add_argument("--capacity-fraction", type=float, default=0.92, help="share of the free device memory the capacity check may take")
    ap.add_argument("--wg-waves", type=int, default=0, help="one-launch attention kernels: 0 automatic, 4 or 8 waves per workgroup")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay leg")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB read + 1 GiB write elementwise kernel (counter calibration under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (one process, one MI355X, no collectives); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2512_06727_amd import binding, synth
    from paper_2512_06727_amd.harness import Session

    binding.lib()
    if args.op == "l1dist":
        return bench_l1_distance(args)
    if args.op == "prefill":
        return bench_prefill(args)
    if args.capacity_check:
        return capacity_check(args)
    if args.per_head:
        return bench_per_head(args)
    base = synth.CONFIGS[args.workload]
    w = base.scaled(n_steps=args.steps + args.warmup)
    if args.batch:
        w = w.scaled(batch=args.batch)
    if args.cached:
        w = w.scaled(n_cached=args.cached)
    if args.policy:
        w = w.scaled(policy=args.policy)
    if args.no_reuse:
        w = w.scaled(reuse="none")
    if args.reuse:
        w = w.scaled(reuse=args.reuse)
    if args.act:
        w = w.scaled(act=args.act)
    m = measure_decode(w, args, args.steps, args.warmup, graph=not args.no_graph)
    reuse, elem = m["reuse"], synth.DTYPE_BYTES[w.dtype]
    lat_elem, row_meta = (1, 8) if args.latent == "int8" else (elem, 0)
    dev = torch.device("cuda:0")

    # HBM bytes per launch from the committed rocprofv3 counter summary of this same workload - only if that summary was
    # taken with the kernels that are running now (it records a hash of the kernel sources)
    traffic, traffic_note = None, "no counter summary for this workload"
    tpath = os.path.join(ROOT, "profiles", "attend_i8_mfma_long_context_pmc.md" if args.latent == "int8" else "attend_mfma_long_context_pmc.md")
    if os.path.exists(tpath) and args.workload == 4 and args.variant == "cache" and not (args.batch or args.cached or args.no_reuse or args.policy or args.reuse):
        import re
        text = open(tpath).read()
        mt = re.search(r"traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)", text)
        mh = re.search(r"kernel_source_sha256\s*=\s*([0-9a-f]+)", text)
        if mt and mh and mh.group(1) == kernel_source_hash():
            traffic, traffic_note = float(mt.group(1)), f"rocprofv3 FETCH_SIZE + WRITE_SIZE, {os.path.relpath(tpath, ROOT)}"
        else:
            traffic_note = f"{os.path.relpath(tpath, ROOT)} was taken with other kernel sources than the ones running: not quoted"

    # what a kernel that only reads reaches on this GPU: sweeps over a 4 GiB buffer (long enough that the
    # ramp-up and tail of a launch do not count)
    probe = torch.zeros(1 << 32, dtype=torch.uint8, device=dev)
    n_probe = probe.numel()
    read_ceiling = binding.probe_read_bandwidth(probe, repeats=4)
    del probe

    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)          # reads 2^30 bytes, writes 2^30 bytes
        torch.cuda.synchronize()
        del src, dst

    # capacity: how many cached tokens (batch x context) fit in 288 GB, compressed vs not
    hbm = 288e9
    widths = m["widths"]
    full_tok = 2 * elem * w.n_layers * w.d_kv
    lat_tok = sum(r * lat_elem + (row_meta if r else 0) for pair in widths for r in pair)
    plan = m["plan"]
    roof = roofline_entry(w, m, args.latent)
    roof.update({"traffic": traffic, "traffic_source": traffic_note, "read_ceiling_GBs": read_ceiling,
                 "frac_of_read_ceiling": roof["achieved"] / read_ceiling, "read_ceiling_bytes": n_probe})
    result = {
        "metric": "decode-attn tokens/s over latent KV cache",
        "value": m["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": m["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic" if args.fill == "encode" else "synthetic (random latents, profiling fill)",
        "config": {"workload": w.name, "batch": w.batch, "cached_tokens": w.n_cached, "layers": w.n_layers,
                   "q_heads": w.n_q_heads, "kv_heads": w.n_kv_heads, "d_head": w.d_head, "latent": w.latent, "latent_format": args.latent, "variant": args.variant,
                   "reuse": w.reuse, "policy": w.policy, "reused_head_fraction": float(reuse[1:].mean()) if w.n_layers > 1 else 0.0,
                   "splits": plan.n_splits, "mfma": bool(plan.uses_mfma), "prefill_s": m["prefill_s"],
                   "step_call": "kvcar_append_attend" if m["one_call"] else "kvcar_encode_append + kvcar_decode_attention",
                   "encoder_in_attention_kernel": bool(plan.append_in_kernel) and m["one_call"]},
        "roofline": roof,
        "graph_replay": None if m["graph_ms"] is None else {"ms_per_step": m["graph_ms"], "tokens_per_s": w.batch / (m["graph_ms"] * 1e-3),
                                                             "note": "one captured step (all layers) replayed at fixed positions"},
        "capacity_tokens_288GB": {"uncompressed": int(hbm // full_tok), "latent": int(hbm // lat_tok),
                                  "bytes_per_token_uncompressed": full_tok, "bytes_per_token_latent": lat_tok},
    }
    del m
    torch.cuda.empty_cache()
    if args.workload == 4 and not args.no_workloads and not (args.batch or args.cached):
        # the other four configurations, each at its full size, in the same run (no graph leg, no CPU leg)
        block = {}
        for i in range(4):
            wi = synth.CONFIGS[i].scaled(n_steps=args.steps + args.warmup)
            mi = measure_decode(wi, args, args.steps, args.warmup, graph=False, plain=True)
            ri = roofline_entry(wi, mi, "dtype")
            block[wi.name] = {"config": {"batch": wi.batch, "cached_tokens": wi.n_cached, "layers": wi.n_layers, "dtype": wi.dtype, "latent": wi.latent,
                                         "hidden": wi.hidden, "act": wi.act, "reuse": wi.reuse, "splits": mi["plan"].n_splits,
                                         "mfma": bool(mi["plan"].uses_mfma), "launches_per_layer_fused": mi["plan"].fused,
                                         "encoder_in_attention_kernel": bool(mi["plan"].append_in_kernel)},
                              "ms_per_step": mi["ms_per_step"], "tokens_per_s": mi["tokens_per_s"], "steps": args.steps, "roofline": ri}
            del mi
            torch.cuda.empty_cache()
        result["workloads"] = block
    if args.cpu_seconds > 0:
        result["cpu_baseline"] = cpu_baseline(w, reuse, args.cpu_seconds, n_steps=base.n_steps)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
