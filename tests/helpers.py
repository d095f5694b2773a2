"""Glue shared by the tests: builds an oracle instance from a synthetic workload.
Holds no arithmetic of the method."""
import numpy as np

from oracle import kvcar_oracle as O
from paper_2512_06727_amd import synth


def oracle_ae(ae: synth.AEWeights) -> O.Autoencoder:
    cv = lambda pairs: [(w.double().numpy(), None if b is None else b.double().numpy()) for w, b in pairs]
    return O.Autoencoder(ae.heads, cv(ae.enc), cv(ae.dec), act=ae.act, slope=ae.slope)


def build_oracle(w: synth.Workload, reuse=None, with_bias=False, layers=None):
    reuse = synth.reuse_map(w) if reuse is None else reuse
    orc = O.KVCAROracle(w.n_layers, w.n_q_heads, w.n_kv_heads, w.d_head, w.batch, w.max_seq, w.dtype)
    for layer in range(w.n_layers):
        orc.set_reuse_map(layer, reuse[layer, 0], reuse[layer, 1])
    for layer in (range(w.n_layers) if layers is None else layers):
        for which in (0, 1):
            orc.set_autoencoder(layer, which, oracle_ae(synth.autoencoder(w, layer, which, reuse, with_bias)))
    return orc


def oracle_prefill(orc, w, layer, t0, t1, b0=0, b1=None):
    b1 = w.batch if b1 is None else b1
    k = synth.kv_tokens(w, layer, 0, b0, b1, t0, t1).double().numpy()
    v = synth.kv_tokens(w, layer, 1, b0, b1, t0, t1).double().numpy()
    assert b0 == 0
    orc.encode_append(layer, k, v, t0)
