"""Memory accounting of the oracle pinned to the numbers the paper prints
(tests/golden/paper_accounting.txt lists them with their places in the paper)."""
import numpy as np

from oracle import kvcar_oracle as O
from paper_2512_06727_amd import synth


def test_eq3_worked_example():
    n = O.kv_cache_bytes(2, 24, 1024, 2048, 8)
    assert n == 1610612736
    assert round(n / 1e9, 2) == 1.61
    assert round(n / (345e6 * 2), 2) == 2.33


def test_table2_autoencoder_savings():
    trunc = lambda x: int(x * 1e4) / 100      # the paper truncates to two decimals
    assert O.savings_autoencoder(11, 22, 0.5) == 0.25
    assert trunc(O.savings_autoencoder(6, 22, 0.5)) == 13.63
    assert trunc(O.savings_autoencoder(5, 22, 0.5)) == 11.36
    assert O.savings_autoencoder(22, 22, 0.5) == 0.5
    assert int(O.savings_autoencoder(10, 12, 0.5) * 1e3) / 10 == 41.6


def test_table3_reuse_savings():
    trunc = lambda x: int(x * 1e4) / 100
    assert O.savings_reuse(144, 12, 12) == 0.5
    assert O.savings_reuse(72, 12, 12) == 0.25
    assert trunc(O.savings_reuse(19, 12, 12)) == 6.59
    assert trunc(O.savings_reuse(25, 12, 12)) == 8.68
    assert O.savings_reuse(36, 12, 12) == 0.125


def test_table4_combined_from_latent_widths():
    """10 of 12 GPT-2 layers compressed 2x (layers 0 and 2 left uncompressed), 36 head
    tensors reused (3 K + 3 V heads in each odd layer).  A reused head inside a
    compressed layer gives back its proportional share of the latent, which is the
    accounting behind the paper's 41.6 + 12.5/2 = 47.85 (exact value 138/288)."""
    H, dh, D = 12, 64, 768
    widths = np.zeros((12, 2))
    for layer in range(12):
        stored = H - (3 if layer % 2 == 1 else 0)
        per_head = dh if layer in (0, 2) else dh // 2
        widths[layer, :] = stored * per_head
    full = O.kv_cache_bytes(2, 12, D, 1024, 8)
    got = 1.0 - O.latent_cache_bytes(2, widths, 1024, 8) / full
    assert abs(got - 138 / 288) < 1e-15
    assert abs(got * 100 - 47.85) < 0.1
    # the two parts separately
    assert abs(O.savings_autoencoder(10, 12, 0.5) + O.savings_reuse(36, 12, 12) / 2 - got) < 1e-15


def test_latent_bytes_of_the_synthetic_workloads():
    """Eq. 3 generalised to the per-layer stored widths of the synthetic workloads."""
    w = synth.CONFIGS[4]
    reuse = synth.reuse_map(w)
    widths = np.array([[synth.autoencoder(w, n, which, reuse).latent for which in (0, 1)] for n in range(w.n_layers)])
    stored = (~reuse).sum(-1)
    np.testing.assert_array_equal(widths, stored * (w.latent // w.n_kv_heads))
    full = O.kv_cache_bytes(2, w.n_layers, w.d_kv, 8192, 256)
    assert full == 47244640256                                  # "about 47 GB uncompressed"
    lat = O.latent_cache_bytes(2, widths, 8192, 256)
    assert lat == 2 * int(widths.sum()) * 8192 * 256
    assert lat < full // 2
