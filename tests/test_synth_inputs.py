"""The seeded input generators: deterministic, chunk-addressable, right shapes."""
import numpy as np

import lq_synth


def test_configs_match_the_five_layers():
    c = lq_synth.CONFIGS
    assert (c["c1"].r, c["c1"].c, c["c1"].n_tokens, c["c1"].bits, c["c1"].mode) == (512, 512, 2048, 4, "nu")
    assert (c["c2"].r, c["c2"].c, c["c2"].n_tokens) == (4096, 4096, 262144)
    assert (c["c3"].r, c["c3"].c, c["c3"].bits) == (4096, 11008, 3)
    assert (c["c4"].r, c["c4"].c, c["c4"].mode, c["c4"].group_size) == (28672, 8192, "aff", 128)
    assert (c["c5"].r, c["c5"].c, c["c5"].bits, c["c5"].group_size) == (53248, 16384, 2, 64)
    assert (c["c5nu"].mode, c["c5nu"].bits, c["c5nu"].seed) == ("nu", 3, c["c5"].seed)


def test_weights_deterministic_and_row_addressable():
    cfg = lq_synth.CONFIGS["c1"]
    W = lq_synth.weights(cfg)
    assert W.shape == (512, 512) and W.dtype == np.float32
    np.testing.assert_array_equal(W, lq_synth.weights(cfg))
    rows = [300, 5, 511]
    np.testing.assert_array_equal(lq_synth.weights(cfg, rows), W[rows])
    frac = np.mean(np.abs(W) > 0.1)
    assert 0.003 < frac < 0.01            # 1 % of entries drawn from N(0, 0.2^2)


def test_activation_chunks_and_outlier_channels():
    cfg = lq_synth.CONFIGS["c1"]
    X = lq_synth.activations(cfg)
    assert X.shape == (2048, 512) and X.dtype == np.float32
    ch = lq_synth.outlier_channels(cfg)
    assert ch.size == 8
    s = X.std(axis=0)
    assert np.all(s[ch] > 15) and np.all(np.delete(s, ch) < 1.5)
    small = cfg.scaled(n_tokens=1000)
    np.testing.assert_array_equal(lq_synth.activation_chunk(small, 0), X[:1000])
    silu = lq_synth.CONFIGS["c3"].scaled(c=64, n_tokens=512)
    Xs = lq_synth.activation_chunk(silu, 0)
    assert Xs.shape == (512, 64) and abs(float(Xs.mean())) < 0.05
