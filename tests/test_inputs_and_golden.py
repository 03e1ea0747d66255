"""Input generator determinism / structure, and the oracle regression fixture."""
import json
import os

import numpy as np

from ea_inputs import CONFIGS, make_layer, widen, bf16_bits_from_f64, f64_from_bf16_bits
from tests.golden.make_golden import build

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_regression_fixture():
    with open(os.path.join(HERE, "golden", "oracle_tiny.json")) as f:
        ref = json.load(f)
    cur = build()
    for key in ("mu", "sigma_diag", "sigma_fro", "scores"):
        assert np.allclose(cur[key], ref[key], rtol=1e-12, atol=1e-14), key
    assert cur["idx"] == ref["idx"]


def test_generator_is_seeded_and_shaped():
    cfg = CONFIGS["c2"]
    a = make_layer(cfg, n=300, window=32)
    b = make_layer(cfg, n=300, window=32)
    c = make_layer(cfg, layer=1, n=300, window=32)
    assert a["k"].dtype == np.uint16 and a["k"].shape == (1, 8, 300, 128)
    assert a["q_win"].shape == (1, 32, 32, 128) and a["v"].shape == (1, 8, 300, 128)
    assert np.array_equal(a["k"], b["k"]) and np.array_equal(a["q_win"], b["q_win"])
    assert not np.array_equal(a["k"], c["k"])
    assert a["q_pos0"] == 268 and a["t_next"] == 300
    # value rows: N(0,1) x log-normal token scale -> mean squared norm ~ d * e^{0.5}
    v = widen(a["v"])
    assert 0.7 < (v * v).sum(-1).mean() / (128 * np.exp(0.5)) < 1.4
    # outlier channels: rotary-invariant pair energy shows the +8 offsets in 4 channels/head
    k = widen(a["k"])[0, 0]
    pair_energy = (k[:, :64] ** 2 + k[:, 64:] ** 2).mean(axis=0)
    assert (pair_energy > 40).sum() >= 2


def test_bf16_round_trip():
    x = np.array([0.0, 1.0, -2.5, 1.00390625, 3.1415926, 1e-3, 65504.0, -1e30])
    bits = bf16_bits_from_f64(x)
    back = f64_from_bf16_bits(bits)
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)
    assert np.array_equal(bf16_bits_from_f64(back), bits)          # idempotent
    # ties to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert f64_from_bf16_bits(bf16_bits_from_f64(np.array([1 + 2.0 ** -8])))[0] == 1.0
    assert f64_from_bf16_bits(bf16_bits_from_f64(np.array([1 + 3 * 2.0 ** -8])))[0] == 1 + 2.0 ** -6
