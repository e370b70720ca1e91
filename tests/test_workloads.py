"""The synthetic generators: shapes, determinism, and the statistics the design notes promise."""
import numpy as np

from workloads import CONFIGS, bf16_bits_to_f64, f64_to_bf16_bits, gen_item, gen_lengths, gen_weights, get_config


def test_bf16_round_trip_and_rounding():
    x = np.array([1.0, -2.5, 0.1, 3.140625, 1.00390625, 1.01171875])
    b = f64_to_bf16_bits(x)
    y = bf16_bits_to_f64(b)
    assert y[0] == 1.0 and y[1] == -2.5 and y[3] == 3.140625
    assert y[4] == 1.0              # 1 + 2^-8 is a tie: rounds to even (1.0)
    assert y[5] == 1.015625         # 1 + 3*2^-8 is a tie: rounds to even (1 + 2^-6)
    assert np.all(np.abs(y - x) <= np.abs(x) * 2.0 ** -8)
    assert np.array_equal(f64_to_bf16_bits(y), b)


def test_shapes_and_determinism():
    cfg = get_config(1, seqlen=256)
    a, b = gen_item(cfg, 0), gen_item(cfg, 0)
    assert a["q_win"].shape == (28, 32, 128) and a["k"].shape == (4, 256, 128) and a["v"].shape == (4, 256, 128)
    assert a["k"].dtype == np.uint16
    assert all(np.array_equal(a[n], b[n]) for n in ("q_win", "k", "v"))
    c = gen_item(get_config(2, seqlen=256), 1)
    assert not np.array_equal(a["k"], c["k"])


def test_ar1_statistics_and_text_tail():
    cfg = get_config(2, seqlen=4096)
    k = bf16_bits_to_f64(gen_item(cfg, 0)["k"])
    audio = k[:, 512:4096 - 256, :]
    lag1 = (audio[:, 1:] * audio[:, :-1]).mean() / (audio ** 2).mean()
    assert 0.9 < lag1 < 0.98
    text = k[:, -256:, :]
    assert 0.9 < text.std() < 1.1
    lag1_text = (text[:, 1:] * text[:, :-1]).mean()
    assert abs(lag1_text) < 0.05


def test_lengths_and_weights():
    cfg = CONFIGS[5]
    L = gen_lengths(cfg)
    assert len(L) == 8 and L.min() >= 2048 and L.max() <= 32768
    assert np.array_equal(L, gen_lengths(cfg))
    w = gen_weights(cfg).reshape(8, 2)
    np.testing.assert_allclose(w.sum(axis=1), 1.0, rtol=1e-6)
    w4 = gen_weights(CONFIGS[4])
    assert w4.shape == (192,) and abs(w4.sum() - 1.0) < 1e-5
    assert np.sort(w4)[-10:].sum() > 0.3          # concentrated: few heads dominate
