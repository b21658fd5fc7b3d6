"""The seeded input generators: determinism, prefix property, distributions,
bf16 rounding.  No arithmetic of the method is involved."""
import math

import numpy as np

import workloads as wl


def test_deterministic_and_distinct_streams():
    a = wl.uniform(7, 3, (5, 4), 0.5)
    b = wl.uniform(7, 3, (5, 4), 0.5)
    np.testing.assert_array_equal(a, b)
    assert not np.array_equal(a, wl.uniform(7, 4, (5, 4), 0.5))
    assert not np.array_equal(a, wl.uniform(8, 3, (5, 4), 0.5))
    assert a.dtype == np.float32 and np.abs(a).max() <= 0.5


def test_prefix_property_and_chunking():
    n = (1 << 22) + 1000           # crosses the generator's chunk boundary
    full = wl.normal(11, 1, (n,))
    np.testing.assert_array_equal(full[:5000], wl.normal(11, 1, (5000,)))
    np.testing.assert_array_equal(full[-1500:], wl.normal(11, 1, (n,))[-1500:])


def test_moments():
    z = wl.normal(5, 1, (400000,)).astype(np.float64)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1.0) < 0.01
    assert abs((z ** 3).mean()) < 0.03 and abs((z ** 4).mean() - 3.0) < 0.1
    u = wl.uniform(5, 2, (400000,), 2.0).astype(np.float64)
    assert abs(u.mean()) < 0.01 and abs(u.var() - 4.0 / 3.0) < 0.01
    assert u.min() < -1.99 and u.max() > 1.99


def test_bf16_round_to_nearest_even():
    f = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -2.5, 0.0, 1.0 + 2 ** -8 + 2 ** -20], np.float32)
    bits = wl.to_bf16_bits(f)
    back = wl.bf16_bits_to_f32(bits)
    # ties go to the even mantissa: 1+2^-8 -> 1, 1+3*2^-8 -> 1+2^-6
    np.testing.assert_array_equal(back, np.array([1.0, 1.0, 1.0 + 2 ** -7, 1.0 + 2 ** -6, -2.5, 0.0, 1.0 + 2 ** -7], np.float32))
    r = wl.uniform(3, 9, (10000,), 1.0)
    rb = wl.bf16_bits_to_f32(wl.to_bf16_bits(r))
    assert np.all(np.abs(rb - r) <= np.abs(r) * 2.0 ** -8)


def test_config_table_matches_the_benchmark_list():
    c1, c2, c3, c4, c5 = wl.CONFIGS
    assert (c1.cell, c1.n_layers, c1.d, c1.L, c1.Ts) == ("sru", 1, 128, 64, (4,))
    assert (c2.cell, c2.n_layers, c2.d, c2.L, c2.d_feat, c2.Ts) == ("sru", 4, 1024, 1000, 40, (1, 4, 16, 64))
    assert (c3.cell, c3.n_layers, c3.d, c3.L, c3.k, c3.Ts) == ("qrnn", 4, 1024, 1000, 2, (1, 4, 16, 64))
    assert (c4.cell, c4.n_layers, c4.d, c4.L, c4.Ts) == ("sru", 8, 4096, 2048, (1, 2, 4, 8, 16, 32, 64, 128))
    assert (c5.cell, c5.n_layers, c5.d, c5.L, c5.k, c5.wdtype, c5.Ts) == ("qrnn", 8, 4096, 4096, 2, "bf16", (16, 64, 256))
    assert c4.weight_bytes_per_layer() == 12288 * 4096 * 4 == c5.weight_bytes_per_layer()
    assert abs(c4.algorithmic_bytes_per_step(4) / 1e6 - 402.9) < 0.1
    assert abs(c4.flops_per_step() / 1e6 - 805.3) < 0.1


def test_make_inputs_shapes_and_bounds():
    c1 = wl.CONFIGS[0]
    inp = wl.make_inputs(c1)
    assert inp["x"].shape == (64, 128) and len(inp["W"]) == 1 and inp["W"][0].shape == (384, 128)
    assert np.abs(inp["W"][0]).max() <= 1 / math.sqrt(128)
    short = wl.make_inputs(c1, L=10)
    np.testing.assert_array_equal(short["x"], inp["x"][:10])
    c2 = wl.CONFIGS[1]
    inp2 = wl.make_inputs(c2, L=8, n_layers=1)
    assert inp2["feat"].shape == (8, 40) and inp2["P"].shape == (1024, 40) and len(inp2["W"]) == 1


def test_fp8_encoder_against_library_conversion():
    """to_fp8_e4m3_bits against torch's float8_e4m3fn conversion: random values over seven decades,
    every code's own value, every midpoint between neighbouring codes (ties go to the even code),
    saturation at 448."""
    import torch
    rng = np.random.default_rng(3)
    a = np.concatenate([rng.standard_normal(50000).astype(np.float32) * s for s in (1e-3, 1e-2, 0.1, 1, 10, 100, 300)])
    want = torch.from_numpy(a).clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    np.testing.assert_array_equal(wl.to_fp8_e4m3_bits(a), want)
    codes = np.arange(256, dtype=np.uint8)
    dec = torch.from_numpy(codes).view(torch.float8_e4m3fn).float().numpy()
    ok = ~np.isnan(dec)
    np.testing.assert_array_equal(wl.to_fp8_e4m3_bits(dec[ok]), codes[ok])
    pos = np.sort(dec[ok & (codes < 0x80)])
    mid = ((pos[1:].astype(np.float64) + pos[:-1]) / 2).astype(np.float32)
    np.testing.assert_array_equal(wl.to_fp8_e4m3_bits(mid), torch.from_numpy(mid).to(torch.float8_e4m3fn).view(torch.uint8).numpy())
    np.testing.assert_array_equal(wl.to_fp8_e4m3_bits(np.array([449, 1000, -1e9], np.float32)), [0x7E, 0x7E, 0xFE])


def test_fp8_quantizer_scales_rows_to_the_format_maximum():
    rng = np.random.default_rng(4)
    w = (rng.standard_normal((12, 40)) * rng.uniform(0.01, 3, (12, 1))).astype(np.float32)
    w[5] = 0
    q = wl.quantize_fp8(w)
    assert q.q.dtype == np.uint8 and q.scale.dtype == np.float32 and q.scale[5] == 1.0 and not q.q[5].any()
    assert ((q.q & 0x7F).max(axis=1)[np.arange(12) != 5] == 0x7E).all()      # each row's largest magnitude maps to 448
    blob = q.blob()
    assert blob.size == 512 + 48 and np.array_equal(blob[:480], q.q.reshape(-1)) and not blob[480:512].any()
    np.testing.assert_array_equal(blob[512:].view(np.float32), q.scale)


def test_lstm_comparator_inputs():
    """The comparison network's inputs: shapes, bounds, determinism, distinct draws for W and U, and the
    byte count per step that the bench prices it with (U every step, W once per block of up to 16 steps)."""
    lc = wl.LSTM_CONFIGS[1]                     # the paper's large LSTM: one layer of width 700
    a, b = wl.make_lstm_inputs(lc, L=5), wl.make_lstm_inputs(lc, L=5)
    assert len(a["W"]) == len(a["U"]) == lc.n_layers
    assert a["W"][0].shape == a["U"][0].shape == (4 * lc.d, lc.d) and a["x"].shape == (5, lc.d)
    assert a["W"][0].dtype == a["x"].dtype == np.float32
    np.testing.assert_array_equal(a["W"][0], b["W"][0])
    np.testing.assert_array_equal(a["x"], b["x"])
    assert not np.array_equal(a["W"][0], a["U"][0])
    assert np.abs(a["W"][0]).max() <= 1.0 / np.sqrt(lc.d) and np.abs(a["U"][0]).max() <= 1.0 / np.sqrt(lc.d)
    big = wl.LSTM_CONFIGS[0]
    per_matrix = 4 * big.d * big.d * 4
    assert big.weight_bytes_per_layer() == 2 * per_matrix
    small = 14 * big.d * 4 * big.n_layers
    assert big.algorithmic_bytes_per_step(1) == big.n_layers * 2 * per_matrix + small
    assert big.algorithmic_bytes_per_step(64) == big.algorithmic_bytes_per_step(16) == big.n_layers * per_matrix * 17 / 16 + small
