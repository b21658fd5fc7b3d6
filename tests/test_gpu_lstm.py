"""lstm_forward on the GPU (the paper's comparison network, Eq. 1, run as Section 3.1 describes) against
the CPU oracle, element by element: every h_t, and every layer's final h and c, to the fp32 bar of 1e-4.
Widths include the paper's own LSTM sizes (350 and 700, Section 4), which are no multiple of the kernels'
256-column chunks (350 not even of four values: the one-value-per-lane path), blocks shorter and longer than
the 16 steps one pass over W takes, ragged last blocks, biases and initial states."""
import math

import numpy as np
import pytest

import oracle
from golden_io import load_example
from gpu_util import gpu_lstm, max_abs

pytestmark = pytest.mark.gpu

TOL = 1e-4


def _inputs(seed, n_layers, d, L, scale=1.5, bias=True):
    rng = np.random.default_rng(seed)
    W = [(rng.uniform(-1, 1, (4 * d, d)) * scale / math.sqrt(d)).astype(np.float32) for _ in range(n_layers)]
    U = [(rng.uniform(-1, 1, (4 * d, d)) * scale / math.sqrt(d)).astype(np.float32) for _ in range(n_layers)]
    b = [rng.uniform(-1, 1, 4 * d).astype(np.float32) for _ in range(n_layers)] if bias else None
    x = rng.standard_normal((L, d)).astype(np.float32)
    h0 = rng.uniform(-1, 1, (n_layers, d)).astype(np.float32)
    c0 = rng.standard_normal((n_layers, d)).astype(np.float32)
    return W, U, b, x, h0, c0


@pytest.mark.parametrize("d,n_layers,L,T,bias", [
    (2, 1, 5, 1, True), (7, 2, 9, 4, True), (64, 2, 21, 16, False), (256, 3, 40, 8, True), (350, 2, 37, 16, True),
    (700, 2, 50, 5, True), (1024, 4, 70, 64, True), (2560, 2, 24, 16, True), (512, 1, 33, 1, True), (100, 3, 18, 40, False),
    (4096, 1, 6, 2, True),
])
def test_lstm_against_oracle(d, n_layers, L, T, bias):
    print(f"lstm d={d} layers={n_layers} L={L} T={T} bias={bias}", flush=True)
    W, U, b, x, h0, c0 = _inputs(8000 + d + T, n_layers, d, L, bias=bias)
    ref = oracle.lstm_forward(W, U, b, x, h_init=h0, c_init=c0, T=T)
    got = gpu_lstm(W, U, b, x, h0, c0, T=T)
    for u, r in zip(got, ref):
        assert np.all(np.isfinite(u))
        assert max_abs(u, r) <= TOL, max_abs(u, r)


def test_lstm_hand_example_on_gpu():
    ex = load_example("lstm_d2_example.txt")
    h, hf, cf = gpu_lstm([ex["W"]], [ex["U"]], [ex["bias"]], ex["x"], ex["h_init"][None], ex["c_init"][None], T=2)
    assert max_abs(h, ex["h"]) <= 1e-6 and max_abs(cf[0], ex["c"][-1]) <= 1e-6 and max_abs(hf[0], ex["h"][-1]) <= 1e-6


def test_lstm_result_does_not_depend_on_the_block_size_bit_for_bit():
    """Every dot product adds its columns in the same order whatever the block size, so T changes no bit."""
    W, U, b, x, h0, c0 = _inputs(8100, 3, 512, 45)
    ref = gpu_lstm(W, U, b, x, h0, c0, T=1)
    for T in (2, 4, 7, 16, 45, 200):
        got = gpu_lstm(W, U, b, x, h0, c0, T=T)
        for u, v in zip(got, ref):
            np.testing.assert_array_equal(u, v)


def test_lstm_chunks_chain_through_final_h_and_c():
    W, U, b, x, h0, c0 = _inputs(8200, 2, 256, 31)
    whole = gpu_lstm(W, U, b, x, h0, c0, T=4)
    a = gpu_lstm(W, U, b, x[:13], h0, c0, T=4)
    z = gpu_lstm(W, U, b, x[13:], a[1], a[2], T=4)
    np.testing.assert_array_equal(np.concatenate([a[0], z[0]]), whole[0])
    np.testing.assert_array_equal(z[1], whole[1])
    np.testing.assert_array_equal(z[2], whole[2])
    ref = oracle.lstm_forward(W, U, b, x, h_init=h0, c_init=c0, T=4)
    assert max_abs(whole[0], ref[0]) <= TOL


def test_lstm_empty_sequence_and_default_state():
    W, U, b, x, h0, c0 = _inputs(8300, 2, 128, 0)
    h, hf, cf = gpu_lstm(W, U, b, x, h0, c0, T=4)
    assert h.shape == (0, 128)
    np.testing.assert_array_equal(hf, h0)
    np.testing.assert_array_equal(cf, c0)
    W, U, b, x, _, _ = _inputs(8301, 2, 128, 10)
    got = gpu_lstm(W, U, b, x, None, None, T=4)               # NULL initial state: zeros
    ref = oracle.lstm_forward(W, U, b, x, T=4)
    for u, r in zip(got, ref):
        assert max_abs(u, r) <= TOL


def test_lstm_saturated_gates_stay_finite():
    """Pre-activations of +-80: the fast sigmoid and tanh must saturate cleanly."""
    W, U, b, x, h0, c0 = _inputs(8400, 1, 256, 12, scale=1.0)
    b[0][:] = np.where(np.arange(4 * 256) % 2 == 0, 80.0, -80.0).astype(np.float32)
    got = gpu_lstm(W, U, b, x, h0, c0, T=4)
    ref = oracle.lstm_forward(W, U, b, x, h_init=h0, c_init=c0, T=4)
    for u, r in zip(got, ref):
        assert np.all(np.isfinite(u))
        assert max_abs(u, r) <= TOL


def test_lstm_rejects_bad_arguments():
    import torch
    import paper_1803_11389_amd as ss
    d = 64
    W = [torch.zeros((4 * d, d), device="cuda")]
    x = torch.zeros((3, d), device="cuda")
    with pytest.raises(ss.SsrnnError) as e:
        ss.lstm_forward(W, W, None, x, T=4, flags=1)
    assert e.value.status == 1                                  # SSRNN_EINVAL
    with pytest.raises(ss.SsrnnError) as e:
        ss.lstm_forward(W, W, None, x, T=4, workspace=ss.Workspace(256))
    assert e.value.status == 3                                  # SSRNN_EWORKSPACE
    with pytest.raises(ss.SsrnnError):
        ss.lstm_forward(W, W, None, x, T=0)
    torch.cuda.synchronize()
