"""Pins for the LSTM oracle (Eq. 1 of arXiv 1803.11389; Section 3.1 for the
order: input products of T steps together, feedback products step by step).

As for the SRU / QRNN oracle, everything here compares it with something other
than itself: a hand-worked example with feedback (tests/golden), the separately
written one-step brute force, closed forms of special cases, a scalar network
iterated with math.tanh, a library matrix product for the two weight layouts,
block-size invariance, chunk chaining, the stack rule and boundedness.
"""
import math

import numpy as np
import pytest

import oracle
from golden_io import load_example

GOLDEN_TOL = 5e-7   # the fixture's ln 3 entries are stored as fp32 weights
BLOCKS = (1, 2, 3, 4, 16)


def _rand_lstm(rng, n_layers, d, scale=1.0):
    W = [(rng.uniform(-1, 1, (4 * d, d)) * scale / math.sqrt(d)).astype(np.float32) for _ in range(n_layers)]
    U = [(rng.uniform(-1, 1, (4 * d, d)) * scale / math.sqrt(d)).astype(np.float32) for _ in range(n_layers)]
    b = [rng.uniform(-1, 1, 4 * d).astype(np.float32) for _ in range(n_layers)]
    return W, U, b


def _sig(z):
    return 1.0 / (1.0 + np.exp(-z))


# ---------------------------------------------------------------- hand-worked

@pytest.mark.parametrize("T", BLOCKS)
def test_lstm_hand_example(T):
    ex = load_example("lstm_d2_example.txt")
    args = ([ex["W"]], [ex["U"]], [ex["bias"]])
    h, h_final, c_final = oracle.lstm_forward(*args, ex["x"], h_init=ex["h_init"][None], c_init=ex["c_init"][None], T=T)
    np.testing.assert_allclose(h, ex["h"], rtol=0, atol=GOLDEN_TOL)
    np.testing.assert_allclose(c_final[0], ex["c"][-1], rtol=0, atol=GOLDEN_TOL)
    np.testing.assert_allclose(h_final[0], ex["h"][-1], rtol=0, atol=GOLDEN_TOL)
    for n in range(1, len(ex["x"])):          # every intermediate cell value: run the prefixes
        _, h_n, c_n = oracle.lstm_forward(*args, ex["x"][:n], h_init=ex["h_init"][None], c_init=ex["c_init"][None], T=T)
        np.testing.assert_allclose(c_n[0], ex["c"][n - 1], rtol=0, atol=GOLDEN_TOL)
        np.testing.assert_allclose(h_n[0], ex["h"][n - 1], rtol=0, atol=GOLDEN_TOL)


def test_lstm_step_hand_example():
    ex = load_example("lstm_d2_example.txt")
    h, c = ex["h_init"].copy(), ex["c_init"].copy()
    for t in range(len(ex["x"])):
        h, c = oracle.lstm_step(ex["W"], ex["U"], ex["bias"], ex["x"][t], h, c)
        np.testing.assert_allclose(h, ex["h"][t], rtol=0, atol=GOLDEN_TOL)
        np.testing.assert_allclose(c, ex["c"][t], rtol=0, atol=GOLDEN_TOL)


# ---------------------------------------------------- blocked == step by step

def _stack_bruteforce(W, U, b, x, h_init, c_init):
    n_layers, d = len(W), W[0].shape[1]
    h = [h_init[l].astype(np.float64) for l in range(n_layers)]
    c = [c_init[l].astype(np.float64) for l in range(n_layers)]
    out = np.zeros((len(x), d))
    for t in range(len(x)):
        v = x[t].astype(np.float64)
        for l in range(n_layers):
            h[l], c[l] = oracle.lstm_step(W[l], U[l], None if b is None else b[l], v, h[l], c[l])
            v = h[l]
        out[t] = v
    return out, np.stack(h), np.stack(c)


@pytest.mark.parametrize("seed,n_layers,d,L,T,with_bias", [
    (1, 1, 3, 9, 1, True), (2, 2, 5, 11, 4, False), (3, 3, 4, 20, 16, True), (4, 2, 8, 7, 64, True), (5, 1, 1, 6, 2, True),
])
def test_lstm_blocked_equals_bruteforce_bitwise(seed, n_layers, d, L, T, with_bias):
    rng = np.random.default_rng(7000 + seed)
    W, U, b = _rand_lstm(rng, n_layers, d, scale=2.0)
    if not with_bias:
        b = None
    x = rng.standard_normal((L, d)).astype(np.float32)
    h0 = rng.uniform(-1, 1, (n_layers, d))
    c0 = rng.standard_normal((n_layers, d))
    h, hf, cf = oracle.lstm_forward(W, U, b, x, h_init=h0, c_init=c0, T=T)
    h_bf, hf_bf, cf_bf = _stack_bruteforce(W, U, b, x, h0, c0)
    np.testing.assert_array_equal(h, h_bf)
    np.testing.assert_array_equal(hf, hf_bf)
    np.testing.assert_array_equal(cf, cf_bf)


def test_lstm_result_does_not_depend_on_the_block_size():
    rng = np.random.default_rng(7100)
    W, U, b = _rand_lstm(rng, 2, 6, scale=2.0)
    x = rng.standard_normal((23, 6)).astype(np.float32)
    ref = oracle.lstm_forward(W, U, b, x, T=1)
    for T in (2, 4, 5, 23, 64):                         # divides, does not divide, equals, exceeds the length
        got = oracle.lstm_forward(W, U, b, x, T=T)
        for u, v in zip(got, ref):
            np.testing.assert_array_equal(u, v)


# ------------------------------------------------------------- closed forms

def test_lstm_all_zero_weights_halve_the_cell():
    """W = U = b = 0: f = i = o = 1/2 and c-hat = 0, so c_t = c_init / 2^(t+1) and h_t = tanh(c_t) / 2."""
    d, L = 4, 9
    Z = [np.zeros((4 * d, d), np.float32)]
    c0 = np.array([[1.0, -2.0, 0.5, 3.0]])
    h, hf, cf = oracle.lstm_forward(Z, Z, None, np.ones((L, d), np.float32), h_init=np.full((1, d), 0.7), c_init=c0, T=4)
    for t in range(L):
        np.testing.assert_allclose(h[t], 0.5 * np.tanh(c0[0] / 2.0 ** (t + 1)), rtol=1e-15, atol=0)
    np.testing.assert_allclose(cf[0], c0[0] / 2.0 ** L, rtol=1e-15, atol=0)
    np.testing.assert_array_equal(hf[0], h[-1])


def test_lstm_closed_input_gate_and_open_forget_gate_keep_the_cell():
    """i == 0 (b_i = -800), f == 1 (b_f = +800): c_t = c_init whatever the weights say; with o == 1
    (b_o = +800) h_t = tanh(c_init) for every t."""
    rng = np.random.default_rng(7200)
    d, L = 5, 12
    W, U, _ = _rand_lstm(rng, 1, d)
    for M in (W[0], U[0]):
        M[: 3 * d] = 0.0                                  # gates from their biases alone; the candidate keeps its weights
    b = np.zeros(4 * d, np.float32)
    b[0:d], b[d:2 * d], b[2 * d:3 * d] = 800.0, -800.0, 800.0
    c0 = rng.standard_normal((1, d))
    h, hf, cf = oracle.lstm_forward(W, U, [b], rng.standard_normal((L, d)).astype(np.float32), c_init=c0, T=5)
    np.testing.assert_array_equal(cf, c0)
    np.testing.assert_allclose(h, np.broadcast_to(np.tanh(c0), (L, d)), rtol=0, atol=1e-15)


def test_lstm_closed_forget_gate_and_open_input_gate_give_the_candidate():
    """f == 0, i == 1, o == 1: c_t = c-hat_t and h_t = tanh(c-hat_t), with
    c-hat_t = tanh(W_c x_t + U_c h_{t-1} + b_c): a plain tanh recurrent network, iterated here with numpy."""
    rng = np.random.default_rng(7300)
    d, L = 4, 10
    W, U, _ = _rand_lstm(rng, 1, d, scale=2.0)
    for M in (W[0], U[0]):
        M[: 3 * d] = 0.0
    b = np.zeros(4 * d, np.float32)
    b[0:d], b[d:2 * d], b[2 * d:3 * d] = -800.0, 800.0, 800.0
    b[3 * d:] = rng.uniform(-1, 1, d).astype(np.float32)
    x = rng.standard_normal((L, d)).astype(np.float32)
    h0 = rng.uniform(-1, 1, (1, d))
    h, hf, cf = oracle.lstm_forward(W, U, [b], x, h_init=h0, c_init=rng.standard_normal((1, d)), T=3)
    Wc, Uc, bc = W[0][3 * d:].astype(np.float64), U[0][3 * d:].astype(np.float64), b[3 * d:].astype(np.float64)
    prev = h0[0]
    for t in range(L):
        chat = np.tanh(Wc @ x[t].astype(np.float64) + Uc @ prev + bc)
        prev = np.tanh(chat)
        np.testing.assert_allclose(h[t], prev, rtol=0, atol=1e-14)
    np.testing.assert_allclose(cf[0], chat, rtol=0, atol=1e-14)


def test_scalar_lstm_iterated_with_math_functions():
    """d = 1: every product is a scalar, so the whole network is a dozen math.exp / math.tanh calls per step."""
    w = [0.7, -1.3, 0.4, 1.9]
    u = [-0.6, 0.8, 1.1, -1.7]
    b = [0.1, -0.2, 0.3, 0.05]
    xs = [0.5, -1.0, 2.0, 0.25, -0.75, 1.5]
    W = [np.array(w, np.float32).reshape(4, 1)]
    U = [np.array(u, np.float32).reshape(4, 1)]
    bb = [np.array(b, np.float32)]
    w, u, b = [float(np.float32(v)) for v in w], [float(np.float32(v)) for v in u], [float(np.float32(v)) for v in b]
    h, hf, cf = oracle.lstm_forward(W, U, bb, np.array(xs, np.float32).reshape(-1, 1), h_init=[[0.3]], c_init=[[-0.4]], T=4)
    hp, c = 0.3, -0.4
    for t, x in enumerate(xs):
        f = 1.0 / (1.0 + math.exp(-(w[0] * x + u[0] * hp + b[0])))
        i = 1.0 / (1.0 + math.exp(-(w[1] * x + u[1] * hp + b[1])))
        o = 1.0 / (1.0 + math.exp(-(w[2] * x + u[2] * hp + b[2])))
        g = math.tanh(w[3] * x + u[3] * hp + b[3])
        c = f * c + i * g
        hp = o * math.tanh(c)
        assert abs(h[t, 0] - hp) <= 1e-15
    assert abs(cf[0, 0] - c) <= 1e-15 and abs(hf[0, 0] - hp) <= 1e-15


def test_lstm_without_feedback_against_library_product_and_solved_recurrence():
    """U = 0: the gates depend on x alone, so they come from ONE library matrix product over the whole
    sequence (which pins the row blocks f | i | o | c-hat and the row-major layout of W), and
    c_t = f_t c_{t-1} + i_t chat_t has the solution c_t = P_t (c_init + sum_{s<=t} i_s chat_s / P_s) with
    P_t = f_0 ... f_t, evaluated with cumulative products and sums, no loop over time."""
    rng = np.random.default_rng(7400)
    d, L = 6, 17
    W, _, b = _rand_lstm(rng, 1, d, scale=1.5)
    U = [np.zeros((4 * d, d), np.float32)]
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((1, d))
    h, hf, cf = oracle.lstm_forward(W, U, b, x, h_init=rng.uniform(-1, 1, (1, d)), c_init=c0, T=4)
    pre = x.astype(np.float64) @ W[0].astype(np.float64).T + b[0].astype(np.float64)      # [L, 4d]
    f, i, o, g = _sig(pre[:, :d]), _sig(pre[:, d:2 * d]), _sig(pre[:, 2 * d:3 * d]), np.tanh(pre[:, 3 * d:])
    P = np.cumprod(f, axis=0)
    c = P * (c0[0] + np.cumsum(i * g / P, axis=0))
    np.testing.assert_allclose(h, o * np.tanh(c), rtol=0, atol=1e-12)
    np.testing.assert_allclose(cf[0], c[-1], rtol=0, atol=1e-12)


def test_lstm_feedback_products_against_library_product():
    """Every step of a random network again, the two matrix-vector products taken by the library from the
    oracle's own previous output: pins the layout of U (rows f | i | o | c-hat, row-major, multiplied with
    h_{t-1}, not with h_t and not transposed) and that the bias enters once."""
    rng = np.random.default_rng(7500)
    d, L = 7, 13
    W, U, b = _rand_lstm(rng, 1, d, scale=2.0)
    x = rng.standard_normal((L, d)).astype(np.float32)
    h0 = rng.uniform(-1, 1, (1, d))
    c0 = rng.standard_normal((1, d))
    h, hf, cf = oracle.lstm_forward(W, U, b, x, h_init=h0, c_init=c0, T=5)
    Wd, Ud, bd = W[0].astype(np.float64), U[0].astype(np.float64), b[0].astype(np.float64)
    c = c0[0]
    for t in range(L):
        prev = h0[0] if t == 0 else h[t - 1]
        pre = Wd @ x[t].astype(np.float64) + Ud @ prev + bd
        c = _sig(pre[:d]) * c + _sig(pre[d:2 * d]) * np.tanh(pre[3 * d:])
        np.testing.assert_allclose(h[t], _sig(pre[2 * d:3 * d]) * np.tanh(c), rtol=0, atol=1e-13)
        c = c.copy()
    np.testing.assert_allclose(cf[0], c, rtol=0, atol=1e-12)


# ------------------------------------------------------ structure of the call

def test_lstm_stack_feeds_h_to_the_next_layer():
    rng = np.random.default_rng(7600)
    d, L = 5, 9
    W, U, b = _rand_lstm(rng, 3, d)
    x = rng.standard_normal((L, d)).astype(np.float32)
    h0 = rng.uniform(-1, 1, (3, d))
    c0 = rng.standard_normal((3, d))
    h, hf, cf, h_all = oracle.lstm_forward(W, U, b, x, h_init=h0, c_init=c0, T=4, return_all=True)
    cur = x.astype(np.float64)
    for l in range(3):
        cur, hf_l, cf_l = oracle.lstm_forward([W[l]], [U[l]], [b[l]], cur, h_init=h0[l:l + 1], c_init=c0[l:l + 1], T=2)
        np.testing.assert_array_equal(h_all[l], cur)
        np.testing.assert_array_equal(hf[l], hf_l[0])
        np.testing.assert_array_equal(cf[l], cf_l[0])
    np.testing.assert_array_equal(h, cur)


def test_lstm_chunk_chaining_equals_one_call():
    rng = np.random.default_rng(7700)
    d, L, m = 4, 19, 7
    W, U, b = _rand_lstm(rng, 2, d, scale=2.0)
    x = rng.standard_normal((L, d)).astype(np.float32)
    whole = oracle.lstm_forward(W, U, b, x, T=4)
    a = oracle.lstm_forward(W, U, b, x[:m], T=4)
    z = oracle.lstm_forward(W, U, b, x[m:], h_init=a[1], c_init=a[2], T=4)
    np.testing.assert_array_equal(np.concatenate([a[0], z[0]]), whole[0])
    np.testing.assert_array_equal(z[1], whole[1])
    np.testing.assert_array_equal(z[2], whole[2])


def test_lstm_empty_sequence_returns_the_initial_state():
    rng = np.random.default_rng(7800)
    W, U, b = _rand_lstm(rng, 2, 3)
    h0, c0 = rng.uniform(-1, 1, (2, 3)), rng.standard_normal((2, 3))
    h, hf, cf = oracle.lstm_forward(W, U, b, np.zeros((0, 3), np.float32), h_init=h0, c_init=c0, T=4)
    assert h.shape == (0, 3)
    np.testing.assert_array_equal(hf, h0)
    np.testing.assert_array_equal(cf, c0)


def test_lstm_outputs_are_bounded():
    """|h_t| < 1 always; |c_t| <= |c_{t-1}| + 1 since f, i < 1 and |c-hat| < 1."""
    rng = np.random.default_rng(7900)
    W, U, b = _rand_lstm(rng, 2, 8, scale=6.0)
    x = (rng.standard_normal((40, 8)) * 5).astype(np.float32)
    h, hf, cf, h_all = oracle.lstm_forward(W, U, b, x, T=8, return_all=True)
    assert np.all(np.abs(h_all) < 1.0)
    assert np.all(np.abs(cf) <= 40.0)
