"""Pins for the CPU oracle: everything here checks oracle/ against something
other than itself -- hand-worked examples (tests/golden), closed forms of the
recurrence, a library matrix product, brute force and invariants.  CPU only.

References are to arXiv 1803.11389: Eq. (2) SRU, Eq. (3) QRNN, Section 3 and
Eq. (4) multi-time-step blocking.
"""
import math

import numpy as np
import pytest

import oracle
from golden_io import load_example

GOLDEN_TOL = 5e-7   # the fixtures' ln 3 entries are stored as fp32 weights
BLOCKS = (1, 2, 3, 4, 16, 64)


def _rng(seed):
    return np.random.default_rng(seed)


def _rand_sru(rng, n_layers, d, scale=1.0):
    W = [(rng.uniform(-1, 1, (3 * d, d)) * scale / math.sqrt(d)).astype(np.float32) for _ in range(n_layers)]
    b = [rng.uniform(-1, 1, 2 * d).astype(np.float32) for _ in range(n_layers)]
    return W, b


def _rand_qrnn(rng, n_layers, d, k, scale=1.0):
    W = [(rng.uniform(-1, 1, (3 * d, k * d)) * scale / math.sqrt(k * d)).astype(np.float32) for _ in range(n_layers)]
    b = [rng.uniform(-1, 1, 3 * d).astype(np.float32) for _ in range(n_layers)]
    return W, b


# ---------------------------------------------------------------- hand-worked

@pytest.mark.parametrize("name", ["sru_d2_example_a.txt", "sru_d2_example_b.txt"])
@pytest.mark.parametrize("T", BLOCKS)
def test_sru_hand_example(name, T):
    ex = load_example(name)
    bias = None if ex["bias"] is None else [ex["bias"]]
    h, c_final = oracle.sru_forward([ex["W"]], bias, ex["x"], c_init=ex["c_init"][None, :], T=T)
    np.testing.assert_allclose(h, ex["h"], rtol=0, atol=GOLDEN_TOL)
    np.testing.assert_allclose(c_final[0], ex["c"][-1], rtol=0, atol=GOLDEN_TOL)
    # every intermediate cell value: run the prefixes
    for n in range(1, len(ex["x"])):
        _, c_n = oracle.sru_forward([ex["W"]], bias, ex["x"][:n], c_init=ex["c_init"][None, :], T=T)
        np.testing.assert_allclose(c_n[0], ex["c"][n - 1], rtol=0, atol=GOLDEN_TOL)


@pytest.mark.parametrize("T", BLOCKS)
def test_qrnn_hand_example(T):
    ex = load_example("qrnn_d2_k2_example.txt")
    h, c_final, xh = oracle.qrnn_forward([ex["W"]], None, ex["x"], c_init=ex["c_init"][None, :], T=T, k=2)
    np.testing.assert_allclose(h, ex["h"], rtol=0, atol=GOLDEN_TOL)
    np.testing.assert_allclose(c_final[0], ex["c"][-1], rtol=0, atol=GOLDEN_TOL)
    np.testing.assert_array_equal(xh[0, 0], ex["x"][-1].astype(np.float64))
    for n in range(1, len(ex["x"])):
        _, c_n, _ = oracle.qrnn_forward([ex["W"]], None, ex["x"][:n], c_init=ex["c_init"][None, :], T=T, k=2)
        np.testing.assert_allclose(c_n[0], ex["c"][n - 1], rtol=0, atol=GOLDEN_TOL)


def test_step_functions_hand_examples():
    for name in ("sru_d2_example_a.txt", "sru_d2_example_b.txt"):
        ex = load_example(name)
        c = ex["c_init"].copy()
        for t in range(len(ex["x"])):
            h, c = oracle.sru_step(ex["W"], ex["bias"], ex["x"][t], c)
            np.testing.assert_allclose(h, ex["h"][t], rtol=0, atol=GOLDEN_TOL)
            np.testing.assert_allclose(c, ex["c"][t], rtol=0, atol=GOLDEN_TOL)
    ex = load_example("qrnn_d2_k2_example.txt")
    c = ex["c_init"].copy()
    prev = np.zeros(2)
    for t in range(len(ex["x"])):
        h, c = oracle.qrnn_step(ex["W"], None, np.stack([ex["x"][t], prev]), c, 2)
        prev = ex["x"][t]
        np.testing.assert_allclose(h, ex["h"][t], rtol=0, atol=GOLDEN_TOL)
        np.testing.assert_allclose(c, ex["c"][t], rtol=0, atol=GOLDEN_TOL)


# ---------------------------------------------------- blocked == step by step

def _sru_stack_bruteforce(W, b, x, c_init):
    n_layers, d = len(W), W[0].shape[1]
    c = [c_init[l].astype(np.float64) for l in range(n_layers)]
    hs = np.zeros((len(x), d))
    for t in range(len(x)):
        v = x[t].astype(np.float64)
        for l in range(n_layers):
            v, c[l] = oracle.sru_step(W[l], None if b is None else b[l], v, c[l])
        hs[t] = v
    return hs, np.stack(c)


def _qrnn_stack_bruteforce(W, b, x, c_init, xhist, k):
    n_layers, d = len(W), W[0].shape[0] // 3
    c = [c_init[l].astype(np.float64) for l in range(n_layers)]
    # win[l][j] = layer l's input at lag j (row 0 overwritten each step)
    win = [np.concatenate([np.zeros((1, d)), xhist[l].astype(np.float64)], 0) for l in range(n_layers)]
    hs = np.zeros((len(x), d))
    for t in range(len(x)):
        v = x[t].astype(np.float64)
        for l in range(n_layers):
            win[l][0] = v
            v, c[l] = oracle.qrnn_step(W[l], None if b is None else b[l], win[l], c[l], k)
            win[l] = np.roll(win[l], 1, axis=0)   # lag j -> lag j+1; row 0 is rewritten next step
        hs[t] = v
    hist = np.stack([w[1:] for w in win]) if k > 1 else np.zeros((n_layers, 0, d))
    return hs, np.stack(c), hist


@pytest.mark.parametrize("seed,n_layers,d,L,T,bf16", [
    (1, 1, 3, 7, 1, False), (2, 2, 5, 11, 4, False), (3, 3, 8, 20, 16, False),
    (4, 2, 4, 9, 64, False), (5, 2, 6, 13, 5, True),
])
def test_sru_blocked_equals_bruteforce_bitwise(seed, n_layers, d, L, T, bf16):
    from workloads import to_bf16_bits
    rng = _rng(seed)
    W, b = _rand_sru(rng, n_layers, d, scale=2.0)
    if bf16:
        W = [to_bf16_bits(w) for w in W]
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((n_layers, d)).astype(np.float32)
    h, c = oracle.sru_forward(W, b, x, c_init=c0, T=T)
    hb, cb = _sru_stack_bruteforce(W, b, x, c0)
    np.testing.assert_array_equal(h, hb)
    np.testing.assert_array_equal(c, cb)


@pytest.mark.parametrize("seed,n_layers,d,L,T,k,bf16", [
    (11, 1, 3, 7, 1, 2, False), (12, 2, 5, 11, 4, 2, False), (13, 3, 4, 20, 16, 3, False),
    (14, 2, 4, 9, 64, 1, False), (15, 2, 6, 13, 5, 2, True), (16, 1, 3, 2, 3, 4, False),
])
def test_qrnn_blocked_equals_bruteforce_bitwise(seed, n_layers, d, L, T, k, bf16):
    from workloads import to_bf16_bits
    rng = _rng(seed)
    W, b = _rand_qrnn(rng, n_layers, d, k, scale=2.0)
    if bf16:
        W = [to_bf16_bits(w) for w in W]
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((n_layers, d)).astype(np.float32)
    xh0 = rng.standard_normal((n_layers, k - 1, d)).astype(np.float32)
    h, c, xh = oracle.qrnn_forward(W, b, x, c_init=c0, xhist_init=xh0, T=T, k=k)
    hb, cb, xhb = _qrnn_stack_bruteforce(W, b, x, c0, xh0, k)
    np.testing.assert_array_equal(h, hb)
    np.testing.assert_array_equal(c, cb)
    np.testing.assert_array_equal(xh, xhb)


# ------------------------------------------------------- block-size invariance

@pytest.mark.parametrize("cell", ["sru", "qrnn"])
def test_block_size_invariance_bitwise(cell):
    """Section 3: blocking only regroups the same products."""
    rng = _rng(21)
    d, L, n_layers = 16, 70, 3
    x = rng.standard_normal((L, d)).astype(np.float32)
    if cell == "sru":
        W, b = _rand_sru(rng, n_layers, d, 3.0)
        run = lambda T: oracle.sru_forward(W, b, x, T=T)
    else:
        W, b = _rand_qrnn(rng, n_layers, d, 2, 3.0)
        run = lambda T: oracle.qrnn_forward(W, b, x, T=T, k=2)[:2]
    ref = run(1)
    for T in (4, 16, 64, 3, 7, 69, 70, 71, 1000):   # T | L, T does not divide L, T >= L
        out = run(T)
        np.testing.assert_array_equal(out[0], ref[0])
        np.testing.assert_array_equal(out[1], ref[1])


# ----------------------------------------------------------------- closed forms




def test_sru_forget_zero_gives_candidate():
    """f == 0  =>  c_t = xh_t = W x_t  (checked against numpy's product)."""
    rng = _rng(31)
    d, L = 12, 25
    W, _ = _rand_sru(rng, 1, d)
    W[0][d:2 * d] = 0.0
    b = np.zeros(2 * d, np.float32)
    b[:d] = -800.0       # exp(800) overflows to inf in double: sigma == 0 exactly
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((1, d)).astype(np.float32)
    xh = x.astype(np.float64) @ W[0][:d].astype(np.float64).T
    for n in (1, 7, L):
        for T in (1, 4, 16):
            _, c = oracle.sru_forward(W, [b], x[:n], c_init=c0, T=T)
            np.testing.assert_allclose(c[0], xh[n - 1], rtol=1e-13, atol=1e-13)


def test_sru_forget_one_keeps_state():
    rng = _rng(32)
    d, L = 6, 10
    W, _ = _rand_sru(rng, 1, d)
    W[0][d:2 * d] = 0.0
    b = np.zeros(2 * d, np.float32)
    b[:d] = 40.0
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((1, d)).astype(np.float32)
    h, c = oracle.sru_forward(W, [b], x, c_init=c0, T=4)
    # f = 1 - 4e-18 rounds to 1.0 in double
    np.testing.assert_array_equal(c[0], c0[0].astype(np.float64))


def test_sru_forget_half_is_exponential_average():
    """W_f = 0, b_f = 0 => f = 1/2: c_t = sum_s 2^-(t-s+1) xh_s + 2^-(t+1) c_init."""
    rng = _rng(33)
    d, L = 9, 30
    W, _ = _rand_sru(rng, 1, d)
    W[0][d:2 * d] = 0.0
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((1, d)).astype(np.float32)
    xh = x.astype(np.float64) @ W[0][:d].astype(np.float64).T
    for n in (1, 2, 13, L):
        _, c = oracle.sru_forward(W, None, x[:n], c_init=c0, T=5)
        wts = 0.5 ** (n - np.arange(n))                      # 2^-(t-s+1), t = n-1
        expect = (wts[:, None] * xh[:n]).sum(0) + 0.5 ** n * c0[0]
        np.testing.assert_allclose(c[0], expect, rtol=1e-12, atol=1e-13)


def test_sru_reset_zero_is_identity_through_a_stack():
    """r == 0 => h_t = x_t exactly, for any depth."""
    rng = _rng(34)
    d, L, n_layers = 8, 12, 4
    W, _ = _rand_sru(rng, n_layers, d)
    b = []
    for l in range(n_layers):
        W[l][2 * d:] = 0.0
        bl = rng.uniform(-1, 1, 2 * d).astype(np.float32)
        bl[d:] = -800.0
        b.append(bl)
    x = rng.standard_normal((L, d)).astype(np.float32)
    h, _ = oracle.sru_forward(W, b, x, T=4)
    np.testing.assert_array_equal(h, x.astype(np.float64))


def test_sru_zero_weights():
    """W = 0, b = 0: c_t = 2^-(t+1) c_init, h_t = tanh(c_t)/2 + x_t/2."""
    d, L = 5, 8
    rng = _rng(35)
    W = [np.zeros((3 * d, d), np.float32)]
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((1, d)).astype(np.float32)
    h, c = oracle.sru_forward(W, None, x, c_init=c0, T=3)
    ct = c0[0].astype(np.float64)[None, :] * (0.5 ** (np.arange(L) + 1))[:, None]
    np.testing.assert_allclose(h, 0.5 * np.tanh(ct) + 0.5 * x, rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(c[0], ct[-1], rtol=1e-15)


def test_qrnn_zero_weights():
    """W = 0: z = 0, f = o = 1/2, h_t = tanh(2^-(t+1) c_init)/2."""
    d, L = 5, 8
    rng = _rng(36)
    W = [np.zeros((3 * d, 2 * d), np.float32)]
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((1, d)).astype(np.float32)
    h, c, _ = oracle.qrnn_forward(W, None, x, c_init=c0, T=3, k=2)
    ct = c0[0].astype(np.float64)[None, :] * (0.5 ** (np.arange(L) + 1))[:, None]
    np.testing.assert_allclose(h, 0.5 * np.tanh(ct), rtol=1e-14, atol=1e-16)


def _recurrence_closed_form(f, cand, c0):
    """c_t = (prod_{s<=t} f_s) c0 + sum_s (prod_{s<u<=t} f_u)(1-f_s) cand_s,
    evaluated with explicit products (no running state).  f, cand: [L, d]."""
    L = f.shape[0]
    out = np.zeros_like(f)
    for t in range(L):
        acc = np.prod(f[: t + 1], axis=0) * c0
        for s in range(t + 1):
            acc = acc + np.prod(f[s + 1: t + 1], axis=0) * (1.0 - f[s]) * cand[s]
        out[t] = acc
    return out


def _sigmoid(z):
    return 0.5 * (1.0 + np.tanh(0.5 * z))     # a different route to the logistic function


@pytest.mark.parametrize("seed", [41, 42])
def test_sru_layer_against_library_product_and_solved_recurrence(seed):
    """Weight layout (row blocks W | W_f | W_r, bias b_f | b_r) and the whole of
    Eq. (2), with the products from numpy and the recurrence in solved form."""
    rng = _rng(seed)
    d, L = 7, 14
    W, b = _rand_sru(rng, 1, d, scale=3.0)
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((1, d)).astype(np.float32)
    X = x.astype(np.float64)
    U = X @ W[0].astype(np.float64).T                      # [L, 3d]
    cand = U[:, :d]
    f = _sigmoid(U[:, d:2 * d] + b[0][:d])
    r = _sigmoid(U[:, 2 * d:] + b[0][d:])
    c = _recurrence_closed_form(f, cand, c0[0].astype(np.float64))
    h_expect = r * np.tanh(c) + (1.0 - r) * X
    h, c_final = oracle.sru_forward(W, b, x, c_init=c0, T=4)
    np.testing.assert_allclose(h, h_expect, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(c_final[0], c[-1], rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("seed,k", [(43, 2), (44, 3), (45, 1)])
def test_qrnn_layer_against_library_product_and_solved_recurrence(seed, k):
    """Column block j of W multiplies x_{t-j}; rows z | f | o; Eq. (3)."""
    rng = _rng(seed)
    d, L = 6, 12
    W, b = _rand_qrnn(rng, 1, d, k, scale=3.0)
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((1, d)).astype(np.float32)
    xh0 = rng.standard_normal((1, k - 1, d)).astype(np.float32)
    # padded[k-1 + t] = x_t, padded[k-1-1-j] = lag j+1 before the start
    padded = np.concatenate([xh0[0][::-1].astype(np.float64), x.astype(np.float64)], 0)
    Wd = W[0].astype(np.float64)
    U = np.zeros((L, 3 * d))
    for j in range(k):
        U += padded[k - 1 - j: k - 1 - j + L] @ Wd[:, j * d:(j + 1) * d].T
    U += b[0]
    z = np.tanh(U[:, :d])
    f = _sigmoid(U[:, d:2 * d])
    o = _sigmoid(U[:, 2 * d:])
    c = _recurrence_closed_form(f, z, c0[0].astype(np.float64))
    h_expect = o * np.tanh(c)
    h, c_final, xh = oracle.qrnn_forward(W, b, x, c_init=c0, xhist_init=xh0, T=5, k=k)
    np.testing.assert_allclose(h, h_expect, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(c_final[0], c[-1], rtol=1e-11, atol=1e-12)


def test_stack_feeds_h_to_next_layer():
    """A 2-layer run equals layer 2 applied to layer 1's output."""
    rng = _rng(46)
    d, L = 6, 15
    W, b = _rand_sru(rng, 2, d, 2.0)
    x = rng.standard_normal((L, d)).astype(np.float32)
    h2, c2, h_all = oracle.sru_forward(W, b, x, T=4, return_all=True)
    h1, c1 = oracle.sru_forward(W[:1], b[:1], x, T=4)
    np.testing.assert_array_equal(h_all[0], h1)
    # layer 2 alone on h1 (passed as double, so nothing is rounded)
    h2b, c2b = oracle.sru_forward(W[1:], b[1:], h1, T=4)
    np.testing.assert_array_equal(h2, h2b)
    np.testing.assert_array_equal(c2[1], c2b[0])
    np.testing.assert_array_equal(c2[0], c1[0])


def test_linear_projection_against_numpy():
    rng = _rng(47)
    P = rng.standard_normal((9, 4)).astype(np.float32)
    feat = rng.standard_normal((13, 4)).astype(np.float32)
    y = oracle.linear_forward(P, feat)
    np.testing.assert_allclose(y, feat.astype(np.float64) @ P.astype(np.float64).T, rtol=1e-14, atol=1e-15)


# ------------------------------------------------------------------ invariants

def test_chunk_chaining_equals_one_call():
    """Only c (and the QRNN input window) carries state, so a sequence cut at
    any point and resumed gives the same outputs."""
    rng = _rng(51)
    d, L, n_layers, k = 8, 23, 3, 3
    x = rng.standard_normal((L, d)).astype(np.float32)
    W, b = _rand_sru(rng, n_layers, d, 2.0)
    h, c = oracle.sru_forward(W, b, x, T=4)
    for m in (1, 5, 22):
        h1, c1 = oracle.sru_forward(W, b, x[:m], T=4)
        h2, c2 = oracle.sru_forward(W, b, x[m:], c_init=c1, T=4)
        np.testing.assert_array_equal(np.concatenate([h1, h2]), h)
        np.testing.assert_array_equal(c2, c)
    W, b = _rand_qrnn(rng, n_layers, d, k, 2.0)
    h, c, xh = oracle.qrnn_forward(W, b, x, T=4, k=k)
    for m in (1, 2, 5, 22):
        h1, c1, xh1 = oracle.qrnn_forward(W, b, x[:m], T=4, k=k)
        h2, c2, xh2 = oracle.qrnn_forward(W, b, x[m:], c_init=c1, xhist_init=xh1, T=4, k=k)
        np.testing.assert_array_equal(np.concatenate([h1, h2]), h)
        np.testing.assert_array_equal(c2, c)
        np.testing.assert_array_equal(xh2, xh)


def test_cell_state_is_a_convex_combination():
    rng = _rng(52)
    d, L = 10, 40
    W, b = _rand_sru(rng, 1, d, 4.0)
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((1, d)).astype(np.float32)
    xh = x.astype(np.float64) @ W[0][:d].astype(np.float64).T
    for n in range(1, L + 1, 3):
        _, c = oracle.sru_forward(W, b, x[:n], c_init=c0, T=4)
        lo = np.minimum(c0[0], xh[:n].min(0)) - 1e-12
        hi = np.maximum(c0[0], xh[:n].max(0)) + 1e-12
        assert np.all(c[0] >= lo) and np.all(c[0] <= hi)
    Wq, bq = _rand_qrnn(rng, 2, d, 2, 6.0)
    h, c, _ = oracle.qrnn_forward(Wq, bq, x, T=8, k=2)
    assert np.all(np.abs(h) < 1.0) and np.all(np.abs(c) <= 1.0)


def test_future_inputs_do_not_change_past_outputs():
    rng = _rng(53)
    d, L = 6, 20
    W, b = _rand_qrnn(rng, 2, d, 2, 2.0)
    x = rng.standard_normal((L, d)).astype(np.float32)
    h, _, _ = oracle.qrnn_forward(W, b, x, T=7, k=2)
    x2 = x.copy()
    x2[12:] += 1.0
    h2, _, _ = oracle.qrnn_forward(W, b, x2, T=7, k=2)
    np.testing.assert_array_equal(h[:12], h2[:12])
    assert np.abs(h[12:] - h2[12:]).max() > 1e-3


def test_bf16_weights_are_widened_exactly():
    from workloads import bf16_bits_to_f32, to_bf16_bits
    rng = _rng(54)
    d, L = 8, 10
    W, b = _rand_sru(rng, 2, d, 2.0)
    Wb = [to_bf16_bits(w) for w in W]
    Wf = [bf16_bits_to_f32(w) for w in Wb]
    x = rng.standard_normal((L, d)).astype(np.float32)
    np.testing.assert_array_equal(oracle.sru_forward(Wb, b, x, T=4)[0], oracle.sru_forward(Wf, b, x, T=4)[0])
    assert np.abs(oracle.sru_forward(W, b, x, T=4)[0] - oracle.sru_forward(Wf, b, x, T=4)[0]).max() > 1e-6


# ------------------------------------------------------- 8-bit float weights

# Values of OCP FP8 E4M3 codes as the format's specification lists them (bias 7, subnormals
# m/8 * 2^-6, no infinities, largest finite 0x7E = 448), typed here by hand.
E4M3_SPEC_VALUES = {
    0x00: 0.0, 0x01: 2.0 ** -9, 0x02: 2.0 ** -8, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x09: 1.125 * 2.0 ** -6,
    0x0F: 1.875 * 2.0 ** -6, 0x10: 2.0 ** -5, 0x30: 0.5, 0x37: 0.9375, 0x38: 1.0, 0x39: 1.125, 0x3C: 1.5, 0x40: 2.0,
    0x44: 3.0, 0x48: 4.0, 0x70: 128.0, 0x77: 240.0, 0x78: 256.0, 0x7D: 416.0, 0x7E: 448.0,
    0x81: -(2.0 ** -9), 0xB8: -1.0, 0xC0: -2.0, 0xFE: -448.0,
}


class _Fp8:
    """Codes and row scales in the byte layout oracle/ssrnn_oracle.cpp documents, assembled here."""

    def __init__(self, q, scale):
        self.q = np.ascontiguousarray(q, np.uint8)
        self.scale = np.ascontiguousarray(scale, np.float32)

    def blob(self):
        n = self.q.size
        off = (n + 255) // 256 * 256
        out = np.zeros(off + 4 * self.scale.size, np.uint8)
        out[:n] = self.q.reshape(-1)
        out[off:] = self.scale.view(np.uint8)
        return out


def test_fp8_code_values_follow_the_format():
    """One code at a time through a d = 1 QRNN step (k = 1): with the forget row 0 (f = 1/2), c_0 = 0
    and the output row 0 (o = 1/2), h = tanh(tanh(w * x) / 2) / 2 where w is the candidate weight."""
    for code, value in E4M3_SPEC_VALUES.items():
        for scale in (1.0, 0.75):
            W = _Fp8(np.array([[code], [0x00], [0x00]], np.uint8), np.array([scale, 1.0, 1.0], np.float32))
            x = 0.001953125 if abs(value) > 4 else 0.5
            h, c = oracle.qrnn_step(W, None, np.array([[x]]), np.zeros(1), 1)
            assert c[0] == pytest.approx(0.5 * math.tanh(scale * value * x), rel=1e-14, abs=1e-300), hex(code)
            assert h[0] == pytest.approx(0.5 * math.tanh(c[0]), rel=1e-14, abs=1e-300), hex(code)


def test_fp8_weights_equal_their_fp32_values_bitwise():
    """Every non-NaN code, decoded by torch's float8_e4m3fn and scaled by powers of two (exact in
    fp32), run as fp32 weights, must give the same bits as the 8-bit path: pins the decoding of all
    254 codes, the row a scale belongs to and where the scales start (with and without padding)."""
    import torch
    rng = _rng(58)
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], np.uint8)
    for cell, d, k, L, T in (("sru", 16, 1, 9, 4), ("sru", 6, 1, 7, 3), ("qrnn", 8, 2, 9, 4), ("qrnn", 5, 3, 6, 2)):
        ncol = k * d
        q = rng.choice(codes, size=(3 * d, ncol))
        q.reshape(-1)[:min(q.size, codes.size)] = codes[:min(q.size, codes.size)]     # every code at least once where it fits
        scale = (2.0 ** rng.integers(-9, -3, 3 * d)).astype(np.float32)
        dec = torch.from_numpy(q.copy()).view(torch.float8_e4m3fn).to(torch.float32).numpy()
        Wf = (dec * scale[:, None]).astype(np.float32)
        assert np.array_equal(Wf.astype(np.float64), dec.astype(np.float64) * scale[:, None].astype(np.float64))
        W8 = _Fp8(q, scale)
        x = rng.standard_normal((L, d)).astype(np.float32)
        if cell == "sru":
            a, b = oracle.sru_forward([W8, W8], None, x, T=T), oracle.sru_forward([Wf, Wf], None, x, T=T)
        else:
            a, b = oracle.qrnn_forward([W8, W8], None, x, T=T, k=k), oracle.qrnn_forward([Wf, Wf], None, x, T=T, k=k)
        for u, v in zip(a, b):
            np.testing.assert_array_equal(u, v)
        # the step functions read the same storage
        if cell == "sru":
            np.testing.assert_array_equal(oracle.sru_step(W8, None, x[0], np.zeros(d))[0], oracle.sru_step(Wf, None, x[0], np.zeros(d))[0])
        else:
            xw = rng.standard_normal((k, d))
            np.testing.assert_array_equal(oracle.qrnn_step(W8, None, xw, np.zeros(d), k)[0], oracle.qrnn_step(Wf, None, xw, np.zeros(d), k)[0])


def test_fp8_row_scales_are_applied_per_row():
    """Scales that are not powers of two: u = diag(scale) * Q * x, checked through the SRU with the
    reset row at 0 (r = 1/2) and the forget row at 0 (f = 1/2): c_1 = (scale_i * (Q x)_i) / 2."""
    rng = _rng(59)
    d = 12
    q = np.zeros((3 * d, d), np.uint8)
    q[:d] = rng.integers(0x20, 0x50, (d, d)).astype(np.uint8) | (rng.integers(0, 2, (d, d)).astype(np.uint8) << 7)
    scale = rng.uniform(0.01, 0.2, 3 * d).astype(np.float32)
    import torch
    Q = torch.from_numpy(q[:d].copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    x = rng.standard_normal(d)
    h, c = oracle.sru_step(_Fp8(q, scale), None, x, np.zeros(d))
    want_c = 0.5 * scale[:d].astype(np.float64) * (Q @ x)
    np.testing.assert_allclose(c, want_c, rtol=1e-13, atol=0)
    np.testing.assert_allclose(h, 0.5 * np.tanh(want_c) + 0.5 * x, rtol=1e-13, atol=0)


def _bf16_round_numpy(a):
    """Nearest bfloat16, ties to even, of a float32 array, by integer arithmetic
    on the bit patterns (written here, not taken from workloads or the oracle)."""
    u = np.asarray(a, np.float32).view(np.uint32).astype(np.uint64)
    keep = u >> 16
    rest = u & 0xFFFF
    up = (rest > 0x8000) | ((rest == 0x8000) & ((keep & 1) == 1))
    out = ((keep + up.astype(np.uint64)) << 16).astype(np.uint32)
    return out.view(np.float32)


def test_operand_rounding_mode_rounds_only_the_matrix_operand():
    """round_operand=True: the block X of Eq. (4) enters the products as
    bfloat16; the SRU highway term still uses the exact x_t.  Pinned by
    (i) inputs that bfloat16 holds exactly: nothing changes, bit for bit;
    (ii) 1 + 2^-9, a quarter of a bfloat16 step above 1: the gates are those of
    x = 1 while the highway term keeps 1 + 2^-9; (iii) a random layer against
    numpy products of explicitly rounded inputs.  The mode is an argument of
    the call: a call without it rounds nothing, whatever ran before."""
    rng = _rng(77)
    d, L = 6, 9
    W, b = _rand_sru(rng, 1, d, 2.0)
    # (i)
    x_exact = _bf16_round_numpy(rng.standard_normal((L, d)).astype(np.float32))
    ref = oracle.sru_forward(W, b, x_exact, T=4)
    got = oracle.sru_forward(W, b, x_exact, T=4, round_operand=True)
    np.testing.assert_array_equal(got[0], ref[0])
    np.testing.assert_array_equal(got[1], ref[1])
    # (ii) r = 1/2 exactly (W_r = 0, b_r = 0): h = tanh(c)/2 + x/2
    W1 = [np.zeros((3, 1), np.float32)]
    W1[0][0, 0] = 1.0                                   # candidate = x
    xq = np.array([[1.0 + 2.0 ** -9]], np.float32)
    h, c = oracle.sru_forward(W1, None, xq, T=1, round_operand=True)        # f = 1/2: c = (rounded x) / 2
    assert c[0, 0] == 0.5
    assert h[0, 0] == 0.5 * math.tanh(0.5) + 0.5 * float(xq[0, 0])
    h0, c0 = oracle.sru_forward(W1, None, xq, T=1)
    assert c0[0, 0] == 0.5 * float(xq[0, 0])
    # (iii)
    x = rng.standard_normal((L, d)).astype(np.float32)
    Xr = _bf16_round_numpy(x).astype(np.float64)
    U = Xr @ W[0].astype(np.float64).T
    f = _sigmoid(U[:, d:2 * d] + b[0][:d])
    r = _sigmoid(U[:, 2 * d:] + b[0][d:])
    cc = _recurrence_closed_form(f, U[:, :d], np.zeros(d))
    h_expect = r * np.tanh(cc) + (1.0 - r) * x.astype(np.float64)
    h, _ = oracle.sru_forward(W, b, x, T=3, round_operand=True)
    np.testing.assert_allclose(h, h_expect, rtol=1e-11, atol=1e-12)
    # QRNN: window rows are rounded too
    k = 2
    Wq, bq = _rand_qrnn(rng, 1, d, k, 2.0)
    xh0 = rng.standard_normal((1, k - 1, d)).astype(np.float32)
    padded = np.concatenate([_bf16_round_numpy(xh0[0][::-1]).astype(np.float64), Xr], 0)
    Wd = Wq[0].astype(np.float64)
    U = np.zeros((L, 3 * d))
    for j in range(k):
        U += padded[k - 1 - j: k - 1 - j + L] @ Wd[:, j * d:(j + 1) * d].T
    U += bq[0]
    cc = _recurrence_closed_form(_sigmoid(U[:, d:2 * d]), np.tanh(U[:, :d]), np.zeros(d))
    hq, _, _ = oracle.qrnn_forward(Wq, bq, x, xhist_init=xh0, T=4, k=k, round_operand=True)
    np.testing.assert_allclose(hq, _sigmoid(U[:, 2 * d:]) * np.tanh(cc), rtol=1e-11, atol=1e-12)


def test_reverse_direction_is_the_forward_pass_over_the_reversed_sequence():
    """reverse=True walks every layer from the last step to the first (Section 2.1:
    the second direction of a bidirectional network is an independent pass).  Pins:
    (i) bit for bit, reverse(x) = flip(forward(flip(x))), final state and window
    included, for stacks, ragged blocks and given initial state / window;
    (ii) against the step functions walked backwards by hand (they know nothing of
    direction); (iii) h at the last time step depends on x at that step only."""
    rng = _rng(91)
    d, L, n_layers = 5, 11, 3
    W, b = _rand_sru(rng, n_layers, d, 2.0)
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((n_layers, d)).astype(np.float32)
    for T in (1, 4, 16):
        h_r, c_r = oracle.sru_forward(W, b, x, c_init=c0, T=T, reverse=True)
        h_f, c_f = oracle.sru_forward(W, b, x[::-1].copy(), c_init=c0, T=T)
        np.testing.assert_array_equal(h_r, h_f[::-1])
        np.testing.assert_array_equal(c_r, c_f)
    # (ii) one SRU layer by hand, from the last step to the first
    c = c0[0].astype(np.float64).copy()
    h_hand = np.zeros((L, d))
    for t in range(L - 1, -1, -1):
        h_hand[t], c = oracle.sru_step(W[0], b[0], x[t], c)
    h1, c1 = oracle.sru_forward(W[:1], b[:1], x, c_init=c0[:1], T=4, reverse=True)
    np.testing.assert_array_equal(h1, h_hand)
    np.testing.assert_array_equal(c1[0], c)
    # (iii)
    x2 = x.copy()
    x2[:-1] += 1.0
    h2, _ = oracle.sru_forward(W[:1], b[:1], x2, c_init=c0[:1], T=4, reverse=True)
    np.testing.assert_array_equal(h2[-1], h1[-1])
    assert not np.array_equal(h2[0], h1[0])
    # QRNN, window of 3: the window of step t holds x_t, x_{t+1}, x_{t+2}; xhist_init are the inputs beyond the end
    k = 3
    Wq, bq = _rand_qrnn(rng, 2, d, k, 2.0)
    xh0 = rng.standard_normal((2, k - 1, d)).astype(np.float32)
    for T in (1, 3, 16):
        h_r, c_r, xh_r = oracle.qrnn_forward(Wq, bq, x, c_init=c0[:2], xhist_init=xh0, T=T, k=k, reverse=True)
        h_f, c_f, xh_f = oracle.qrnn_forward(Wq, bq, x[::-1].copy(), c_init=c0[:2], xhist_init=xh0, T=T, k=k)
        np.testing.assert_array_equal(h_r, h_f[::-1])
        np.testing.assert_array_equal(c_r, c_f)
        np.testing.assert_array_equal(xh_r, xh_f)
    c = c0[0].astype(np.float64).copy()
    h_hand = np.zeros((L, d))
    ext = np.concatenate([x.astype(np.float64), xh0[0].astype(np.float64)], 0)      # row L + j: the input j+1 steps beyond the end
    for t in range(L - 1, -1, -1):
        h_hand[t], c = oracle.qrnn_step(Wq[0], bq[0], ext[t:t + k], c, k)
    h1, c1, xh1 = oracle.qrnn_forward(Wq[:1], bq[:1], x, c_init=c0[:1], xhist_init=xh0[:1], T=4, k=k, reverse=True)
    np.testing.assert_array_equal(h1, h_hand)
    np.testing.assert_array_equal(c1[0], c)
    np.testing.assert_array_equal(xh1[0], x[:k - 1].astype(np.float64))              # lag j+1 of the walk's end = time j


def test_edge_cases():
    d = 4
    rng = _rng(55)
    W, b = _rand_sru(rng, 2, d)
    c0 = rng.standard_normal((2, d)).astype(np.float32)
    h, c = oracle.sru_forward(W, b, np.zeros((0, d), np.float32), c_init=c0, T=4)   # L = 0
    assert h.shape == (0, d)
    np.testing.assert_array_equal(c, c0.astype(np.float64))
    with pytest.raises(ValueError):
        oracle.sru_forward(W, b, np.zeros((3, d), np.float32), T=0)
    with pytest.raises(ValueError):
        oracle.qrnn_forward([np.zeros((3 * d, 2 * d), np.float32)], None, np.zeros((3, d), np.float32), T=0, k=2)
