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


def _random_cases(n=24, seed=20241201):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        d = int(rng.choice([1, 3, 4, 12, 60, 64, 96, 250, 256, 260, 350, 384, 512, 700, 1000, 1024, 1536]))
        n_layers = int(rng.integers(1, 4))
        T = int(rng.choice([1, 2, 3, 5, 8, 15, 16, 17, 33]))
        L = int(rng.integers(1, 3 * min(T, 16) + 4))
        cases.append((d, n_layers, L, T, bool(rng.integers(0, 2)), int(rng.integers(0, 1 << 30))))
    return cases


@pytest.mark.parametrize("case", _random_cases(), ids=lambda c: f"d{c[0]}-n{c[1]}-L{c[2]}-T{c[3]}{'-b' if c[4] else ''}")
def test_lstm_random_shape_against_oracle(case):
    d, n_layers, L, T, bias, seed = case
    print(f"lstm case {case}", flush=True)
    W, U, b, x, h0, c0 = _inputs(seed, n_layers, d, L, scale=2.0, bias=bias)
    ref = oracle.lstm_forward(W, U, b, x, h_init=h0, c_init=c0, T=T)
    got = gpu_lstm(W, U, b, x, h0, c0, T=T)
    for u, r in zip(got, ref):
        assert u.shape == r.shape and np.all(np.isfinite(u))
        assert max_abs(u, r) <= TOL, max_abs(u, r)


def test_lstm_forward_can_be_recorded_into_a_graph():
    """lstm_forward only enqueues kernels on the given stream (no memset, no host synchronisation, no
    allocation), so a call can be captured into a HIP graph: every replay, with new inputs and with eager
    work in between, gives the eager result bit for bit."""
    import torch
    import paper_1803_11389_amd as ss
    from gpu_util import to_dev
    d, n_layers, L, T = 256, 2, 19, 4
    W, U, b, x0, h0, c0 = _inputs(8500, n_layers, d, L)
    Wd, Ud, bd = [to_dev(w) for w in W], [to_dev(u) for u in U], [to_dev(v) for v in b]
    x, h_in, c_in = to_dev(x0), to_dev(h0), to_dev(c0)
    ws = ss.Workspace(ss.load_library().lstm_workspace_bytes(n_layers, d, T))
    h = torch.empty((L, d), dtype=torch.float32, device="cuda")
    hf = torch.empty((n_layers, d), dtype=torch.float32, device="cuda")
    cf = torch.empty((n_layers, d), dtype=torch.float32, device="cuda")

    def call():
        ss.lstm_forward(Wd, Ud, bd, x, h_in, c_in, T=T, h=h, h_final=hf, c_final=cf, workspace=ws)

    call()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            call()
    torch.cuda.synchronize()
    rng = np.random.default_rng(8501)
    for rep in range(3):
        x.copy_(to_dev(rng.standard_normal((L, d)).astype(np.float32)))
        c_in.copy_(to_dev(rng.standard_normal((n_layers, d)).astype(np.float32)))
        h.zero_(); hf.zero_(); cf.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got = (h.clone(), hf.clone(), cf.clone())
        call()                                   # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(got[0], h) and torch.equal(got[1], hf) and torch.equal(got[2], cf), rep
    ref = oracle.lstm_forward(W, U, b, x.cpu().numpy(), h_init=h0, c_init=c_in.cpu().numpy(), T=T)
    assert max_abs(h.cpu().numpy(), ref[0]) <= TOL and max_abs(cf.cpu().numpy(), ref[2]) <= TOL


def test_lstm_comparator_workloads_against_oracle():
    """The two workloads the bench times the comparison network on, with the bench's inputs: the paper's large
    LSTM (one layer of 700, Section 4) over its 1,024 steps, and the first 40 steps of the 8-layer d = 2560 stack."""
    import workloads as wl
    small = wl.LSTM_CONFIGS[1]
    inp = wl.make_lstm_inputs(small)
    print(f"{small.name}: L={small.L}", flush=True)
    ref = oracle.lstm_forward(inp["W"], inp["U"], None, inp["x"], T=16)
    got = gpu_lstm(inp["W"], inp["U"], None, inp["x"], T=16)
    for u, r in zip(got, ref):
        assert max_abs(u, r) <= TOL, max_abs(u, r)
    big = wl.LSTM_CONFIGS[0]
    inp = wl.make_lstm_inputs(big, L=40)
    print(f"{big.name}: first 40 steps", flush=True)
    ref = oracle.lstm_forward(inp["W"], inp["U"], None, inp["x"], T=16)
    got = gpu_lstm(inp["W"], inp["U"], None, inp["x"], T=16)
    for u, r in zip(got, ref):
        assert np.all(np.isfinite(u))
        assert max_abs(u, r) <= TOL, max_abs(u, r)
