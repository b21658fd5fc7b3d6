"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element
by element, on the same seeded inputs.

Tolerance (fp32 weights): max |delta| <= 1e-4 on every output and on the final
state.  bf16 weights: max |delta| / max |reference| <= 2e-2 over the tensor.
"""
import math

import numpy as np
import pytest

import oracle
import workloads as wl
from golden_io import load_example
from gpu_util import gpu_qrnn, gpu_sru, max_abs, to_dev

pytestmark = pytest.mark.gpu

TOL = 1e-4
GENERIC, VALU, MFMA = 1 << 4, 2 << 4, 3 << 4
STAGES = 1


def _rng(seed):
    return np.random.default_rng(seed)


def _sru_inputs(seed, n_layers, d, L, with_bias=True, with_c0=True, scale=1.0, bf16=False):
    rng = _rng(seed)
    W = [(rng.uniform(-1, 1, (3 * d, d)) * scale / math.sqrt(d)).astype(np.float32) for _ in range(n_layers)]
    if bf16:
        W = [wl.to_bf16_bits(w) for w in W]
    b = [rng.uniform(-1, 1, 2 * d).astype(np.float32) for _ in range(n_layers)] if with_bias else None
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((n_layers, d)).astype(np.float32) if with_c0 else None
    return W, b, x, c0


def _qrnn_inputs(seed, n_layers, d, L, k, with_bias=True, with_state=True, scale=1.0, bf16=False):
    rng = _rng(seed)
    W = [(rng.uniform(-1, 1, (3 * d, k * d)) * scale / math.sqrt(k * d)).astype(np.float32) for _ in range(n_layers)]
    if bf16:
        W = [wl.to_bf16_bits(w) for w in W]
    b = [rng.uniform(-1, 1, 3 * d).astype(np.float32) for _ in range(n_layers)] if with_bias else None
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((n_layers, d)).astype(np.float32) if with_state else None
    xh0 = rng.standard_normal((n_layers, k - 1, d)).astype(np.float32) if with_state else None
    return W, b, x, c0, xh0


def _check_sru(W, b, x, c0, T, flags, tol=TOL):
    print(f"sru d={W[0].shape[1]} layers={len(W)} L={len(x)} T={T} flags={flags:#x}", flush=True)
    h_ref, c_ref = oracle.sru_forward(W, b, x, c_init=c0, T=T)
    h, c = gpu_sru(W, b, x, c0, T=T, flags=flags)
    assert np.all(np.isfinite(h)) and np.all(np.isfinite(c))
    assert max_abs(h, h_ref) <= tol, f"h: {max_abs(h, h_ref)}"
    assert max_abs(c, c_ref) <= tol, f"c: {max_abs(c, c_ref)}"


def _check_qrnn(W, b, x, c0, xh0, T, k, flags, tol=TOL):
    print(f"qrnn d={W[0].shape[0] // 3} layers={len(W)} L={len(x)} T={T} k={k} flags={flags:#x}", flush=True)
    h_ref, c_ref, xh_ref = oracle.qrnn_forward(W, b, x, c_init=c0, xhist_init=xh0, T=T, k=k)
    h, c, xh = gpu_qrnn(W, b, x, c0, xh0, T=T, k=k, flags=flags)
    assert np.all(np.isfinite(h)) and np.all(np.isfinite(c))
    assert max_abs(h, h_ref) <= tol, f"h: {max_abs(h, h_ref)}"
    assert max_abs(c, c_ref) <= tol, f"c: {max_abs(c, c_ref)}"
    if k > 1:
        # the window of the top layers holds computed activations, layer 0's holds inputs (exact)
        np.testing.assert_array_equal(xh[0], xh_ref[0].astype(np.float32))
        assert max_abs(xh, xh_ref) <= tol


# ----------------------------------------------------- hand-worked examples

@pytest.mark.parametrize("T", [1, 2, 3, 8])
def test_hand_examples_on_gpu(T):
    for name in ("sru_d2_example_a.txt", "sru_d2_example_b.txt"):
        ex = load_example(name)
        bias = None if ex["bias"] is None else [ex["bias"]]
        h, c = gpu_sru([ex["W"]], bias, ex["x"], ex["c_init"][None, :], T=T)
        assert max_abs(h, ex["h"]) <= 2e-6 and max_abs(c[0], ex["c"][-1]) <= 2e-6
    ex = load_example("qrnn_d2_k2_example.txt")
    h, c, xh = gpu_qrnn([ex["W"]], None, ex["x"], ex["c_init"][None, :], None, T=T, k=2)
    assert max_abs(h, ex["h"]) <= 2e-6 and max_abs(c[0], ex["c"][-1]) <= 2e-6
    np.testing.assert_array_equal(xh[0, 0], ex["x"][-1])


# -------------------------------------------------- generic kernel, any shape

@pytest.mark.parametrize("d,n_layers,L,T", [
    (2, 1, 5, 1), (5, 2, 11, 4), (64, 3, 33, 16), (128, 2, 19, 64), (70, 2, 21, 7), (130, 1, 9, 9),
])
def test_sru_generic_small_shapes(d, n_layers, L, T):
    W, b, x, c0 = _sru_inputs(100 + d, n_layers, d, L, scale=2.0)
    _check_sru(W, b, x, c0, T, GENERIC)


@pytest.mark.parametrize("d,n_layers,L,T,k", [
    (2, 1, 5, 1, 2), (5, 2, 11, 4, 2), (64, 3, 33, 16, 3), (128, 2, 19, 64, 2), (70, 2, 21, 7, 1),
    (6, 2, 2, 1, 4), (6, 3, 9, 2, 4), (33, 2, 40, 1, 3),
])
def test_qrnn_generic_small_shapes(d, n_layers, L, T, k):
    W, b, x, c0, xh0 = _qrnn_inputs(200 + d + k, n_layers, d, L, k, scale=2.0)
    _check_qrnn(W, b, x, c0, xh0, T, k, GENERIC)


def test_generic_bf16_weights_match_exactly_widened_weights():
    W, b, x, c0 = _sru_inputs(301, 2, 96, 20, bf16=True)
    _check_sru(W, b, x, c0, 4, GENERIC)      # fp32 activations: the fp32 tolerance holds
    Wq, bq, xq, cq, xhq = _qrnn_inputs(302, 2, 96, 20, 2, bf16=True)
    _check_qrnn(Wq, bq, xq, cq, xhq, 5, 2, GENERIC)


def test_defaults_zero_state_and_no_bias():
    W, _, x, _ = _sru_inputs(303, 2, 64, 17, with_bias=False, with_c0=False)
    _check_sru(W, None, x, None, 4, 0)
    Wq, _, xq, _, _ = _qrnn_inputs(304, 2, 64, 17, 2, with_bias=False, with_state=False)
    _check_qrnn(Wq, None, xq, None, None, 4, 2, 0)


# ------------------------------------------- bandwidth (vector ALU) kernel

@pytest.mark.parametrize("d,n_layers,L,T", [
    (256, 2, 13, 1), (256, 1, 10, 2), (512, 3, 21, 4), (768, 2, 19, 3), (1024, 2, 37, 8),
    (1024, 2, 20, 5), (2048, 2, 9, 4), (4096, 2, 9, 4), (4096, 2, 5, 8), (4096, 1, 3, 1), (1280, 2, 7, 2),
    (1024, 2, 50, 16), (512, 2, 30, 12), (4096, 2, 20, 16), (256, 3, 40, 9),
])
def test_sru_valu_kernel(d, n_layers, L, T):
    W, b, x, c0 = _sru_inputs(400 + d + T, n_layers, d, L, scale=2.0)
    _check_sru(W, b, x, c0, T, VALU | STAGES)


@pytest.mark.parametrize("d,n_layers,L,T,k", [
    (256, 2, 13, 1, 2), (512, 3, 21, 4, 2), (1024, 2, 37, 8, 2), (1024, 2, 11, 2, 3), (256, 2, 6, 1, 4),
    (2048, 2, 9, 4, 2), (4096, 1, 6, 4, 2), (768, 2, 10, 3, 1), (1024, 2, 40, 16, 2), (512, 2, 35, 11, 3),
])
def test_qrnn_valu_kernel(d, n_layers, L, T, k):
    W, b, x, c0, xh0 = _qrnn_inputs(500 + d + T + k, n_layers, d, L, k, scale=2.0)
    _check_qrnn(W, b, x, c0, xh0, T, k, VALU | STAGES)


@pytest.mark.parametrize("cell,d,n_layers,L,T,k", [
    ("sru", 512, 2, 23, 4, 1), ("sru", 1024, 3, 30, 1, 1), ("sru", 4096, 1, 9, 2, 1), ("sru", 2048, 2, 21, 8, 1),
    ("qrnn", 512, 2, 26, 4, 2), ("qrnn", 1024, 2, 17, 3, 3), ("qrnn", 4096, 1, 10, 4, 2), ("sru", 8192, 1, 6, 4, 1),
])
def test_valu_kernel_bf16_weights(cell, d, n_layers, L, T, k):
    """bf16 weights on the vector-ALU kernel: the weights are widened in registers
    and the input block stays fp32, so the result meets the fp32 bar against the
    oracle on the same bf16 weights."""
    print(f"valu bf16 {cell} d={d} layers={n_layers} L={L} T={T} k={k}", flush=True)
    if cell == "sru":
        W, b, x, c0 = _sru_inputs(1300 + d + T, n_layers, d, L, bf16=True)
        h_ref, c_ref = oracle.sru_forward(W, b, x, c_init=c0, T=T)
        h, c = gpu_sru(W, b, x, c0, T=T, flags=VALU)
    else:
        W, b, x, c0, xh0 = _qrnn_inputs(1300 + d + T + k, n_layers, d, L, k, bf16=True)
        h_ref, c_ref, _ = oracle.qrnn_forward(W, b, x, c_init=c0, xhist_init=xh0, T=T, k=k)
        h, c, _ = gpu_qrnn(W, b, x, c0, xh0, T=T, k=k, flags=VALU)
    assert max_abs(h, h_ref) <= TOL and max_abs(c, c_ref) <= TOL, (max_abs(h, h_ref), max_abs(c, c_ref))


def test_valu_kernel_refuses_what_it_cannot_take():
    import paper_1803_11389_amd as ss
    W, b, x, c0 = _sru_inputs(601, 1, 100, 4)
    with pytest.raises(ss.SsrnnError) as e:
        gpu_sru(W, b, x, c0, T=4, flags=VALU)
    assert e.value.status == 2


# ------------------------------------------------------- properties on the GPU

def test_block_size_invariance_on_gpu():
    W, b, x, c0 = _sru_inputs(701, 3, 512, 50, scale=2.0)
    ref = gpu_sru(W, b, x, c0, T=1)
    for T in (2, 3, 4, 7, 8, 16, 49, 50, 64):
        out = gpu_sru(W, b, x, c0, T=T)
        assert max_abs(out[0], ref[0]) <= TOL and max_abs(out[1], ref[1]) <= TOL


def test_chunk_chaining_on_gpu():
    W, b, x, c0, xh0 = _qrnn_inputs(702, 3, 256, 30, 3, scale=2.0)
    h, c, xh = gpu_qrnn(W, b, x, c0, xh0, T=4, k=3)
    for m in (1, 2, 13):
        h1, c1, xh1 = gpu_qrnn(W, b, x[:m], c0, xh0, T=4, k=3)
        h2, c2, xh2 = gpu_qrnn(W, b, x[m:], c1, xh1, T=4, k=3)
        assert max_abs(np.concatenate([h1, h2]), h) <= 1e-5
        assert max_abs(c2, c) <= 1e-5 and max_abs(xh2, xh) <= 1e-5


@pytest.mark.parametrize("cell,d,k,T,bf16,packed", [
    ("sru", 256, 1, 4, False, False), ("qrnn", 256, 3, 4, False, False), ("qrnn", 512, 2, 16, False, True),
    ("sru", 512, 1, 32, True, False), ("qrnn", 256, 4, 2, False, False),
])
def test_stream_session_chunks_of_any_length(cell, d, k, T, bf16, packed):
    """One stream fed through StreamSession in chunks of 1, 5, 0, 17, ... steps (shorter and longer than
    T, and shorter than the QRNN window) against the oracle run over the whole sequence at once."""
    import torch
    import paper_1803_11389_amd as ss
    from gpu_util import _weights
    chunks = [1, 5, 0, 17, 3, 1, 1, 40, 2, 9]
    L = sum(chunks)
    if cell == "sru":
        W, b, x, c0 = _sru_inputs(720 + d + T, 2, d, L, scale=2.0, bf16=bf16)
        xh0 = None
        h_ref, c_ref = oracle.sru_forward(W, b, x, c_init=c0, T=T)
    else:
        W, b, x, c0, xh0 = _qrnn_inputs(720 + d + T + k, 2, d, L, k, scale=2.0, bf16=bf16)
        h_ref, c_ref, xh_ref = oracle.qrnn_forward(W, b, x, c_init=c0, xhist_init=xh0, T=T, k=k)
    sess = ss.StreamSession(cell, _weights(W, packed), [to_dev(v) for v in b], T=T, k=k,
                            flags=ss.WEIGHTS_PACKED if packed else 0, c_init=to_dev(c0), xhist_init=to_dev(xh0))
    xd = to_dev(x)
    outs, at = [], 0
    for n in chunks:
        print(f"session {cell} d={d} chunk {n} at {at}", flush=True)
        outs.append(sess.feed(xd[at:at + n]).cpu().numpy())
        at += n
    torch.cuda.synchronize()
    h = np.concatenate(outs)
    assert sess.steps == L and h.shape == (L, d)
    if bf16:
        assert _rel_err(h, h_ref) <= BF16_TOL and _rel_err(sess.c.cpu().numpy(), c_ref) <= BF16_TOL
    else:
        assert max_abs(h, h_ref) <= TOL, max_abs(h, h_ref)
        assert max_abs(sess.c.cpu().numpy(), c_ref) <= TOL
        if cell == "qrnn":
            assert max_abs(sess.xhist.cpu().numpy(), xh_ref) <= TOL


def test_empty_sequence_returns_initial_state():
    W, b, x, c0, xh0 = _qrnn_inputs(703, 2, 64, 0, 3)
    h, c, xh = gpu_qrnn(W, b, x, c0, xh0, T=4, k=3)
    assert h.shape == (0, 64)
    np.testing.assert_array_equal(c, c0)
    np.testing.assert_array_equal(xh, xh0)
    Ws, bs, xs, cs = _sru_inputs(704, 2, 64, 0, with_c0=False)
    _, c = gpu_sru(Ws, bs, xs, None, T=4)
    np.testing.assert_array_equal(c, np.zeros((2, 64), np.float32))


def test_saturated_gates_stay_finite():
    """Large pre-activations: sigma and tanh saturate to 0 / 1 / -1 without NaN."""
    d, L = 64, 12
    rng = _rng(705)
    W = [(rng.uniform(-1, 1, (3 * d, d)) * 40.0).astype(np.float32)]
    x = (rng.standard_normal((L, d)) * 10).astype(np.float32)
    h_ref, c_ref = oracle.sru_forward(W, None, x, T=4)
    h, c = gpu_sru(W, None, x, None, T=4)
    assert np.all(np.isfinite(h)) and np.all(np.isfinite(c))
    scale = max(1.0, float(np.abs(c_ref).max()))
    assert max_abs(h, h_ref) <= 1e-4 * max(1.0, float(np.abs(h_ref).max()))
    assert max_abs(c, c_ref) <= 1e-5 * scale * 10


# ---------------------------------------------------------------- config C1

def test_config1_sru_d128():
    c1 = wl.CONFIGS[0]
    inp = wl.make_inputs(c1)
    for flags in (0, GENERIC):
        _check_sru(inp["W"], None, inp["x"], None, c1.Ts[0], flags)


# ------------------------------------------------------ matrix-core kernel

BF16_TOL = 2e-2


def _rel_err(a, ref):
    return max_abs(a, ref) / max(float(np.abs(ref).max()), 1e-6)


@pytest.mark.parametrize("d,n_layers,L,T", [
    (256, 2, 40, 16), (256, 2, 23, 9), (512, 2, 70, 32), (1024, 2, 100, 64), (1024, 1, 150, 128),
    (512, 2, 300, 256), (256, 2, 600, 400), (4096, 1, 20, 16), (256, 2, 33, 12), (2048, 2, 64, 64),
    (256, 2, 90, 40), (512, 2, 210, 100), (1024, 1, 75, 70),   # narrow layers, tile counts that round up
])
def test_sru_mfma_kernel_fp32(d, n_layers, L, T):
    W, b, x, c0 = _sru_inputs(800 + d + T, n_layers, d, L, scale=2.0)
    _check_sru(W, b, x, c0, T, MFMA | STAGES)


@pytest.mark.parametrize("d,n_layers,L,T,k", [
    (256, 2, 40, 16, 2), (512, 2, 70, 32, 2), (1024, 2, 100, 64, 2), (256, 2, 50, 20, 3),
    (512, 1, 200, 128, 2), (256, 2, 300, 256, 2), (128, 2, 30, 4, 2), (256, 2, 10, 1, 2),
    (256, 2, 500, 400, 2), (256, 2, 70, 33, 4), (512, 3, 37, 100, 3), (1024, 2, 5, 16, 2),
])
def test_qrnn_mfma_kernel_fp32(d, n_layers, L, T, k):
    W, b, x, c0, xh0 = _qrnn_inputs(900 + d + T + k, n_layers, d, L, k, scale=2.0)
    _check_qrnn(W, b, x, c0, xh0, T, k, MFMA | STAGES)


@pytest.mark.parametrize("cell,d,n_layers,L,T,k", [
    ("qrnn", 256, 2, 40, 16, 2), ("qrnn", 1024, 3, 100, 64, 2), ("qrnn", 512, 2, 300, 256, 2),
    ("sru", 512, 2, 70, 32, 1), ("qrnn", 256, 2, 30, 4, 2), ("sru", 1024, 2, 150, 128, 1),
    ("qrnn", 512, 2, 45, 17, 3), ("qrnn", 512, 2, 600, 400, 2),
])
def test_mfma_kernel_bf16_weights(cell, d, n_layers, L, T, k):
    """bf16 weights, inputs rounded to bf16 inside the kernel, fp32 accumulation
    and state: tensor-level relative error against the oracle (which reads the
    same bf16 weights but keeps activations exact)."""
    print(f"bf16 {cell} d={d} layers={n_layers} L={L} T={T} k={k}", flush=True)
    if cell == "sru":
        W, b, x, c0 = _sru_inputs(1000 + d + T, n_layers, d, L, bf16=True)
        h_ref, c_ref = oracle.sru_forward(W, b, x, c_init=c0, T=T)
        h, c = gpu_sru(W, b, x, c0, T=T, flags=MFMA)
    else:
        W, b, x, c0, xh0 = _qrnn_inputs(1000 + d + T + k, n_layers, d, L, k, bf16=True)
        h_ref, c_ref, _ = oracle.qrnn_forward(W, b, x, c_init=c0, xhist_init=xh0, T=T, k=k)
        h, c, _ = gpu_qrnn(W, b, x, c0, xh0, T=T, k=k, flags=MFMA)
    assert np.all(np.isfinite(h))
    assert _rel_err(h, h_ref) <= BF16_TOL, _rel_err(h, h_ref)
    assert _rel_err(c, c_ref) <= BF16_TOL, _rel_err(c, c_ref)
    _check_against_rounding_oracle(cell, W, b, x, c0, xh0 if cell == "qrnn" else None, T, k, h, c)


BF16_MATCHED_TOL = 1e-3


def _check_against_rounding_oracle(cell, W, b, x, c0, xh0, T, k, h, c):
    """The same GPU result against the oracle run that rounds the matrix operand
    X to bfloat16 as the kernel does: what is left is fp32 accumulation order,
    the fast exp/rcp, and the rare input that rounds to the neighbouring
    bfloat16 because the two sides' fp32 activations differ in the last place
    (each such flip moves a pre-activation by about |w||x| 2^-8, a few 1e-5)."""
    if cell == "sru":
        h_ref, c_ref = oracle.sru_forward(W, b, x, c_init=c0, T=T, round_operand=True)
    else:
        h_ref, c_ref, _ = oracle.qrnn_forward(W, b, x, c_init=c0, xhist_init=xh0, T=T, k=k, round_operand=True)
    assert _rel_err(h, h_ref) <= BF16_MATCHED_TOL, _rel_err(h, h_ref)
    assert _rel_err(c, c_ref) <= BF16_MATCHED_TOL, _rel_err(c, c_ref)


@pytest.mark.parametrize("T,packed", [(2, False), (24, False), (24, True)])
def test_forward_can_be_recorded_into_a_graph(T, packed):
    """*_forward only enqueues kernels on the given stream (no memset, no host
    synchronisation, no allocation), so a call can be captured into a HIP graph:
    every replay, with new inputs and with eager work in between, gives the eager
    result bit for bit."""
    import torch
    import paper_1803_11389_amd as ss
    d, n_layers, L, k = 512, 3, 61, 2
    W, b, x0, c0, xh0 = _qrnn_inputs(1500 + T, n_layers, d, L, k, scale=2.0)
    Wd = [to_dev(w) for w in W]
    flags = 0
    if packed:
        Wd = [ss.pack_weights(w) for w in Wd]
        flags = ss.WEIGHTS_PACKED
    bd = [to_dev(v) for v in b]
    x, c_in, xh_in = to_dev(x0), to_dev(c0), to_dev(xh0)
    ws = ss.Workspace.for_shape(n_layers, d, k, T, ss.F32)
    h = torch.empty((L, d), dtype=torch.float32, device="cuda")
    c = torch.empty((n_layers, d), dtype=torch.float32, device="cuda")
    xh = torch.empty((n_layers, k - 1, d), dtype=torch.float32, device="cuda")

    def call():
        ss.qrnn_forward(Wd, bd, x, c_in, xh_in, T=T, k=k, flags=flags, h=h, c_final=c, xhist_final=xh, workspace=ws)

    call()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            call()
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    for rep in range(3):
        x.copy_(to_dev(rng.standard_normal((L, d)).astype(np.float32)))
        c_in.copy_(to_dev(rng.standard_normal((n_layers, d)).astype(np.float32)))
        h.zero_(); c.zero_(); xh.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got = (h.clone(), c.clone(), xh.clone())
        call()                                   # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(got[0], h) and torch.equal(got[1], c) and torch.equal(got[2], xh), rep
    h_ref, c_ref, _ = oracle.qrnn_forward(W, b, x.cpu().numpy(), c_init=c_in.cpu().numpy(), xhist_init=xh0, T=T, k=k)
    assert max_abs(h.cpu().numpy(), h_ref) <= TOL and max_abs(c.cpu().numpy(), c_ref) <= TOL


def test_read_probe_runs_and_leaves_its_input_alone():
    import torch
    import paper_1803_11389_amd as ss
    buf = torch.arange(3 * 4096 + 4, dtype=torch.float32, device="cuda")      # 16-byte multiple, ragged for the waves
    keep = buf.clone()
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    ss.read_probe(buf, sink)
    ss.read_probe([buf, keep, buf], sink, groups=7)
    ss.read_probe(buf[:4], sink)
    torch.cuda.synchronize()
    assert torch.equal(buf, keep)


def test_kernels_agree_with_each_other():
    """Same inputs through the generic, vector-ALU and matrix-core kernels."""
    W, b, x, c0 = _sru_inputs(1101, 2, 512, 24, scale=2.0)
    outs = [gpu_sru(W, b, x, c0, T=8, flags=f) for f in (GENERIC, VALU, MFMA)]
    for o in outs[1:]:
        assert max_abs(o[0], outs[0][0]) <= 2e-5 and max_abs(o[1], outs[0][1]) <= 2e-5
