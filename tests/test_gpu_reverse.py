"""SSRNN_REVERSE on the GPU: every layer walks the sequence from its last step
to its first (the second direction of a bidirectional network, Section 2.1 of
the paper).  Against the oracle's reverse pass element by element (fp32 bar 1e-4,
bf16 weights 2e-2 of the tensor scale), and bit for bit against the GPU's own
forward pass over the time-reversed sequence, which runs the same kernels on the
same operands in the same order."""
import numpy as np
import pytest

import oracle
from gpu_util import gpu_qrnn, gpu_sru, max_abs
from test_gpu_parity import BF16_TOL, TOL, _qrnn_inputs, _rel_err, _sru_inputs

pytestmark = pytest.mark.gpu

STAGES, WAVEFRONT = 1, 3
GENERIC, VALU, MFMA = 1 << 4, 2 << 4, 3 << 4
REVERSE = 1 << 11


@pytest.mark.parametrize("cell,d,n_layers,L,T,k,bf16,packed,flags", [
    ("sru", 256, 1, 37, 4, 1, False, False, 0),            # one layer, vector ALU, input and output read in place against time
    ("sru", 512, 3, 50, 1, 1, False, False, STAGES),
    ("sru", 256, 4, 100, 16, 1, False, False, MFMA),       # matrix cores: layer 0 is staged
    ("sru", 1024, 3, 130, 64, 1, False, True, 0),
    ("sru", 100, 2, 19, 5, 1, False, False, 0),            # generic kernel
    ("qrnn", 256, 3, 41, 4, 2, False, False, 0),
    ("qrnn", 256, 2, 23, 2, 4, False, False, STAGES),      # window longer than the block
    ("qrnn", 512, 3, 90, 20, 3, False, False, MFMA),
    ("qrnn", 512, 4, 300, 100, 2, True, True, 0),
    ("qrnn", 48, 2, 30, 3, 3, False, False, GENERIC),
    ("qrnn", 2048, 8, 600, 70, 2, True, True, 0),          # 64-features-per-workgroup kernel in the wide launches
    ("sru", 256, 2, 7, 16, 1, False, False, 0),            # one block longer than the sequence
])
def test_reverse_against_oracle_and_against_forward_on_the_reversed_sequence(cell, d, n_layers, L, T, k, bf16, packed, flags):
    print(f"reverse {cell} d={d} layers={n_layers} L={L} T={T} k={k} bf16={bf16} packed={packed} flags={flags:#x}", flush=True)
    if cell == "sru":
        W, b, x, c0 = _sru_inputs(5000 + d + T, n_layers, d, L, scale=2.0, bf16=bf16)
        ref = oracle.sru_forward(W, b, x, c_init=c0, T=T, reverse=True)
        rev = gpu_sru(W, b, x, c0, T=T, flags=flags | REVERSE, packed=packed)
        fwd = gpu_sru(W, b, x[::-1].copy(), c0, T=T, flags=flags, packed=packed)
    else:
        W, b, x, c0, xh0 = _qrnn_inputs(5000 + d + T + k, n_layers, d, L, k, scale=2.0, bf16=bf16)
        ref = oracle.qrnn_forward(W, b, x, c_init=c0, xhist_init=xh0, T=T, k=k, reverse=True)
        rev = gpu_qrnn(W, b, x, c0, xh0, T=T, k=k, flags=flags | REVERSE, packed=packed)
        fwd = gpu_qrnn(W, b, x[::-1].copy(), c0, xh0, T=T, k=k, flags=flags, packed=packed)
    for got, want in zip(rev, ref):
        if np.asarray(want).size:
            assert np.all(np.isfinite(got))
            if bf16:
                assert _rel_err(got, want) <= BF16_TOL, _rel_err(got, want)
            else:
                assert max_abs(got, want) <= TOL, max_abs(got, want)
    np.testing.assert_array_equal(rev[0], fwd[0][::-1])
    for a, f in zip(rev[1:], fwd[1:]):
        np.testing.assert_array_equal(a, f)
    if cell == "qrnn" and k > 1:
        # layer 0's window after the walk: its inputs at times 0 .. k-2, exactly
        np.testing.assert_array_equal(rev[2][0], x[:k - 1])


def test_reverse_chunks_chain_from_the_end():
    """The last 13 steps first, then the remaining 28 with the carried state and window: the same as one call."""
    W, b, x, c0, xh0 = _qrnn_inputs(5100, 3, 256, 41, 3, scale=2.0)
    whole = gpu_qrnn(W, b, x, c0, xh0, T=4, k=3, flags=REVERSE)
    tail = gpu_qrnn(W, b, x[28:], c0, xh0, T=4, k=3, flags=REVERSE)
    head = gpu_qrnn(W, b, x[:28], tail[1], tail[2], T=4, k=3, flags=REVERSE)
    ref = oracle.qrnn_forward(W, b, x, c_init=c0, xhist_init=xh0, T=4, k=3, reverse=True)
    h = np.concatenate([head[0], tail[0]], 0)
    assert max_abs(h, ref[0]) <= TOL and max_abs(head[1], ref[1]) <= TOL and max_abs(head[2], ref[2]) <= TOL
    assert max_abs(h, whole[0]) <= 2e-6 and max_abs(head[1], whole[1]) <= 2e-6


def test_reverse_of_an_empty_sequence_returns_the_initial_state():
    W, b, x, c0 = _sru_inputs(5200, 2, 256, 0)
    h, c = gpu_sru(W, b, x, c0, T=4, flags=REVERSE)
    assert h.shape == (0, 256)
    np.testing.assert_array_equal(c, c0)
