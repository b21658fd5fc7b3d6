"""GPU tests of 8-bit float (E4M3) weights with row scales: every kernel that
takes them (vector ALU and generic on row-major codes, matrix cores on packed
codes) against the CPU oracle, which widens the same codes from the format's
definition.  The bars are those of the other weight types: where the input
block stays fp32 (vector ALU, generic) max |delta| <= 1e-4; on the matrix cores
the block is rounded to bf16, so 2e-2 of the tensor's largest magnitude against
the exact oracle and 1e-3 against the oracle that rounds the same operand."""
import math

import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import gpu_qrnn, gpu_sru, max_abs, to_dev, weight_to_dev
from test_gpu_parity import BF16_TOL, TOL, _check_against_rounding_oracle, _rel_err

pytestmark = pytest.mark.gpu

GENERIC, VALU, MFMA = 1 << 4, 2 << 4, 3 << 4


def _inputs(seed, cell, n_layers, d, L, k, scale=2.0, with_bias=True, with_state=True):
    rng = np.random.default_rng(seed)
    ncol = k * d
    W = [wl.quantize_fp8((rng.uniform(-1, 1, (3 * d, ncol)) * scale / math.sqrt(ncol)).astype(np.float32) *
                         rng.uniform(0.3, 3.0, (3 * d, 1)).astype(np.float32)) for _ in range(n_layers)]
    nb = 2 if cell == "sru" else 3
    b = [rng.uniform(-1, 1, nb * d).astype(np.float32) for _ in range(n_layers)] if with_bias else None
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((n_layers, d)).astype(np.float32) if with_state else None
    xh0 = rng.standard_normal((n_layers, k - 1, d)).astype(np.float32) if (with_state and k > 1) else None
    return W, b, x, c0, xh0


def _run(cell, W, b, x, c0, xh0, T, k, flags=0, packed=False):
    if cell == "sru":
        h_ref, c_ref = oracle.sru_forward(W, b, x, c_init=c0, T=T)
        h, c = gpu_sru(W, b, x, c0, T=T, flags=flags, packed=packed)
    else:
        h_ref, c_ref, _ = oracle.qrnn_forward(W, b, x, c_init=c0, xhist_init=xh0, T=T, k=k)
        h, c, _ = gpu_qrnn(W, b, x, c0, xh0, T=T, k=k, flags=flags, packed=packed)
    assert np.all(np.isfinite(h)) and np.all(np.isfinite(c))
    return h, c, h_ref, c_ref


def test_every_code_is_widened_as_the_format_defines():
    """Bit-exact check of the widening on all three kernels.  One SRU step from c = 0 with the forget
    and reset rows all zero codes (f = r = 1/2 exactly): c_1 = scale_i * (sum_j value(q_ij) x_j) / 2.
    Every candidate row has 16 non-zero codes, x is 1/2 or 1 and the scales are powers of two, so each
    product and every partial sum fits fp32 exactly whatever the order: the GPU's c must equal the
    oracle's bit for bit.  All 254 non-NaN codes occur, in all 16 byte positions of a 16-byte load."""
    rng = np.random.default_rng(77)
    d = 1024
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], np.uint8)
    q = np.zeros((3 * d, d), np.uint8)
    seen = set()
    for i in range(d):
        for j in range(16):
            pair = 16 * i + j                               # pairs 0 .. 4063 are every (code, byte position) once
            code, pos = codes[pair % 254], (pair // 254) % 16
            col = 64 * j + 16 * (i % 4) + pos
            q[i, col] = code
            seen.add((int(code), col % 16))
    assert len(seen) == 254 * 16
    scale = np.ones(3 * d, np.float32)
    scale[:d] = (2.0 ** rng.integers(-12, -5, d)).astype(np.float32)
    W = [wl.Fp8Weight(q, scale)]
    x = rng.choice(np.array([0.5, 1.0], np.float32), size=(1, d))
    h_ref, c_ref = oracle.sru_forward(W, None, x, T=1)
    assert np.array_equal(c_ref.astype(np.float32).astype(np.float64), c_ref)      # the reference itself is exact in fp32
    for flags, packed in ((VALU, False), (GENERIC, False), (MFMA, True)):
        print(f"codes: flags={flags:#x} packed={packed}", flush=True)
        h, c = gpu_sru(W, None, x, None, T=1, flags=flags, packed=packed)
        np.testing.assert_array_equal(c, c_ref.astype(np.float32))
        assert max_abs(h, h_ref) <= 2e-6, (flags, max_abs(h, h_ref))


@pytest.mark.parametrize("cell,d,n_layers,L,T,k", [
    ("sru", 1024, 2, 9, 1, 1), ("sru", 1024, 2, 11, 2, 1), ("sru", 2048, 2, 13, 4, 1), ("sru", 1024, 2, 20, 8, 1),
    ("sru", 4096, 1, 7, 3, 1), ("qrnn", 1024, 2, 9, 1, 2), ("qrnn", 1024, 2, 14, 4, 2), ("qrnn", 1024, 2, 19, 8, 3),
    ("qrnn", 2048, 1, 6, 2, 2), ("sru", 8192, 1, 3, 2, 1), ("qrnn", 4096, 1, 5, 2, 3),
])
def test_vector_alu_kernel_fp8(cell, d, n_layers, L, T, k):
    print(f"fp8 valu {cell} d={d} layers={n_layers} L={L} T={T} k={k}", flush=True)
    W, b, x, c0, xh0 = _inputs(3000 + d + T + k, cell, n_layers, d, L, k)
    h, c, h_ref, c_ref = _run(cell, W, b, x, c0, xh0, T, k, flags=VALU)
    assert max_abs(h, h_ref) <= TOL, max_abs(h, h_ref)
    assert max_abs(c, c_ref) <= TOL, max_abs(c, c_ref)


@pytest.mark.parametrize("cell,d,n_layers,L,T,k", [
    ("sru", 100, 2, 9, 4, 1), ("qrnn", 48, 2, 20, 16, 3), ("sru", 1024, 1, 12, 12, 1), ("qrnn", 130, 2, 7, 2, 2),
])
def test_generic_kernel_fp8(cell, d, n_layers, L, T, k):
    """Shapes whose code count is not a multiple of 256 put padding before the scales."""
    print(f"fp8 generic {cell} d={d} layers={n_layers} L={L} T={T} k={k}", flush=True)
    W, b, x, c0, xh0 = _inputs(3100 + d + T + k, cell, n_layers, d, L, k)
    h, c, h_ref, c_ref = _run(cell, W, b, x, c0, xh0, T, k, flags=GENERIC)
    assert max_abs(h, h_ref) <= TOL, max_abs(h, h_ref)
    assert max_abs(c, c_ref) <= TOL, max_abs(c, c_ref)


@pytest.mark.parametrize("cell,d,L,T,k", [("sru", 1024, 45, 20, 1), ("qrnn", 1024, 70, 64, 2), ("sru", 2048, 30, 9, 1)])
def test_row_major_fp8_long_blocks_are_cut_to_the_vector_alu_kernels_length(cell, d, L, T, k):
    """Row-major codes have no matrix-core kernel: a block longer than 8 steps is processed 8 steps per
    weight pass on the vector-ALU kernel (same results, fp32 bar) instead of falling to the generic kernel."""
    print(f"fp8 row-major long block {cell} d={d} L={L} T={T} k={k}", flush=True)
    W, b, x, c0, xh0 = _inputs(3300 + d + T + k, cell, 2, d, L, k)
    h, c, h_ref, c_ref = _run(cell, W, b, x, c0, xh0, T, k)
    assert max_abs(h, h_ref) <= TOL, max_abs(h, h_ref)
    assert max_abs(c, c_ref) <= TOL, max_abs(c, c_ref)


@pytest.mark.parametrize("cell,d,n_layers,L,T,k", [
    ("sru", 512, 2, 40, 16, 1), ("sru", 1024, 2, 9, 1, 1), ("sru", 1024, 2, 70, 32, 1), ("sru", 2048, 2, 100, 64, 1),
    ("sru", 1024, 1, 150, 128, 1), ("sru", 512, 2, 300, 256, 1), ("sru", 4096, 1, 20, 16, 1), ("sru", 4096, 2, 12, 4, 1),
    ("qrnn", 512, 2, 40, 16, 2), ("qrnn", 1024, 2, 100, 64, 2), ("qrnn", 512, 2, 45, 17, 3), ("qrnn", 512, 2, 300, 256, 2),
    ("qrnn", 4096, 1, 260, 256, 2), ("qrnn", 256, 2, 50, 33, 2), ("sru", 512, 2, 210, 100, 1), ("qrnn", 512, 2, 600, 400, 2),
    ("qrnn", 1024, 2, 37, 8, 4), ("sru", 8192, 1, 40, 40, 1),
])
def test_matrix_core_kernel_fp8_packed(cell, d, n_layers, L, T, k):
    print(f"fp8 packed {cell} d={d} layers={n_layers} L={L} T={T} k={k}", flush=True)
    W, b, x, c0, xh0 = _inputs(3200 + d + T + k, cell, n_layers, d, L, k)
    h, c, h_ref, c_ref = _run(cell, W, b, x, c0, xh0, T, k, packed=True)
    assert _rel_err(h, h_ref) <= BF16_TOL, _rel_err(h, h_ref)
    assert _rel_err(c, c_ref) <= BF16_TOL, _rel_err(c, c_ref)
    _check_against_rounding_oracle(cell, W, b, x, c0, xh0, T, k, h, c)


def test_pack_keeps_codes_and_scales():
    import paper_1803_11389_amd as ss
    from test_gpu_packed import packed_layout
    rng = np.random.default_rng(5)
    for d, k in ((128, 1), (256, 2), (384, 1)):
        w = wl.Fp8Weight(rng.integers(0, 256, (3 * d, k * d), dtype=np.uint8), rng.uniform(0.1, 1, 3 * d).astype(np.float32))
        assert ss.weight_bytes(d, k, ss.FP8) == w.blob().size == ss.packed_weight_bytes(d, k, ss.FP8)
        got = ss.pack_weights(weight_to_dev(w)).buf.cpu().numpy()
        n = 3 * d * k * d
        np.testing.assert_array_equal(got[:n], packed_layout(w.q))
        off = (n + 255) // 256 * 256
        np.testing.assert_array_equal(got[off:].view(np.float32), w.scale)


def test_fp8_shapes_no_kernel_takes_are_refused():
    import paper_1803_11389_amd as ss
    W, b, x, c0, _ = _inputs(9, "sru", 1, 256, 8, 1)
    Wd = [weight_to_dev(w) for w in W]
    with pytest.raises(ss.SsrnnError):          # row-major codes do not reach the matrix cores
        ss.sru_forward(Wd, None, to_dev(x), None, T=4, flags=MFMA)
    with pytest.raises(ss.SsrnnError):          # d % 1024 != 0
        ss.sru_forward(Wd, None, to_dev(x), None, T=4, flags=VALU)
    assert ss.packed_weight_bytes(192, 1, ss.FP8) == 0


def test_fp8_workload_prefix_through_default_selection():
    """The 8-bit d = 4096 workloads: a short prefix, row-major (T = 1, 2: vector ALU) and packed (T = 16)."""
    for name, T, L, packed in (("X2", 1, 3, False), ("X2", 2, 4, False), ("X2", 16, 32, True), ("X3", 16, 20, True)):
        cfg = wl.by_name(name)
        inp = wl.make_inputs(cfg, L=L, n_layers=2)
        print(f"{cfg.name} T={T} L={L} packed={packed}", flush=True)
        h, c, h_ref, c_ref = _run(cfg.cell, inp["W"], None, inp["x"], None, None, T, cfg.k, packed=packed)
        if packed:
            assert _rel_err(h, h_ref) <= BF16_TOL and _rel_err(c, c_ref) <= BF16_TOL
        else:
            assert max_abs(h, h_ref) <= TOL and max_abs(c, c_ref) <= TOL
