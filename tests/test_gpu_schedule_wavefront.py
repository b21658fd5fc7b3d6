"""The wavefront schedule (independent (block, layer) stages share a launch)
against the per-stage schedule in streaming order: the same kernels do the same
arithmetic per stage, so the outputs, the final state and the final window
must be the same bits; plus oracle parity where the stack is deeper than one
launch holds and where blocks are shorter than the QRNN window."""
import numpy as np
import pytest

import oracle
from gpu_util import gpu_qrnn, gpu_sru, max_abs
from test_gpu_parity import BF16_TOL, TOL, _qrnn_inputs, _rel_err, _sru_inputs

pytestmark = pytest.mark.gpu

STAGES, WAVEFRONT = 1, 3
GENERIC, VALU, MFMA = 1 << 4, 2 << 4, 3 << 4


@pytest.mark.parametrize("cell,d,n_layers,L,T,k,bf16,packed,kernel", [
    ("sru", 256, 3, 37, 4, 1, False, False, 0), ("sru", 512, 5, 50, 1, 1, False, False, VALU),
    ("sru", 256, 4, 100, 16, 1, False, False, MFMA), ("sru", 1024, 3, 130, 64, 1, False, True, 0),
    ("qrnn", 256, 3, 41, 4, 2, False, False, 0), ("qrnn", 256, 4, 23, 2, 4, False, False, 0),
    ("qrnn", 256, 3, 9, 1, 3, False, False, VALU), ("qrnn", 512, 3, 90, 20, 3, False, False, MFMA),
    ("qrnn", 512, 4, 300, 100, 2, True, True, 0), ("sru", 100, 3, 19, 5, 1, False, False, 0),
    ("qrnn", 48, 4, 30, 3, 3, False, False, GENERIC), ("sru", 256, 2, 600, 256, 1, True, False, 0),
    ("qrnn", 128, 3, 50, 16, 2, False, False, MFMA),       # narrow layer: columns split over workgroups
])
def test_wavefront_equals_stage_by_stage_bitwise(cell, d, n_layers, L, T, k, bf16, packed, kernel):
    import paper_1803_11389_amd as ss
    print(f"wavefront {cell} d={d} layers={n_layers} L={L} T={T} k={k} bf16={bf16} packed={packed} kernel={kernel:#x}", flush=True)
    if cell == "sru":
        W, b, x, c0 = _sru_inputs(4000 + d + T, n_layers, d, L, scale=2.0, bf16=bf16)
        xh0 = None
        ref = oracle.sru_forward(W, b, x, c_init=c0, T=T)
        run = lambda flags: gpu_sru(W, b, x, c0, T=T, flags=flags | kernel, packed=packed)
    else:
        W, b, x, c0, xh0 = _qrnn_inputs(4000 + d + T + k, n_layers, d, L, k, scale=2.0, bf16=bf16)
        ref = oracle.qrnn_forward(W, b, x, c_init=c0, xhist_init=xh0, T=T, k=k)
        run = lambda flags: gpu_qrnn(W, b, x, c0, xh0, T=T, k=k, flags=flags | kernel, packed=packed)
    # Narrow layers: the library splits a stage's columns over fewer workgroups when a launch holds several
    # stages, which re-associates the fp32 sums.  With the split switched off both schedules add in the same
    # order and must give the same bits; the library's own choice is then checked against the oracle.
    ns = ss.OPT_NO_SPLIT
    a, w, auto = run(STAGES | ns), run(WAVEFRONT | ns), run(ns)
    for u, v, z in zip(a, w, auto):
        np.testing.assert_array_equal(u, v)
        np.testing.assert_array_equal(u, z)      # the default of a call with several blocks and layers is the wavefront
    for got in (w, run(0), run(STAGES)):
        for u, r in zip(got, ref):
            if bf16:
                assert _rel_err(u, r) <= BF16_TOL
            else:
                assert max_abs(u, r) <= TOL, max_abs(u, r)


@pytest.mark.parametrize("cell,k", [("sru", 1), ("qrnn", 3)])
def test_stacks_deeper_than_one_launch_holds(cell, k):
    """19 layers: a step of the wavefront is up to 19 stages wide and goes out as three launches."""
    n_layers, d, L, T = 19, 256, 45, 2
    print(f"deep stack {cell}", flush=True)
    if cell == "sru":
        W, b, x, c0 = _sru_inputs(4100, n_layers, d, L, scale=2.0)
        got = gpu_sru(W, b, x, c0, T=T)
        ref = oracle.sru_forward(W, b, x, c_init=c0, T=T)
    else:
        W, b, x, c0, xh0 = _qrnn_inputs(4101, n_layers, d, L, k, scale=2.0)
        got = gpu_qrnn(W, b, x, c0, xh0, T=T, k=k)
        ref = oracle.qrnn_forward(W, b, x, c_init=c0, xhist_init=xh0, T=T, k=k)
    for u, r in zip(got, ref):
        assert max_abs(u, r) <= TOL, max_abs(u, r)


def test_fewer_blocks_than_layers_and_single_block():
    W, b, x, c0, xh0 = _qrnn_inputs(4102, 6, 256, 7, 2, scale=2.0)
    for T in (4, 7, 16):          # two blocks, one block, one short block
        print(f"few blocks T={T}", flush=True)
        got = gpu_qrnn(W, b, x, c0, xh0, T=T, k=2, flags=WAVEFRONT)
        ref = oracle.qrnn_forward(W, b, x, c_init=c0, xhist_init=xh0, T=T, k=2)
        for u, r in zip(got, ref):
            assert max_abs(u, r) <= TOL, max_abs(u, r)


@pytest.mark.parametrize("cell,k,T,mode,d,n_layers", [
    ("sru", 1, 64, "bf16", 4096, 2), ("qrnn", 2, 32, "bf16", 4096, 2), ("qrnn", 2, 64, "fp8", 4096, 2), ("sru", 1, 32, "fp8", 4096, 2),
    ("qrnn", 3, 33, "bf16", 2048, 5), ("sru", 1, 20, "f32", 2048, 6), ("qrnn", 2, 48, "fp8", 2048, 4),
])
def test_two_feature_tiles_per_workgroup_give_the_same_bits(cell, k, T, mode, d, n_layers):
    """Packed weights, 17 <= T <= 64 and launches wide enough to fill the chip with d/32 workgroups per
    stage: the matrix-core kernel gives a workgroup 32 features (half the input-block traffic).  Per
    feature the arithmetic and its order are those of the one-tile kernel, so the bits must agree; the
    result is also held to the oracle.  Biases, initial state and a ragged last block included."""
    import workloads as wl
    import paper_1803_11389_amd as ss
    L = (2 if d >= 4096 else 5) * T + 3        # enough blocks in flight that d/32 workgroups per stage fill the chip
    print(f"two tiles {cell} k={k} T={T} {mode} d={d} layers={n_layers}", flush=True)
    rng = np.random.default_rng(4200 + T + k + d)
    ncol = k * d
    Wf = [(rng.uniform(-1, 1, (3 * d, ncol)) * 2.0 / np.sqrt(ncol)).astype(np.float32) for _ in range(n_layers)]
    W = [wl.quantize_fp8(w) for w in Wf] if mode == "fp8" else [wl.to_bf16_bits(w) for w in Wf] if mode == "bf16" else Wf if mode == "bf16" else Wf
    nb = 2 if cell == "sru" else 3
    b = [rng.uniform(-1, 1, nb * d).astype(np.float32) for _ in range(n_layers)]
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((n_layers, d)).astype(np.float32)
    xh0 = rng.standard_normal((n_layers, k - 1, d)).astype(np.float32) if k > 1 else None
    if cell == "sru":
        run = lambda flags=0: gpu_sru(W, b, x, c0, T=T, flags=flags, packed=True)
        ref = oracle.sru_forward(W, b, x, c_init=c0, T=T)
    else:
        run = lambda flags=0: gpu_qrnn(W, b, x, c0, xh0, T=T, k=k, flags=flags, packed=True)
        ref = oracle.qrnn_forward(W, b, x, c_init=c0, xhist_init=xh0, T=T, k=k)
    two = run()
    one = run(ss.OPT_ONE_TILE)
    for u, v in zip(two, one):
        np.testing.assert_array_equal(u, v)
    for u, r in zip(two, ref):
        if np.asarray(r).size:
            if mode == "f32":
                assert max_abs(u, r) <= TOL, max_abs(u, r)
            else:
                assert _rel_err(u, r) <= BF16_TOL, _rel_err(u, r)


@pytest.mark.parametrize("cell,k,T,d,n_layers,nblocks,mode", [
    ("sru", 1, 100, 4096, 4, 4, "bf16"), ("qrnn", 2, 70, 2048, 8, 8, "bf16"), ("sru", 1, 256, 4096, 4, 4, "bf16"),
    ("qrnn", 3, 130, 2048, 8, 9, "bf16"),
    ("sru", 1, 24, 4096, 4, 6, "fp8"), ("qrnn", 2, 70, 2048, 8, 8, "fp8"), ("sru", 1, 256, 4096, 4, 4, "fp8"),
    ("qrnn", 3, 130, 2048, 8, 9, "fp8"), ("qrnn", 2, 50, 4096, 4, 5, "fp8"),
    # narrow weight types reach this kernel with shorter blocks as well (8-bit from 5 steps, bf16 from 9)
    ("sru", 1, 12, 4096, 4, 6, "fp8"), ("qrnn", 2, 7, 4096, 4, 7, "fp8"), ("qrnn", 2, 16, 2048, 8, 9, "bf16"),
    ("sru", 1, 9, 4096, 4, 5, "bf16"),
    # fp32 weights: blocks of 9 to 32 steps
    ("sru", 1, 12, 4096, 4, 6, "f32"), ("qrnn", 2, 30, 2048, 8, 9, "f32"), ("sru", 1, 16, 4096, 4, 5, "f32"),
])
def test_packed_weights_on_the_64_feature_kernel(cell, k, T, d, n_layers, nblocks, mode):
    """Packed weights of any type, blocks of up to 256 steps and launches wide enough for d/64 workgroups per stage to
    fill the chip: the kernel whose waves own a feature tile each and share the input block through LDS.
    Against the oracle (bf16 bar), against the oracle that rounds the same operand, and against the 16-feature
    kernel on the same inputs (the two sum a row's products in different orders, so not bit for bit)."""
    import workloads as wl
    import paper_1803_11389_amd as ss
    from test_gpu_parity import _check_against_rounding_oracle
    L = (nblocks - 1) * T + max(1, T // 3)           # a ragged last block
    print(f"64-feature kernel {cell} k={k} T={T} d={d} layers={n_layers} L={L} {mode}", flush=True)
    rng = np.random.default_rng(4300 + T + k + d)
    ncol = k * d
    Wf = [(rng.uniform(-1, 1, (3 * d, ncol)) * 2.0 / np.sqrt(ncol)).astype(np.float32) for _ in range(n_layers)]
    W = [wl.quantize_fp8(w) for w in Wf] if mode == "fp8" else [wl.to_bf16_bits(w) for w in Wf] if mode == "bf16" else Wf
    nb = 2 if cell == "sru" else 3
    b = [rng.uniform(-1, 1, nb * d).astype(np.float32) for _ in range(n_layers)]
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((n_layers, d)).astype(np.float32)
    xh0 = rng.standard_normal((n_layers, k - 1, d)).astype(np.float32) if k > 1 else None
    if cell == "sru":
        run = lambda flags=0: gpu_sru(W, b, x, c0, T=T, flags=flags, packed=True)
        ref = oracle.sru_forward(W, b, x, c_init=c0, T=T)
    else:
        run = lambda flags=0: gpu_qrnn(W, b, x, c0, xh0, T=T, k=k, flags=flags, packed=True)
        ref = oracle.qrnn_forward(W, b, x, c_init=c0, xhist_init=xh0, T=T, k=k)
    wide = run()
    narrow = run(ss.OPT_ONE_TILE)
    for u, v, r in zip(wide, narrow, ref):
        if np.asarray(r).size:
            assert np.all(np.isfinite(u))
            if mode == "f32":                         # fp32 weights: the fp32 bar, and fp32 re-association between the kernels
                assert max_abs(u, r) <= TOL, max_abs(u, r)
                assert max_abs(u, v) <= 5e-5, max_abs(u, v)
            else:
                assert _rel_err(u, r) <= BF16_TOL, _rel_err(u, r)
                assert _rel_err(u, v) <= 1e-3, _rel_err(u, v)
    assert not all(np.array_equal(u, v) for u, v in zip(wide, narrow)), "the 64-feature kernel was not taken"
    if mode != "f32":
        _check_against_rounding_oracle(cell, W, b, x, c0, xh0, T, k, wide[0], wide[1])
