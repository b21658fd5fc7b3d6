"""Seeded sweep of shapes through the default kernel selection and, where the
width allows, through the packed-weight path: every case against the CPU
oracle, element by element.  The draw mixes widths that reach each kernel
(generic for odd widths, vector ALU, matrix cores with and without the split
over workgroups), windows k = 1..4, block sizes that are not multiples of the
16-step tile or that exceed the sequence, several blocks with a ragged tail,
biases and initial state."""
import math

import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import gpu_qrnn, gpu_sru, max_abs

pytestmark = pytest.mark.gpu

WIDTHS = [16, 48, 100, 128, 160, 256, 512, 768, 1024, 2048]
BLOCKS = [1, 2, 3, 5, 8, 13, 16, 17, 31, 32, 33, 47, 64, 65, 100, 128, 129, 200, 256, 300]


def _cases(n=160, seed=20241127):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        cell = "sru" if rng.random() < 0.45 else "qrnn"
        d = int(rng.choice(WIDTHS))
        k = 1 if cell == "sru" else int(rng.integers(1, 5))
        T = int(rng.choice(BLOCKS))
        n_layers = int(rng.integers(1, 4))
        # a few blocks and a tail, kept small enough for the oracle at the wide shapes
        L = int(min(rng.integers(1, 3 * T + 8), max(4, 30_000_000 // (3 * d * k * d // 64 + 1))))
        bf16 = bool(rng.random() < 0.3) and d % 64 == 0
        packed = bool(rng.random() < 0.5)
        out.append((i, cell, d, k, T, n_layers, L, bf16, packed))
    return out


def _fp8_cases(n=60, seed=20241128):
    """8-bit weights: widths the vector-ALU kernel takes (multiples of 1024), the packed matrix-core
    kernel takes (multiples of 128 with k*d a multiple of 512) and neither (generic kernel)."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        cell = "sru" if rng.random() < 0.5 else "qrnn"
        d = int(rng.choice([100, 128, 256, 512, 512, 1024, 1024, 1024, 2048, 2048]))
        k = 1 if cell == "sru" else int(rng.choice([1, 2, 2, 3, 4]))
        packed = bool(rng.random() < 0.6)
        T = int(rng.choice(BLOCKS if packed else BLOCKS[:7] + BLOCKS))     # row-major: more short blocks
        n_layers = int(rng.integers(1, 3))
        L = int(min(rng.integers(1, 3 * T + 8), max(4, 30_000_000 // (3 * d * k * d // 64 + 1))))
        out.append((i, cell, d, k, T, n_layers, L, packed))
    return out


def _packable(d, k, bf16):
    kstep = 64 if bf16 else 32
    return d % 16 == 0 and d % kstep == 0 and (k * d) % (4 * kstep) == 0


@pytest.mark.parametrize("case", _cases(), ids=lambda c: f"{c[0]}-{c[1]}-d{c[2]}-k{c[3]}-T{c[4]}-n{c[5]}-L{c[6]}{'-bf16' if c[7] else ''}{'-packed' if c[8] else ''}")
def test_random_shape_against_oracle(case):
    import paper_1803_11389_amd as ss
    i, cell, d, k, T, n_layers, L, bf16, packed = case
    print(f"case {case}", flush=True)
    rng = np.random.default_rng(9000 + i)
    ncol = k * d
    W = [(rng.uniform(-1, 1, (3 * d, ncol)) * 1.5 / math.sqrt(ncol)).astype(np.float32) for _ in range(n_layers)]
    if bf16:
        W = [wl.to_bf16_bits(w) for w in W]
    nb = 2 if cell == "sru" else 3
    bias = [rng.uniform(-1, 1, nb * d).astype(np.float32) if rng.random() < 0.7 else None for _ in range(n_layers)]
    if all(b is None for b in bias):
        bias = None
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((n_layers, d)).astype(np.float32) if rng.random() < 0.6 else None
    xh0 = rng.standard_normal((n_layers, k - 1, d)).astype(np.float32) if (k > 1 and rng.random() < 0.6) else None
    use_packed = packed and _packable(d, k, bf16)
    if cell == "sru":
        h_ref, c_ref = oracle.sru_forward(W, bias, x, c_init=c0, T=T)
        h, c = gpu_sru(W, bias, x, c0, T=T, packed=use_packed)
    else:
        h_ref, c_ref, xh_ref = oracle.qrnn_forward(W, bias, x, c_init=c0, xhist_init=xh0, T=T, k=k)
        h, c, xh = gpu_qrnn(W, bias, x, c0, xh0, T=T, k=k, packed=use_packed)
    assert np.all(np.isfinite(h)) and np.all(np.isfinite(c))
    if bf16:
        # bf16 weights: on the matrix-core path the input block is rounded to bf16 as well
        sh, sc = max(float(np.abs(h_ref).max()), 1e-6), max(float(np.abs(c_ref).max()), 1e-6)
        assert max_abs(h, h_ref) / sh <= 2e-2 and max_abs(c, c_ref) / sc <= 2e-2
    else:
        assert max_abs(h, h_ref) <= 1e-4, max_abs(h, h_ref)
        assert max_abs(c, c_ref) <= 1e-4, max_abs(c, c_ref)
        if cell == "qrnn" and k > 1:
            assert max_abs(xh, xh_ref) <= 1e-4


@pytest.mark.parametrize("case", _fp8_cases(), ids=lambda c: f"fp8-{c[0]}-{c[1]}-d{c[2]}-k{c[3]}-T{c[4]}-n{c[5]}-L{c[6]}{'-packed' if c[7] else ''}")
def test_random_shape_fp8_against_oracle(case):
    i, cell, d, k, T, n_layers, L, packed = case
    print(f"fp8 case {case}", flush=True)
    rng = np.random.default_rng(9500 + i)
    ncol = k * d
    W = [wl.quantize_fp8((rng.uniform(-1, 1, (3 * d, ncol)) * 1.5 / math.sqrt(ncol)).astype(np.float32) *
                         rng.uniform(0.5, 2.0, (3 * d, 1)).astype(np.float32)) for _ in range(n_layers)]
    nb = 2 if cell == "sru" else 3
    bias = [rng.uniform(-1, 1, nb * d).astype(np.float32) for _ in range(n_layers)] if rng.random() < 0.7 else None
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.standard_normal((n_layers, d)).astype(np.float32) if rng.random() < 0.6 else None
    xh0 = rng.standard_normal((n_layers, k - 1, d)).astype(np.float32) if (k > 1 and rng.random() < 0.6) else None
    # packed codes go to the matrix cores (whole k-steps of 128 codes per lag block, four waves' worth per row)
    use_packed = packed and d % 128 == 0 and (k * d) % 512 == 0
    if cell == "sru":
        h_ref, c_ref = oracle.sru_forward(W, bias, x, c_init=c0, T=T)
        h, c = gpu_sru(W, bias, x, c0, T=T, packed=use_packed)
    else:
        h_ref, c_ref, _ = oracle.qrnn_forward(W, bias, x, c_init=c0, xhist_init=xh0, T=T, k=k)
        h, c, _ = gpu_qrnn(W, bias, x, c0, xh0, T=T, k=k, packed=use_packed)
    assert np.all(np.isfinite(h)) and np.all(np.isfinite(c))
    if use_packed:
        sh, sc = max(float(np.abs(h_ref).max()), 1e-6), max(float(np.abs(c_ref).max()), 1e-6)
        assert max_abs(h, h_ref) / sh <= 2e-2 and max_abs(c, c_ref) / sc <= 2e-2
    else:
        assert max_abs(h, h_ref) <= 1e-4, max_abs(h, h_ref)
        assert max_abs(c, c_ref) <= 1e-4, max_abs(c, c_ref)
