"""GPU tests of the weight pre-pack (ssrnn_pack_weights) and of the matrix-core
kernel that reads packed weights: the pack is a pure permutation (checked byte
for byte against the layout include/ssrnn.h and the kernel header state), and
the forward results meet the same bars against the CPU oracle as the row-major
path."""
import numpy as np
import pytest

import oracle
from gpu_util import gpu_qrnn, gpu_sru, max_abs, to_dev
from test_gpu_parity import BF16_TOL, TOL, _check_against_rounding_oracle, _qrnn_inputs, _rel_err, _sru_inputs

pytestmark = pytest.mark.gpu

MFMA = 3 << 4


def packed_layout(W):
    """The documented layout, written out with numpy: 16-byte chunk
    (((ft*nks + s)*3 + gate)*2 + half)*64 + lane holds bytes
    [s*128 + (lane//16)*32 + half*16, +16) of row gate*d + ft*16 + lane%16."""
    rows, _ = W.shape
    d = rows // 3
    raw = np.ascontiguousarray(W).view(np.uint8).reshape(rows, -1)
    nks = raw.shape[1] // 128
    v = raw.reshape(3, d // 16, 16, nks, 4, 2, 16)        # gate, ft, li, s, kg, half, byte
    out = v.transpose(1, 3, 0, 5, 4, 2, 6)                # ft, s, gate, half, kg, li, byte  (lane = kg*16 + li)
    return np.ascontiguousarray(out).reshape(-1)


@pytest.mark.parametrize("d,k,bf16", [(16, 2, False), (64, 1, True), (256, 2, False), (1024, 1, True), (96, 3, False)])
def test_pack_is_the_documented_permutation(d, k, bf16):
    import paper_1803_11389_amd as ss
    rng = np.random.default_rng(d + k)
    if bf16:
        if (d * 2) % 128 != 0:
            pytest.skip("bf16 rows of this width are not whole k-steps")
        W = rng.integers(0, 65536, (3 * d, k * d), dtype=np.uint16)
    else:
        if (d * 4) % 128 != 0:
            assert ss.packed_weight_bytes(d, k, ss.F32) == 0
            with pytest.raises(ss.SsrnnError):
                ss.pack_weights(to_dev(rng.standard_normal((3 * d, k * d)).astype(np.float32)))
            return
        W = rng.standard_normal((3 * d, k * d)).astype(np.float32)
    assert ss.packed_weight_bytes(d, k, ss.BF16 if bf16 else ss.F32) == W.nbytes
    got = ss.pack_weights(to_dev(W)).cpu().numpy().view(np.uint8).reshape(-1)
    np.testing.assert_array_equal(got, packed_layout(W))


@pytest.mark.parametrize("d,n_layers,L,T", [
    (256, 2, 40, 16), (256, 2, 23, 9), (512, 2, 70, 32), (1024, 2, 100, 64), (1024, 1, 150, 128),
    (512, 2, 300, 256), (256, 2, 600, 400), (4096, 1, 20, 16), (2048, 2, 64, 64), (4096, 2, 12, 4),
    (1024, 2, 9, 1), (4096, 1, 130, 128), (256, 2, 90, 40), (512, 2, 210, 100), (1024, 1, 75, 70),
])
def test_sru_packed_fp32(d, n_layers, L, T):
    print(f"packed sru d={d} layers={n_layers} L={L} T={T}", flush=True)
    W, b, x, c0 = _sru_inputs(1800 + d + T, n_layers, d, L, scale=2.0)
    h_ref, c_ref = oracle.sru_forward(W, b, x, c_init=c0, T=T)
    h, c = gpu_sru(W, b, x, c0, T=T, packed=True)
    assert max_abs(h, h_ref) <= TOL, max_abs(h, h_ref)
    assert max_abs(c, c_ref) <= TOL, max_abs(c, c_ref)


@pytest.mark.parametrize("d,n_layers,L,T,k", [
    (256, 2, 40, 16, 2), (512, 2, 70, 32, 2), (1024, 2, 100, 64, 2), (256, 2, 50, 20, 3),
    (512, 1, 200, 128, 2), (256, 2, 300, 256, 2), (128, 2, 30, 4, 2), (256, 2, 10, 1, 2), (4096, 1, 40, 32, 2),
    (256, 2, 500, 400, 2), (256, 2, 70, 33, 4), (512, 3, 37, 100, 3), (1024, 2, 5, 16, 2),
])
def test_qrnn_packed_fp32(d, n_layers, L, T, k):
    print(f"packed qrnn d={d} layers={n_layers} L={L} T={T} k={k}", flush=True)
    W, b, x, c0, xh0 = _qrnn_inputs(1900 + d + T + k, n_layers, d, L, k, scale=2.0)
    h_ref, c_ref, xh_ref = oracle.qrnn_forward(W, b, x, c_init=c0, xhist_init=xh0, T=T, k=k)
    h, c, xh = gpu_qrnn(W, b, x, c0, xh0, T=T, k=k, packed=True)
    assert max_abs(h, h_ref) <= TOL, max_abs(h, h_ref)
    assert max_abs(c, c_ref) <= TOL, max_abs(c, c_ref)
    assert max_abs(xh, xh_ref) <= TOL


@pytest.mark.parametrize("cell,d,n_layers,L,T,k", [
    ("qrnn", 256, 2, 40, 16, 2), ("qrnn", 1024, 3, 100, 64, 2), ("qrnn", 512, 2, 300, 256, 2),
    ("sru", 512, 2, 70, 32, 1), ("qrnn", 256, 2, 30, 4, 2), ("sru", 1024, 2, 150, 128, 1),
    ("qrnn", 4096, 1, 260, 256, 2), ("qrnn", 512, 2, 45, 17, 3), ("qrnn", 512, 2, 600, 400, 2),
])
def test_packed_bf16(cell, d, n_layers, L, T, k):
    print(f"packed bf16 {cell} d={d} layers={n_layers} L={L} T={T} k={k}", flush=True)
    if cell == "sru":
        W, b, x, c0 = _sru_inputs(2000 + d + T, n_layers, d, L, bf16=True)
        h_ref, c_ref = oracle.sru_forward(W, b, x, c_init=c0, T=T)
        h, c = gpu_sru(W, b, x, c0, T=T, packed=True)
    else:
        W, b, x, c0, xh0 = _qrnn_inputs(2000 + d + T + k, n_layers, d, L, k, bf16=True)
        h_ref, c_ref, _ = oracle.qrnn_forward(W, b, x, c_init=c0, xhist_init=xh0, T=T, k=k)
        h, c, _ = gpu_qrnn(W, b, x, c0, xh0, T=T, k=k, packed=True)
    assert np.all(np.isfinite(h))
    assert _rel_err(h, h_ref) <= BF16_TOL, _rel_err(h, h_ref)
    assert _rel_err(c, c_ref) <= BF16_TOL, _rel_err(c, c_ref)
    _check_against_rounding_oracle(cell, W, b, x, c0, xh0 if cell == "qrnn" else None, T, k, h, c)


def test_packed_flag_is_refused_where_no_matrix_core_kernel_applies():
    import paper_1803_11389_amd as ss
    W, b, x, c0 = _sru_inputs(5, 1, 256, 8)
    Wd = [ss.pack_weights(to_dev(w)) for w in W]
    with pytest.raises(ss.SsrnnError):      # packed weights cannot go through the vector-ALU kernel
        ss.sru_forward(Wd, None, to_dev(x), None, T=4, flags=ss.WEIGHTS_PACKED | ss.KERNEL_VALU)
    with pytest.raises(ss.SsrnnError):
        ss.sru_forward(Wd, None, to_dev(x), None, T=4, flags=ss.WEIGHTS_PACKED | ss.KERNEL_GENERIC)
