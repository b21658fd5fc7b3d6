"""sru_forward_noalloc (the entry point for callers that cannot allocate device
memory) against sru_forward on a caller-owned workspace and against the oracle:
two calls in a row on the library's static scratch, the second on a smaller
input, then a shape the static scratch cannot hold."""
import numpy as np
import pytest

import oracle
from gpu_util import max_abs, to_dev

pytestmark = pytest.mark.gpu


def _case(seed, n_layers, d, L, T, flags):
    """Runs one shape through both entry points; returns nothing, asserts."""
    import torch
    import paper_1803_11389_amd as ss
    rng = np.random.default_rng(seed)
    W = [(rng.uniform(-1, 1, (3 * d, d)) / np.sqrt(d)).astype(np.float32) for _ in range(n_layers)]
    bias = [rng.uniform(-0.5, 0.5, 2 * d).astype(np.float32) for _ in range(n_layers)]
    x = rng.standard_normal((L, d)).astype(np.float32)
    c0 = rng.uniform(-1, 1, (n_layers, d)).astype(np.float32)
    Wd, bd, xd, cd = [to_dev(w) for w in W], [to_dev(b) for b in bias], to_dev(x), to_dev(c0)
    assert ss.workspace_bytes(n_layers, d, 1, min(T, L), ss.F32) <= ss.NOALLOC_SCRATCH_BYTES
    h_ws, c_ws = ss.sru_forward(Wd, bd, xd, cd, T=T, flags=flags)
    h_na = torch.full((L, d), float("nan"), dtype=torch.float32, device="cuda")
    c_na = torch.full((n_layers, d), float("nan"), dtype=torch.float32, device="cuda")
    ss.sru_forward_noalloc(Wd, bd, xd, cd, h_na, c_na, T=T, flags=flags)
    torch.cuda.synchronize()
    h_ref, c_ref = oracle.sru_forward(W, bias, x, c0, T=T)
    eh, ec = max_abs(h_na.cpu().numpy(), h_ref), max_abs(c_na.cpu().numpy(), c_ref)
    print(f"noalloc n_layers={n_layers} d={d} L={L} T={T} flags={flags}: vs oracle h {eh:.3e} c {ec:.3e}", flush=True)
    assert eh <= 1e-4 and ec <= 1e-4                       # fp32 bar against the oracle
    assert torch.equal(h_na, h_ws) and torch.equal(c_na, c_ws)   # same kernels, same operands: same bits


def test_two_calls_in_a_row_the_second_smaller_then_a_shape_too_large():
    import torch
    import paper_1803_11389_amd as ss
    # matrix-core kernel, columns of a narrow layer split over workgroups: hand-off buffers, operand
    # copies and the partial planes all live in the static scratch
    _case(11, 3, 1024, 150, 64, ss.SCHED_STAGES)
    # smaller input right behind it: vector-ALU kernel, wavefront schedule, ragged last block
    _case(12, 2, 512, 37, 4, 0)
    # and the first shape again, now in the default schedule, on whatever the second call left behind
    _case(13, 3, 1024, 150, 64, 0)
    # a shape beyond the static array is refused on the host, nothing queued
    d, n_layers, T = 4096, 8, 128
    assert ss.workspace_bytes(n_layers, d, 1, T, ss.F32) > ss.NOALLOC_SCRATCH_BYTES
    lib = ss.load_library()
    import ctypes
    fake = ctypes.c_void_p(0x1000)
    tab = (ctypes.c_void_p * n_layers)(*([0x1000] * n_layers))
    rc = lib.sru_forward_noalloc(tab, None, fake, None, fake, fake, n_layers, d, 4096, T, ss.F32, 0, None)
    assert rc == 3 and b"static array" in lib.ssrnn_last_error()
    torch.cuda.synchronize()
