"""GPU parity on the benchmark configurations C2-C5 at their real widths and
depths.  The oracle needs seconds per hundred steps at d = 4096, so the wide
configurations are compared on a prefix of the sequence (the method is causal:
the first n outputs do not depend on later inputs), every block size of the
configuration's sweep against one oracle run (the oracle's result does not
depend on T).  C2 and C3 run their full length."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import max_abs, to_dev

pytestmark = pytest.mark.gpu


def _gpu_run(cfg, W_dev, x_dev, T, L):
    import torch
    import paper_1803_11389_amd as ss
    if cfg.cell == "sru":
        h, c = ss.sru_forward(W_dev, None, x_dev[:L].contiguous(), None, T=T)
    else:
        h, c, _ = ss.qrnn_forward(W_dev, None, x_dev[:L].contiguous(), None, None, T=T, k=cfg.k)
    torch.cuda.synchronize()
    return h.cpu().numpy(), c.cpu().numpy()


def _run_config(cfg, L, tol, relative):
    import paper_1803_11389_amd as ss
    inp = wl.make_inputs(cfg, L=L)
    W_dev = [to_dev(w) for w in inp["W"]]
    if cfg.d_feat:
        x_ref = oracle.linear_forward(inp["P"], inp["feat"])
        x_dev = ss.linear_forward(to_dev(inp["P"]), to_dev(inp["feat"]))
        assert max_abs(x_dev.cpu().numpy(), x_ref) <= 1e-5
    else:
        x_ref = inp["x"]
        x_dev = to_dev(inp["x"])
    if cfg.cell == "sru":
        h_ref, c_ref = oracle.sru_forward(inp["W"], None, x_ref, T=64)
    else:
        h_ref, c_ref, _ = oracle.qrnn_forward(inp["W"], None, x_ref, T=64, k=cfg.k)
    scale_h = max(float(np.abs(h_ref).max()), 1e-6) if relative else 1.0
    scale_c = max(float(np.abs(c_ref).max()), 1e-6) if relative else 1.0
    for T in cfg.Ts:
        h, c = _gpu_run(cfg, W_dev, x_dev, T, L)
        eh, ec = max_abs(h, h_ref) / scale_h, max_abs(c, c_ref) / scale_c
        print(f"{cfg.name} L={L} T={T}: err h {eh:.3e} c {ec:.3e}", flush=True)
        assert np.all(np.isfinite(h))
        assert eh <= tol and ec <= tol, (T, eh, ec)


def test_config2_sru4_d1024_asr_full_length():
    _run_config(wl.CONFIGS[1], wl.CONFIGS[1].L, 1e-4, False)


def test_config3_qrnn4_d1024_full_length():
    _run_config(wl.CONFIGS[2], wl.CONFIGS[2].L, 1e-4, False)


def test_config4_sru8_d4096_prefix():
    # 160 steps: full blocks for T <= 32, a ragged tail for T = 64 and 128
    _run_config(wl.CONFIGS[3], 160, 1e-4, False)


def test_config5_qrnn8_d4096_bf16_prefix():
    # 272 = 256 + 16: one full and one short block at T = 256
    _run_config(wl.CONFIGS[4], 272, 2e-2, True)
