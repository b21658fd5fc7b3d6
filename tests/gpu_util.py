"""Helpers for the GPU parity tests: move numpy inputs to the device, call the
library through its Python binding (a thin ctypes layer over the C ABI), bring
results back."""
import numpy as np


def to_dev(a):
    import torch
    if a is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def weight_to_dev(w):
    """A weight matrix on the device: float32 / uint16 arrays as they are, 8-bit
    weights (codes + row scales) as the library's single buffer."""
    import paper_1803_11389_amd as ss
    if hasattr(w, "blob"):
        rows, cols = w.q.shape
        d = rows // 3
        return ss.Fp8Weights(to_dev(w.blob()), d, cols // d)
    return to_dev(w)


def _weights(W, packed):
    """Device copies of the weight matrices; packed: re-tiled by ssrnn_pack_weights."""
    import paper_1803_11389_amd as ss
    Wd = [weight_to_dev(w) for w in W]
    return [ss.pack_weights(w) for w in Wd] if packed else Wd


def gpu_sru(W, bias, x, c_init=None, T=1, flags=0, packed=False):
    import torch
    import paper_1803_11389_amd as ss
    Wd = _weights(W, packed)
    flags |= ss.WEIGHTS_PACKED if packed else 0
    bd = None if bias is None else [to_dev(b) for b in bias]
    h, c = ss.sru_forward(Wd, bd, to_dev(np.asarray(x, np.float32)), to_dev(None if c_init is None else np.asarray(c_init, np.float32)),
                          T=T, flags=flags)
    torch.cuda.synchronize()
    return h.cpu().numpy(), c.cpu().numpy()


def gpu_qrnn(W, bias, x, c_init=None, xhist_init=None, T=1, k=2, flags=0, packed=False):
    import torch
    import paper_1803_11389_amd as ss
    Wd = _weights(W, packed)
    flags |= ss.WEIGHTS_PACKED if packed else 0
    bd = None if bias is None else [to_dev(b) for b in bias]
    h, c, xh = ss.qrnn_forward(Wd, bd, to_dev(np.asarray(x, np.float32)),
                               to_dev(None if c_init is None else np.asarray(c_init, np.float32)),
                               to_dev(None if xhist_init is None else np.asarray(xhist_init, np.float32)),
                               T=T, k=k, flags=flags)
    torch.cuda.synchronize()
    return h.cpu().numpy(), c.cpu().numpy(), xh.cpu().numpy()


def max_abs(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return float(np.max(np.abs(a - b))) if a.size else 0.0


def gpu_lstm(W, U, bias, x, h_init=None, c_init=None, T=1):
    import torch
    import paper_1803_11389_amd as ss
    f32 = lambda a: None if a is None else to_dev(np.asarray(a, np.float32))
    bd = None if bias is None else [f32(b) for b in bias]
    h, hf, cf = ss.lstm_forward([f32(w) for w in W], [f32(u) for u in U], bd, f32(x), f32(h_init), f32(c_init), T=T)
    torch.cuda.synchronize()
    return h.cpu().numpy(), hf.cpu().numpy(), cf.cpu().numpy()
