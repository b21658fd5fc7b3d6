"""Python binding of libssrnn (include/ssrnn.h): single-stream, multi-time-step
inference of stacked SRU / QRNN layers (arXiv 1803.11389) on one MI355X.

This module only marshals arguments: torch supplies device memory and the
current stream, every step of the computation runs in the HIP kernels of
libssrnn.so.  There is no CPU or PyTorch fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libssrnn.so")

F32, BF16, FP8 = 0, 1, 2
SCHED_AUTO, SCHED_STAGES, SCHED_WAVEFRONT = 0, 1, 3
KERNEL_AUTO, KERNEL_GENERIC, KERNEL_VALU, KERNEL_MFMA = 0, 1 << 4, 2 << 4, 3 << 4
WEIGHTS_PACKED = 1 << 8
OPT_NO_SPLIT, OPT_ONE_TILE = 1 << 9, 1 << 10
REVERSE = 1 << 11

# every symbol include/ssrnn.h declares, then those of include/ssrnn_probe.h (measurement aids)
EXPORTS = ("ssrnn_version", "ssrnn_last_error", "ssrnn_workspace_bytes", "sru_forward",
           "qrnn_forward", "ssrnn_linear_forward", "ssrnn_packed_weight_bytes", "ssrnn_pack_weights",
           "ssrnn_weight_bytes", "sru_forward_noalloc", "lstm_workspace_bytes", "lstm_forward")
PROBE_EXPORTS = ("ssrnn_read_probe",)
NOALLOC_SCRATCH_BYTES = 32 << 20   # SSRNN_NOALLOC_SCRATCH_BYTES of include/ssrnn.h

_lib = None


class SsrnnError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"ssrnn status {status}: {message}")
        self.status = status


def load_library():
    """dlopen libssrnn.so (built by paper_1803_11389_amd.build) and declare its
    signatures.  Raises if the library has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_1803_11389_amd.build` "
                          "(there is no fallback implementation)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, ip, lp, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_long, ctypes.c_size_t
    lib.ssrnn_version.restype = ip
    lib.ssrnn_last_error.restype = ctypes.c_char_p
    lib.ssrnn_workspace_bytes.restype = sz
    lib.ssrnn_workspace_bytes.argtypes = [ip] * 5
    lib.sru_forward.restype = ip
    lib.sru_forward.argtypes = [vp] * 6 + [ip, ip, lp, ip, ip, ip, vp, sz, vp]
    lib.sru_forward_noalloc.restype = ip
    lib.sru_forward_noalloc.argtypes = [vp] * 6 + [ip, ip, lp, ip, ip, ip, vp]
    lib.qrnn_forward.restype = ip
    lib.qrnn_forward.argtypes = [vp] * 8 + [ip, ip, lp, ip, ip, ip, ip, vp, sz, vp]
    lib.ssrnn_linear_forward.restype = ip
    lib.ssrnn_linear_forward.argtypes = [vp] * 3 + [ip, ip, lp, vp]
    lib.ssrnn_weight_bytes.restype = sz
    lib.ssrnn_weight_bytes.argtypes = [ip] * 3
    lib.ssrnn_packed_weight_bytes.restype = sz
    lib.ssrnn_packed_weight_bytes.argtypes = [ip] * 3
    lib.ssrnn_pack_weights.restype = ip
    lib.ssrnn_pack_weights.argtypes = [vp, vp, ip, ip, ip, vp]
    lib.lstm_workspace_bytes.restype = sz
    lib.lstm_workspace_bytes.argtypes = [ip] * 3
    lib.lstm_forward.restype = ip
    lib.lstm_forward.argtypes = [vp] * 9 + [ip, ip, lp, ip, ip, vp, sz, vp]
    lib.ssrnn_read_probe.restype = ip
    lib.ssrnn_read_probe.argtypes = [vp, ip, sz, ip, vp, vp]
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise SsrnnError(rc, load_library().ssrnn_last_error().decode())


def version() -> int:
    return load_library().ssrnn_version()


def workspace_bytes(n_layers: int, d: int, k: int, T: int, wdtype: int) -> int:
    return load_library().ssrnn_workspace_bytes(n_layers, d, k, T, wdtype)


def packed_weight_bytes(d: int, k: int, wdtype: int) -> int:
    return load_library().ssrnn_packed_weight_bytes(d, k, wdtype)


def weight_bytes(d: int, k: int, wdtype: int) -> int:
    return load_library().ssrnn_weight_bytes(d, k, wdtype)


class Fp8Weights:
    """One layer's SSRNN_FP8 weight buffer on the device (codes, padding, row
    scales: the layout ssrnn_weight_bytes documents) with its logical shape."""

    def __init__(self, buf, d: int, k: int):
        import torch
        if buf.dtype != torch.uint8 or buf.dim() != 1 or buf.numel() != weight_bytes(d, k, FP8):
            raise ValueError(f"an 8-bit weight buffer for d={d}, k={k} is {weight_bytes(d, k, FP8)} bytes of uint8")
        self.buf, self.d, self.k = buf, int(d), int(k)
        self.shape = (3 * self.d, self.k * self.d)
        self.is_cuda = buf.is_cuda

    def data_ptr(self):
        return self.buf.data_ptr()

    def is_contiguous(self):
        return self.buf.is_contiguous()

    def dim(self):
        return 2


def pack_weights(W, stream=None):
    """ssrnn_pack_weights: returns a new device tensor of W's shape and dtype
    that holds the [3d, k*d] matrix in the matrix-core kernel's order; pass it
    to *_forward with flags | WEIGHTS_PACKED."""
    import torch
    lib = load_library()
    _req(W, "W")
    d = W.shape[0] // 3
    if W.dim() != 2 or W.shape[0] != 3 * d or W.shape[1] % d != 0:
        raise ValueError("W must be [3d, k*d]")
    k = W.shape[1] // d
    wdt = _wdtype(W)
    out = Fp8Weights(torch.empty_like(W.buf), d, k) if wdt == FP8 else torch.empty_like(W)
    _check(lib.ssrnn_pack_weights(_p(W), _p(out), d, k, wdt, _stream_handle(stream)))
    return out


def read_probe(bufs, sink, groups: int = 0, stream=None) -> None:
    """ssrnn_read_probe (include/ssrnn_probe.h): one launch that reads up to eight
    equally long contiguous device tensors once; sink: a device tensor of at least 4 bytes."""
    bufs = list(bufs) if isinstance(bufs, (list, tuple)) else [bufs]
    for b in bufs:
        _req(b, "buf")
    _req(sink, "sink")
    nbytes = bufs[0].numel() * bufs[0].element_size()
    if any(b.numel() * b.element_size() != nbytes for b in bufs):
        raise ValueError("the buffers of one probe launch must be equally long")
    _check(load_library().ssrnn_read_probe(_ptr_table(bufs), len(bufs), nbytes, int(groups), _p(sink), _stream_handle(stream)))


def _wdtype(w) -> int:
    import torch
    if isinstance(w, Fp8Weights):
        return FP8
    if w.dtype == torch.float32:
        return F32
    if w.dtype in (torch.bfloat16, torch.uint16, torch.int16):
        return BF16
    raise TypeError(f"weights must be float32 or bfloat16 (or their 16-bit patterns), got {w.dtype}")


def _ptr_table(tensors: Optional[Sequence]):
    """Host array of device pointers (entries may be None)."""
    if tensors is None:
        return None
    t = (ctypes.c_void_p * len(tensors))()
    for i, a in enumerate(tensors):
        t[i] = None if a is None else a.data_ptr()
    return t


def _p(t):
    return None if t is None else t.data_ptr()


def _req(t, name, shape=None, dtype=None):
    import torch
    if t is None:
        return
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    if dtype is not None and (isinstance(t, Fp8Weights) or t.dtype != dtype):
        raise TypeError(f"{name} must be {dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")


class Workspace:
    """Device scratch for *_forward, reusable across calls of the same or a
    smaller shape."""

    def __init__(self, nbytes: int, device="cuda"):
        import torch
        self.nbytes = int(nbytes)
        self.buf = torch.empty(max(self.nbytes, 256), dtype=torch.uint8, device=device)
        assert self.buf.data_ptr() % 256 == 0

    @classmethod
    def for_shape(cls, n_layers, d, k, T, wdtype, device="cuda"):
        return cls(workspace_bytes(n_layers, d, k, T, wdtype), device)


def _stream_handle(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def sru_forward(W: List, bias: Optional[List], x, c_init=None, *, T: int, flags: int = 0,
                h=None, c_final=None, workspace: Optional[Workspace] = None, stream=None):
    """sru_forward of include/ssrnn.h.  W: list of [3d, d] device tensors; bias:
    None or list of None / [2d]; x: [L, d] fp32.  Returns (h, c_final)."""
    import torch
    lib = load_library()
    n_layers = len(W)
    d = W[0].shape[1]
    wdt = _wdtype(W[0])
    for w in W:
        _req(w, "W[l]", (3 * d, d))
    _req(x, "x", None, torch.float32)
    L = x.shape[0]
    if x.dim() != 2 or x.shape[1] != d:
        raise ValueError("x must be [L, d]")
    _req(c_init, "c_init", (n_layers, d), torch.float32)
    if bias is not None:
        for b in bias:
            _req(b, "bias[l]", (2 * d,), torch.float32)
    if h is None:
        h = torch.empty((L, d), dtype=torch.float32, device=x.device)
    if c_final is None:
        c_final = torch.empty((n_layers, d), dtype=torch.float32, device=x.device)
    _req(h, "h", (L, d), torch.float32)
    _req(c_final, "c_final", (n_layers, d), torch.float32)
    if workspace is None:
        workspace = Workspace.for_shape(n_layers, d, 1, T, wdt, x.device)
    wt, bt = _ptr_table(W), _ptr_table(bias)
    rc = lib.sru_forward(wt, bt, _p(x), _p(c_init), _p(h), _p(c_final), n_layers, d, L, int(T), wdt,
                         int(flags), workspace.buf.data_ptr(), workspace.nbytes, _stream_handle(stream))
    _check(rc)
    return h, c_final


def lstm_forward(W: List, U: List, bias: Optional[List], x, h_init=None, c_init=None, *, T: int, flags: int = 0,
                 h=None, h_final=None, c_final=None, workspace: Optional[Workspace] = None, stream=None):
    """lstm_forward of include/ssrnn.h (the paper's comparison network, Eq. 1).  W, U: lists of [4d, d] fp32
    device tensors; bias: None or list of None / [4d]; x: [L, d] fp32.  Returns (h, h_final, c_final)."""
    import torch
    lib = load_library()
    n_layers = len(W)
    if len(U) != n_layers:
        raise ValueError("W and U must have one matrix per layer each")
    d = W[0].shape[1]
    for w, u in zip(W, U):
        _req(w, "W[l]", (4 * d, d), torch.float32)
        _req(u, "U[l]", (4 * d, d), torch.float32)
    _req(x, "x", None, torch.float32)
    L = x.shape[0]
    if x.dim() != 2 or x.shape[1] != d:
        raise ValueError("x must be [L, d]")
    _req(h_init, "h_init", (n_layers, d), torch.float32)
    _req(c_init, "c_init", (n_layers, d), torch.float32)
    if bias is not None:
        for b in bias:
            _req(b, "bias[l]", (4 * d,), torch.float32)
    if h is None:
        h = torch.empty((L, d), dtype=torch.float32, device=x.device)
    if h_final is None:
        h_final = torch.empty((n_layers, d), dtype=torch.float32, device=x.device)
    if c_final is None:
        c_final = torch.empty((n_layers, d), dtype=torch.float32, device=x.device)
    _req(h, "h", (L, d), torch.float32)
    _req(h_final, "h_final", (n_layers, d), torch.float32)
    _req(c_final, "c_final", (n_layers, d), torch.float32)
    if workspace is None:
        workspace = Workspace(lib.lstm_workspace_bytes(n_layers, d, int(T)), x.device)
    wt, ut, bt = _ptr_table(W), _ptr_table(U), _ptr_table(bias)
    rc = lib.lstm_forward(wt, ut, bt, _p(x), _p(h_init), _p(c_init), _p(h), _p(h_final), _p(c_final), n_layers, d, L,
                          int(T), int(flags), workspace.buf.data_ptr(), workspace.nbytes, _stream_handle(stream))
    _check(rc)
    return h, h_final, c_final


def sru_forward_noalloc(W: List, bias: Optional[List], x, c_init, h, c_final, *, T: int, flags: int = 0, stream=None):
    """sru_forward_noalloc of include/ssrnn.h: sru_forward on the library's static
    device scratch.  Every buffer, outputs included, is the caller's; nothing is
    allocated here or in the library.  Returns (h, c_final)."""
    import torch
    lib = load_library()
    n_layers = len(W)
    d = W[0].shape[1]
    wdt = _wdtype(W[0])
    for w in W:
        _req(w, "W[l]", (3 * d, d))
    _req(x, "x", None, torch.float32)
    L = x.shape[0]
    if x.dim() != 2 or x.shape[1] != d:
        raise ValueError("x must be [L, d]")
    _req(c_init, "c_init", (n_layers, d), torch.float32)
    if bias is not None:
        for b in bias:
            _req(b, "bias[l]", (2 * d,), torch.float32)
    if h is None or c_final is None:
        raise ValueError("h and c_final must be given: this entry point allocates nothing")
    _req(h, "h", (L, d), torch.float32)
    _req(c_final, "c_final", (n_layers, d), torch.float32)
    wt, bt = _ptr_table(W), _ptr_table(bias)
    _check(lib.sru_forward_noalloc(wt, bt, _p(x), _p(c_init), _p(h), _p(c_final), n_layers, d, L, int(T), wdt,
                                   int(flags), _stream_handle(stream)))
    return h, c_final


def qrnn_forward(W: List, bias: Optional[List], x, c_init=None, xhist_init=None, *, T: int, k: int = 2,
                 flags: int = 0, h=None, c_final=None, xhist_final=None,
                 workspace: Optional[Workspace] = None, stream=None):
    """qrnn_forward of include/ssrnn.h.  W: list of [3d, k*d]; x: [L, d] fp32.
    Returns (h, c_final, xhist_final)."""
    import torch
    lib = load_library()
    n_layers = len(W)
    d = W[0].shape[0] // 3
    wdt = _wdtype(W[0])
    for w in W:
        _req(w, "W[l]", (3 * d, k * d))
    _req(x, "x", None, torch.float32)
    L = x.shape[0]
    if x.dim() != 2 or x.shape[1] != d:
        raise ValueError("x must be [L, d]")
    _req(c_init, "c_init", (n_layers, d), torch.float32)
    _req(xhist_init, "xhist_init", (n_layers, k - 1, d), torch.float32)
    if bias is not None:
        for b in bias:
            _req(b, "bias[l]", (3 * d,), torch.float32)
    if h is None:
        h = torch.empty((L, d), dtype=torch.float32, device=x.device)
    if c_final is None:
        c_final = torch.empty((n_layers, d), dtype=torch.float32, device=x.device)
    if xhist_final is None:
        xhist_final = torch.empty((n_layers, k - 1, d), dtype=torch.float32, device=x.device)
    _req(h, "h", (L, d), torch.float32)
    _req(c_final, "c_final", (n_layers, d), torch.float32)
    _req(xhist_final, "xhist_final", (n_layers, k - 1, d), torch.float32)
    if workspace is None:
        workspace = Workspace.for_shape(n_layers, d, k, T, wdt, x.device)
    wt, bt = _ptr_table(W), _ptr_table(bias)
    rc = lib.qrnn_forward(wt, bt, _p(x), _p(c_init), _p(xhist_init), _p(h), _p(c_final),
                          _p(xhist_final) if k > 1 else None, n_layers, d, L, int(T), int(k), wdt,
                          int(flags), workspace.buf.data_ptr(), workspace.nbytes, _stream_handle(stream))
    _check(rc)
    return h, c_final, xhist_final


def linear_forward(P, feat, y=None, stream=None):
    """ssrnn_linear_forward: feat [L, d_in] times P[d_out, d_in]^T -> [L, d_out]."""
    import torch
    lib = load_library()
    _req(P, "P", None, torch.float32)
    _req(feat, "feat", None, torch.float32)
    d_out, d_in = P.shape
    L = feat.shape[0]
    if y is None:
        y = torch.empty((L, d_out), dtype=torch.float32, device=feat.device)
    _req(y, "y", (L, d_out), torch.float32)
    _check(lib.ssrnn_linear_forward(_p(P), _p(feat), _p(y), d_out, d_in, L, _stream_handle(stream)))
    return y


class StreamSession:
    """A single input stream fed in chunks of any length (the on-device use the
    paper motivates, Section 1: inputs arrive over time, T steps are processed
    per weight pass).  Holds the weights, one workspace and the state carried
    between calls -- every layer's cell state and, for the QRNN, its last k-1
    inputs -- and passes that state to *_forward as both the initial and the
    final state (the ABI allows the aliasing), so a chunk boundary changes
    nothing in the results.  Marshalling only: all arithmetic is in the library."""

    def __init__(self, cell: str, W: List, bias: Optional[List] = None, *, T: int, k: int = 1, flags: int = 0,
                 c_init=None, xhist_init=None, device="cuda"):
        import torch
        if cell not in ("sru", "qrnn"):
            raise ValueError("cell must be 'sru' or 'qrnn'")
        self.cell, self.W, self.bias, self.T, self.flags = cell, W, bias, int(T), int(flags)
        self.k = 1 if cell == "sru" else int(k)
        self.n_layers = len(W)
        self.d = W[0].shape[0] // 3
        wdt = _wdtype(W[0])
        self.c = torch.zeros((self.n_layers, self.d), dtype=torch.float32, device=device)
        if c_init is not None:
            self.c.copy_(c_init)
        self.xhist = torch.zeros((self.n_layers, self.k - 1, self.d), dtype=torch.float32, device=device)
        if xhist_init is not None:
            self.xhist.copy_(xhist_init)
        self.workspace = Workspace.for_shape(self.n_layers, self.d, self.k, self.T, wdt, device)
        self.steps = 0

    def feed(self, x, h=None, stream=None):
        """Process the next x.shape[0] time steps of the stream; returns their outputs [len, d]."""
        if self.cell == "sru":
            h, _ = sru_forward(self.W, self.bias, x, self.c, T=self.T, flags=self.flags, h=h, c_final=self.c,
                               workspace=self.workspace, stream=stream)
        else:
            h, _, _ = qrnn_forward(self.W, self.bias, x, self.c, self.xhist, T=self.T, k=self.k, flags=self.flags, h=h,
                                   c_final=self.c, xhist_final=self.xhist, workspace=self.workspace, stream=stream)
        self.steps += int(x.shape[0])
        return h
