"""CPU oracle for single-stream SRU / QRNN inference (arXiv 1803.11389).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and
by the cpu_baseline leg of bench.py.  The GPU library never imports it.

The arithmetic lives in ssrnn_oracle.cpp (plain C++, double precision); this
module only compiles it with g++ and marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ssrnn_oracle.cpp")
_LIB = os.path.join(_HERE, "libssrnn_oracle.so")

F32, BF16, FP8 = 0, 1, 2

_lib = None


def compile_source(src: str, out: str) -> str:
    """g++ one oracle source file into a shared library (no GPU toolchain)."""
    cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-fopenmp",
           "-ffp-contract=off", "-o", out, src]
    subprocess.run(cmd, check=True)
    return out


def build(force: bool = False) -> str:
    """Compile the oracle if its library is missing or older than the source."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        compile_source(_SRC, _LIB)
    return _LIB


def load_library(path: str):
    """dlopen an oracle library and declare its signatures."""
    lib = ctypes.CDLL(path)
    vp, ip, lp = ctypes.c_void_p, ctypes.c_int, ctypes.c_long
    lib.oracle_num_threads.restype = ip
    lib.oracle_set_num_threads.argtypes = [ip]
    lib.oracle_sru_forward.argtypes = [vp] * 7 + [ip, ip, lp, ip, ip, ip, ip]
    lib.oracle_qrnn_forward.argtypes = [vp] * 9 + [ip, ip, lp, ip, ip, ip, ip, ip]
    lib.oracle_sru_step.argtypes = [vp] * 5 + [ip, ip]
    lib.oracle_qrnn_step.argtypes = [vp] * 5 + [ip, ip, ip]
    lib.oracle_linear_forward.argtypes = [vp] * 3 + [ip, ip, lp]
    lib.oracle_lstm_forward.argtypes = [vp] * 10 + [ip, ip, lp, ip]
    lib.oracle_lstm_step.argtypes = [vp] * 7 + [ip]
    return lib


def use_library(lib) -> None:
    """Route this module's calls to another loaded oracle library (the pin
    tests use it to show that a deliberately broken copy fails them);
    use_library(None) goes back to the real one."""
    global _lib
    _lib = lib


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = load_library(_LIB)
    return _lib


def num_threads() -> int:
    return _load().oracle_num_threads()


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def _is_fp8(w) -> bool:
    """8-bit weights come as an object with codes `q` [rows, cols] uint8, `scale`
    [rows] float32 and `blob()`, the byte layout ssrnn_oracle.cpp documents."""
    return hasattr(w, "q") and hasattr(w, "scale") and hasattr(w, "blob")


def _wdt_of(w) -> int:
    if _is_fp8(w):
        return FP8
    if w.dtype == np.float32:
        return F32
    if w.dtype == np.uint16:
        return BF16
    raise TypeError("weights must be float32, uint16 (bf16 bit patterns) or 8-bit codes with row scales")


def _storage(w):
    """(array handed to the C side, logical [rows, cols] shape)."""
    if _is_fp8(w):
        return w.blob(), tuple(w.q.shape)
    w = np.ascontiguousarray(w)
    return w, tuple(w.shape)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _ptr_array(arrs):
    """Host array of pointers; entries may be None."""
    if arrs is None:
        return None, None
    t = (ctypes.c_void_p * len(arrs))()
    for i, a in enumerate(arrs):
        t[i] = None if a is None else a.ctypes.data
    return t, arrs


def _as(a, dtype, shape=None):
    if a is None:
        return None
    a = np.ascontiguousarray(np.asarray(a), dtype=dtype)
    if shape is not None:
        a = a.reshape(shape)
    return a


def sru_forward(W, bias, x, c_init=None, T=1, return_all=False, round_operand=False, reverse=False):
    """W: list of [3d, d] float32 / uint16 arrays or 8-bit weight objects; bias: None or list of
    None / [2d] float32; x: [L, d].  round_operand: the block X of Eq. 4 enters the products rounded to
    bfloat16; reverse: every layer walks the sequence from its last step to its first.
    Returns (h, c_final[, h_all]) as float64."""
    lib = _load()
    n_layers = len(W)
    wdt = _wdt_of(W[0])
    for w in W:
        assert _wdt_of(w) == wdt
    W, shapes = zip(*[_storage(w) for w in W])
    d = shapes[0][1]
    for sh in shapes:
        assert sh == (3 * d, d)
    x = _as(x, np.float64)
    L = x.shape[0]
    assert x.shape == (L, d)
    c_init = _as(c_init, np.float64, (n_layers, d))
    if bias is not None:
        bias = [None if b is None else _as(b, np.float32, (2 * d,)) for b in bias]
    h = np.empty((L, d), np.float64)
    c_final = np.empty((n_layers, d), np.float64)
    h_all = np.empty((n_layers, L, d), np.float64) if return_all else None
    wp, _k1 = _ptr_array(W)
    bp, _k2 = _ptr_array(bias)
    rc = lib.oracle_sru_forward(wp, bp, _ptr(x), _ptr(c_init), _ptr(h), _ptr(c_final),
                                _ptr(h_all), n_layers, d, L, int(T), wdt, int(bool(round_operand)), int(bool(reverse)))
    if rc != 0:
        raise ValueError("oracle_sru_forward rejected its arguments")
    return (h, c_final, h_all) if return_all else (h, c_final)


def qrnn_forward(W, bias, x, c_init=None, xhist_init=None, T=1, k=2, return_all=False, round_operand=False, reverse=False):
    """W: list of [3d, k*d]; bias: None or list of None / [3d]; x: [L, d].  round_operand, reverse: as
    for sru_forward (in reverse the window of step t holds x_t, x_{t+1}, ...).
    Returns (h, c_final, xhist_final[, h_all]) as float64."""
    lib = _load()
    n_layers = len(W)
    wdt = _wdt_of(W[0])
    for w in W:
        assert _wdt_of(w) == wdt
    W, shapes = zip(*[_storage(w) for w in W])
    d = shapes[0][0] // 3
    for sh in shapes:
        assert sh == (3 * d, k * d)
    x = _as(x, np.float64)
    L = x.shape[0]
    assert x.shape == (L, d)
    c_init = _as(c_init, np.float64, (n_layers, d))
    xhist_init = _as(xhist_init, np.float64, (n_layers, k - 1, d))
    if bias is not None:
        bias = [None if b is None else _as(b, np.float32, (3 * d,)) for b in bias]
    h = np.empty((L, d), np.float64)
    c_final = np.empty((n_layers, d), np.float64)
    xhist_final = np.zeros((n_layers, k - 1, d), np.float64)
    h_all = np.empty((n_layers, L, d), np.float64) if return_all else None
    wp, _k1 = _ptr_array(W)
    bp, _k2 = _ptr_array(bias)
    rc = lib.oracle_qrnn_forward(wp, bp, _ptr(x), _ptr(c_init), _ptr(xhist_init), _ptr(h),
                                 _ptr(c_final), _ptr(xhist_final) if k > 1 else None,
                                 _ptr(h_all), n_layers, d, L, int(T), int(k), wdt, int(bool(round_operand)), int(bool(reverse)))
    if rc != 0:
        raise ValueError("oracle_qrnn_forward rejected its arguments")
    return (h, c_final, xhist_final, h_all) if return_all else (h, c_final, xhist_final)


def sru_step(W, bias, x_t, c):
    """One layer, one step, no blocking.  Returns (h_t, c_new) as float64."""
    lib = _load()
    wdt = _wdt_of(W)
    W, shape = _storage(W)
    d = shape[1]
    x_t = _as(x_t, np.float64, (d,))
    c = _as(c, np.float64, (d,)).copy()
    bias = _as(bias, np.float32)
    h = np.empty(d, np.float64)
    rc = lib.oracle_sru_step(_ptr(W), _ptr(bias), _ptr(x_t), _ptr(c), _ptr(h), d, wdt)
    assert rc == 0
    return h, c


def qrnn_step(W, bias, xwin, c, k):
    """xwin: [k, d], row j = x_{t-j}.  Returns (h_t, c_new) as float64."""
    lib = _load()
    wdt = _wdt_of(W)
    W, shape = _storage(W)
    d = shape[0] // 3
    xwin = _as(xwin, np.float64, (k, d))
    c = _as(c, np.float64, (d,)).copy()
    bias = _as(bias, np.float32)
    h = np.empty(d, np.float64)
    rc = lib.oracle_qrnn_step(_ptr(W), _ptr(bias), _ptr(xwin), _ptr(c), _ptr(h), d, int(k), wdt)
    assert rc == 0
    return h, c


def linear_forward(P, feat):
    """feat [L, d_in] times P[d_out, d_in]^T -> [L, d_out] float64."""
    lib = _load()
    P = _as(P, np.float32)
    feat = _as(feat, np.float32)
    d_out, d_in = P.shape
    L = feat.shape[0]
    y = np.empty((L, d_out), np.float64)
    rc = lib.oracle_linear_forward(_ptr(P), _ptr(feat), _ptr(y), d_out, d_in, L)
    assert rc == 0
    return y


def lstm_forward(W, U, bias, x, h_init=None, c_init=None, T=1, return_all=False):
    """Stacked LSTM (Eq. 1), the paper's comparison network; the input products of T steps are formed
    together (Section 3.1).  W, U: lists of [4d, d] float32 (rows f | i | o | c-hat); bias: None or list of
    None / [4d] float32; x: [L, d].  Returns (h, h_final, c_final[, h_all]) as float64."""
    lib = _load()
    n_layers = len(W)
    assert len(U) == n_layers
    W = [_as(w, np.float32) for w in W]
    U = [_as(u, np.float32) for u in U]
    d = W[0].shape[1]
    for w, u in zip(W, U):
        assert w.shape == (4 * d, d) and u.shape == (4 * d, d)
    x = _as(x, np.float64)
    L = x.shape[0]
    assert x.shape == (L, d)
    h_init = _as(h_init, np.float64, (n_layers, d))
    c_init = _as(c_init, np.float64, (n_layers, d))
    if bias is not None:
        bias = [None if b is None else _as(b, np.float32, (4 * d,)) for b in bias]
    h = np.empty((L, d), np.float64)
    h_final = np.empty((n_layers, d), np.float64)
    c_final = np.empty((n_layers, d), np.float64)
    h_all = np.empty((n_layers, L, d), np.float64) if return_all else None
    wp, _k1 = _ptr_array(W)
    up, _k2 = _ptr_array(U)
    bp, _k3 = _ptr_array(bias)
    rc = lib.oracle_lstm_forward(wp, up, bp, _ptr(x), _ptr(h_init), _ptr(c_init), _ptr(h), _ptr(h_final),
                                 _ptr(c_final), _ptr(h_all), n_layers, d, L, int(T))
    if rc != 0:
        raise ValueError("oracle_lstm_forward rejected its arguments")
    return (h, h_final, c_final, h_all) if return_all else (h, h_final, c_final)


def lstm_step(W, U, bias, x_t, h_prev, c):
    """One layer, one step of Eq. 1, brute force.  Returns (h_t, c_new) as float64."""
    lib = _load()
    W = _as(W, np.float32)
    U = _as(U, np.float32)
    d = W.shape[1]
    assert W.shape == (4 * d, d) and U.shape == (4 * d, d)
    bias = _as(bias, np.float32, (4 * d,))
    x_t = _as(x_t, np.float64, (d,))
    h_prev = _as(h_prev, np.float64, (d,))
    c = _as(c, np.float64, (d,)).copy()
    h_t = np.empty(d, np.float64)
    rc = lib.oracle_lstm_step(_ptr(W), _ptr(U), _ptr(bias), _ptr(x_t), _ptr(h_prev), _ptr(c), _ptr(h_t), d)
    if rc != 0:
        raise ValueError("oracle_lstm_step rejected its arguments")
    return h_t, c
