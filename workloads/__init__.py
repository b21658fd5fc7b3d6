"""Seeded synthetic inputs for the five benchmark configurations.

This module holds NO arithmetic of the method (no gates, no recurrence, no
matrix products): only a counter-based random generator, fp32 -> bf16
rounding and fp32 -> scaled 8-bit float encoding of stored weights, and the
table of workload shapes.  It serves both
the CPU oracle's tests and the GPU tests / bench, so both sides read the same
tensors; numpy only.

Generator: value(seed, tensor_id, index) = splitmix64 finaliser of a 64-bit
counter, top 32 bits -> u in (0,1).  Uniform(+-b) = (2u-1)*b; normal = Box-
Muller on the pair of counters (2*index, 2*index+1).  Everything is computed
in float64 and rounded once to float32.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

BASE_SEED = 180311389

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _stream_key(seed: int, tensor_id: int) -> np.uint64:
    with np.errstate(over="ignore"):
        k = _mix(np.array([np.uint64(seed) * _GAMMA + np.uint64(tensor_id)], np.uint64))
        k = _mix(k + _GAMMA)
    return k[0]


def _unit(key: np.uint64, counters: np.ndarray) -> np.ndarray:
    """u in (0,1) as float64, from 64-bit counters."""
    with np.errstate(over="ignore"):
        bits = _mix(key + counters * _GAMMA)
    return ((bits >> np.uint64(32)).astype(np.float64) + 0.5) * (1.0 / 4294967296.0)


def uniform(seed: int, tensor_id: int, shape, bound: float) -> np.ndarray:
    """float32 array, entries (2u-1)*bound."""
    n = int(np.prod(shape))
    out = np.empty(n, np.float32)
    key = _stream_key(seed, tensor_id)
    for s in range(0, n, _CHUNK):
        e = min(n, s + _CHUNK)
        u = _unit(key, np.arange(s, e, dtype=np.uint64))
        out[s:e] = ((2.0 * u - 1.0) * bound).astype(np.float32)
    return out.reshape(shape)


def normal(seed: int, tensor_id: int, shape) -> np.ndarray:
    """float32 array of N(0,1) draws."""
    n = int(np.prod(shape))
    out = np.empty(n, np.float32)
    key = _stream_key(seed, tensor_id)
    for s in range(0, n, _CHUNK):
        e = min(n, s + _CHUNK)
        i = np.arange(s, e, dtype=np.uint64)
        u1 = _unit(key, i * np.uint64(2))
        u2 = _unit(key, i * np.uint64(2) + np.uint64(1))
        out[s:e] = (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)).astype(np.float32)
    return out.reshape(shape)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---- 8-bit float weights (OCP FP8 E4M3: 1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no
# infinities, S.1111.111 is NaN, largest finite value 448, subnormals m/8 * 2^-6) with one fp32 scale per
# matrix row: stored value = scale[row] * e4m3(code).

FP8_MAX = 448.0
FP8_SCALE_ALIGN = 256


def to_fp8_e4m3_bits(a: np.ndarray) -> np.ndarray:
    """Nearest E4M3 code (ties to even, magnitudes above 448 saturate to 448) of each float32; uint8."""
    a = np.ascontiguousarray(a, np.float32)
    sign = ((a.view(np.uint32) >> np.uint32(24)) & np.uint32(0x80)).astype(np.uint8)
    mag = np.minimum(np.abs(a), np.float32(FP8_MAX))
    u = mag.view(np.uint32)
    # normal range (>= 2^-6): drop 20 of the 23 mantissa bits with round-to-nearest-even, re-bias 127 -> 7
    r = u + np.uint32(0x7FFFF) + ((u >> np.uint32(20)) & np.uint32(1))
    normal = ((r >> np.uint32(20)).astype(np.int64) - ((127 - 7) << 3))
    # below 2^-6: multiples of 2^-9 (code 8 = 2^-6 is the smallest normal, so the two ranges join)
    sub = np.rint(mag.astype(np.float64) * 512.0).astype(np.int64)
    code = np.where(mag >= np.float32(2.0 ** -6), normal, sub)
    code = np.clip(code, 0, 0x7E).astype(np.uint8)
    return code | sign


@dataclass(frozen=True)
class Fp8Weight:
    """A [rows, cols] matrix as E4M3 codes q (uint8) and one fp32 scale per row."""
    q: np.ndarray
    scale: np.ndarray

    @property
    def shape(self):
        return self.q.shape

    def blob(self) -> np.ndarray:
        """The byte layout the libraries take for 8-bit weights: the codes row-major,
        zero padding up to a multiple of 256 bytes, then the rows' fp32 scales."""
        n = self.q.size
        off = (n + FP8_SCALE_ALIGN - 1) // FP8_SCALE_ALIGN * FP8_SCALE_ALIGN
        out = np.zeros(off + 4 * self.scale.size, np.uint8)
        out[:n] = np.ascontiguousarray(self.q).reshape(-1)
        out[off:] = np.ascontiguousarray(self.scale, np.float32).view(np.uint8)
        return out


def quantize_fp8(w: np.ndarray) -> Fp8Weight:
    """Per-row absmax scaling: scale = max|row| / 448 (1 for an all-zero row), codes = e4m3(w / scale),
    both in float32."""
    w = np.ascontiguousarray(w, np.float32)
    amax = np.abs(w).max(axis=1)
    scale = np.where(amax > 0, amax / np.float32(FP8_MAX), np.float32(1.0)).astype(np.float32)
    return Fp8Weight(to_fp8_e4m3_bits(w / scale[:, None]), scale)


# tensor ids within one configuration's seed
TID_X, TID_FEAT, TID_PROJ, TID_W0 = 1, 2, 3, 100


@dataclass(frozen=True)
class Workload:
    name: str
    cell: str                 # "sru" | "qrnn"
    n_layers: int
    d: int
    L: int
    Ts: Tuple[int, ...]
    k: int = 1                # causal window (QRNN); 1 for SRU
    wdtype: str = "f32"       # "f32" | "bf16" | "fp8" storage type of the weights
    d_feat: int = 0           # >0: inputs are d_feat-dim features projected to d
    index: int = 0            # position in the benchmark's config list

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    @property
    def ncol(self) -> int:
        return self.k * self.d

    def weight_bytes_per_layer(self) -> int:
        """Matrix bytes (the 12*d bytes of row scales of 8-bit weights are left out)."""
        return 3 * self.d * self.ncol * {"f32": 4, "bf16": 2, "fp8": 1}[self.wdtype]

    def algorithmic_bytes_per_step(self, T: int) -> float:
        """Bytes the method must move per time step for the whole stack: every
        layer's weights once per T steps, plus each layer's input read and
        output written (fp32)."""
        return self.n_layers * (self.weight_bytes_per_layer() / T + 2 * self.d * 4)

    def flops_per_step(self) -> float:
        return self.n_layers * 2.0 * 3 * self.d * self.ncol


CONFIGS: Tuple[Workload, ...] = (
    Workload("C1_sru1_d128", "sru", 1, 128, 64, (4,), index=0),
    Workload("C2_sru4_d1024_asr", "sru", 4, 1024, 1000, (1, 4, 16, 64), d_feat=40, index=1),
    Workload("C3_qrnn4_d1024_k2", "qrnn", 4, 1024, 1000, (1, 4, 16, 64), k=2, index=2),
    Workload("C4_sru8_d4096", "sru", 8, 4096, 2048, (1, 2, 4, 8, 16, 32, 64, 128), index=3),
    Workload("C5_qrnn8_d4096_k2_bf16", "qrnn", 8, 4096, 4096, (16, 64, 256), k=2, wdtype="bf16", index=4),
)


# Not among the benchmark's five: configuration 4 with its weights stored in bf16 and in scaled 8-bit
# floats — the small-T, low-precision-weight points (a half and a quarter of C4's bytes per step, so
# twice and four times the steps/s while HBM-bound) — and configuration 5 in 8-bit floats.
EXTRA: Tuple[Workload, ...] = (
    Workload("X1_sru8_d4096_bf16", "sru", 8, 4096, 2048, (1, 2, 4, 8, 16, 64), wdtype="bf16", index=5),
    Workload("X2_sru8_d4096_fp8", "sru", 8, 4096, 2048, (1, 2, 4, 8, 16, 64), wdtype="fp8", index=6),
    Workload("X3_qrnn8_d4096_k2_fp8", "qrnn", 8, 4096, 4096, (16, 64, 256), k=2, wdtype="fp8", index=7),
)


# The paper's comparison network (Eq. 1, Section 3.1), for the comparator rows of the bench: an LSTM stack
# with as many layers as configuration 4 and about its weight bytes (8 d^2 values per layer at d = 2560
# against 3 d^2 at d = 4096), and the paper's own "large" LSTM (one layer of width 700, 1,024 steps,
# Section 4).  W and U ~ U(+-1/sqrt(d)), biases zero, x ~ N(0, 1).
@dataclass(frozen=True)
class LstmWorkload:
    name: str
    n_layers: int
    d: int
    L: int
    Ts: Tuple[int, ...]
    index: int

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    def weight_bytes_per_layer(self) -> int:
        return 2 * 4 * self.d * self.d * 4

    def algorithmic_bytes_per_step(self, T: int, input_block: int = 16) -> float:
        """Per time step and stack: U once per step, W once per min(T, input_block) steps (the steps one
        pass over W serves), and per layer the input row read, the output row written, the 4d input
        products written and read, h_{t-1} and c read and written."""
        per_layer = 4 * self.d * self.d * 4 * (1.0 + 1.0 / min(T, input_block)) + (2 + 8 + 4) * self.d * 4
        return self.n_layers * per_layer


LSTM_CONFIGS: Tuple[LstmWorkload, ...] = (
    LstmWorkload("L1_lstm8_d2560", 8, 2560, 256, (1, 2, 4, 16, 64), index=8),
    LstmWorkload("L2_lstm1_d700_paper_large", 1, 700, 1024, (1, 4, 16, 64), index=9),
)


def make_lstm_inputs(wl: LstmWorkload, L: Optional[int] = None):
    """Returns a dict: W, U (lists of [4d, d] float32, rows f | i | o | c-hat), x [L, d] float32."""
    L = wl.L if L is None else L
    bound = 1.0 / math.sqrt(wl.d)
    return {"W": [uniform(wl.seed, TID_W0 + 2 * l, (4 * wl.d, wl.d), bound) for l in range(wl.n_layers)],
            "U": [uniform(wl.seed, TID_W0 + 2 * l + 1, (4 * wl.d, wl.d), bound) for l in range(wl.n_layers)],
            "x": normal(wl.seed, TID_X, (L * wl.d,)).reshape(L, wl.d)}


def by_name(prefix: str) -> Workload:
    for c in CONFIGS + EXTRA:
        if c.name.startswith(prefix):
            return c
    raise KeyError(prefix)


def layer_weight(wl: Workload, layer: int) -> np.ndarray:
    """[3d, k*d] weights of one layer, U(+-1/sqrt(k*d)); uint16 bf16 bits if the
    workload stores bf16, an Fp8Weight if it stores 8-bit floats."""
    w = uniform(wl.seed, TID_W0 + layer, (3 * wl.d, wl.ncol), 1.0 / math.sqrt(wl.ncol))
    if wl.wdtype == "fp8":
        return quantize_fp8(w)
    return to_bf16_bits(w) if wl.wdtype == "bf16" else w


def make_inputs(wl: Workload, L: Optional[int] = None, n_layers: Optional[int] = None, threads: int = 8):
    """Returns a dict: W (list), x [L, d] float32 or feat/P for projected
    inputs.  Biases are zero and c_init is zero in every configuration, so
    they are not generated.  L / n_layers may be cut down for prefix tests;
    the draws of a prefix equal the leading draws of the full tensors.  The
    layers of a wide stack are drawn side by side on `threads` threads (every
    value is a function of its counter, so the result does not depend on it)."""
    L_full = wl.L
    L = L_full if L is None else L
    n_layers = wl.n_layers if n_layers is None else n_layers
    if threads > 1 and n_layers > 1 and wl.d >= 2048:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=min(threads, n_layers)) as ex:
            out = {"W": list(ex.map(lambda l: layer_weight(wl, l), range(n_layers)))}
    else:
        out = {"W": [layer_weight(wl, l) for l in range(n_layers)]}
    if wl.d_feat:
        out["feat"] = normal(wl.seed, TID_FEAT, (L_full, wl.d_feat))[:L].copy()
        out["P"] = uniform(wl.seed, TID_PROJ, (wl.d, wl.d_feat), 1.0 / math.sqrt(wl.d_feat))
    else:
        # time-major, so a prefix in time is a prefix of the counter stream
        n = L * wl.d
        out["x"] = normal(wl.seed, TID_X, (n,)).reshape(L, wl.d)
    return out
