"""Seeded synthetic workloads shaped like the paper's SwitchTransformer experts.

Only input generation lives here: ternary symbol matrices drawn from the
i.i.d. source model (Section 4.3.2, Eq. 2), per-row scales, activation
vectors and token-to-expert routing.  None of the compression method's
arithmetic is in this module, so the tests, the benchmark and the CPU oracle
can all draw their inputs from it.

The five workloads mirror the expert shapes of Switch base128 / large128 /
c2048 (Section 5.1) and the natural-sparsity range of Table "Natural
sparsity" (Section 4.1); real weights are not available, synthetic ones from
the source model the paper validates its code against stand in for them.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, replace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libqmoe_synth.so")
_SRC = os.path.join(_HERE, "synth.c")

SEED_BASE = 23101679500


def build() -> str:
    """Compile the generator (plain C, host only)."""
    subprocess.check_call(["gcc", "-O2", "-fPIC", "-shared", "-o", _SO, _SRC, "-lm"])
    return _SO


_lib = None


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        lib = ctypes.CDLL(_SO)
        u64, i64, dbl, vp = ctypes.c_uint64, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.synth_ternary.argtypes = [u64, i64, i64, dbl, vp, vp]
        lib.synth_normal_bf16.argtypes = [u64, i64, vp]
        lib.synth_uniform_f16.argtypes = [u64, i64, dbl, dbl, vp]
        lib.synth_uniform_f64.argtypes = [u64, i64, i64, vp]
        for f in (lib.synth_ternary, lib.synth_normal_bf16, lib.synth_uniform_f16, lib.synth_uniform_f64):
            f.restype = None
        _lib = lib
    return _lib


def _seed(*parts: int) -> int:
    """Combine small integers into one 64-bit stream seed."""
    s = SEED_BASE
    for p in parts:
        s = (s * 0x100000001B3 + int(p) + 0x632BE59BD9B4E019) & 0xFFFFFFFFFFFFFFFF
    return s


def ternary(seed: int, rows: int, cols: int, p0) -> np.ndarray:
    """int8 [rows, cols] in {-1,0,+1}; p0 is a scalar or one zero-probability per row."""
    out = np.empty((rows, cols), dtype=np.int8)
    if np.isscalar(p0):
        _load().synth_ternary(seed, rows, cols, float(p0), None, out.ctypes.data)
    else:
        p = np.ascontiguousarray(p0, dtype=np.float64)
        assert p.shape == (rows,)
        _load().synth_ternary(seed, rows, cols, 0.0, p.ctypes.data, out.ctypes.data)
    return out


def normal_bf16(seed: int, shape) -> np.ndarray:
    """bfloat16 bit patterns (uint16) of standard-normal draws."""
    out = np.empty(shape, dtype=np.uint16)
    _load().synth_normal_bf16(seed, out.size, out.ctypes.data)
    return out


def uniform_f16(seed: int, shape, lo: float, hi: float) -> np.ndarray:
    """binary16 bit patterns (uint16) of uniform[lo,hi) draws."""
    out = np.empty(shape, dtype=np.uint16)
    _load().synth_uniform_f16(seed, out.size, lo, hi, out.ctypes.data)
    return out


def f64_to_bf16(v: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) of finite values that float32 holds exactly or nearly so:
    float32 first, then round-to-nearest-even on the low 16 bits."""
    b = np.ascontiguousarray(v, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return ((b + 0x7FFF + ((b >> 16) & 1)) >> 16).astype(np.uint16)


def minmax_bf16(seed: int, rows: int, lo: float, hi: float) -> np.ndarray:
    """bfloat16 bit patterns [rows, 2] of (w_min, w_max): w_max and -w_min uniform in [lo, hi)."""
    u = uniform_f64(seed, 2 * rows).reshape(rows, 2)
    mag = lo + (hi - lo) * u
    mag[:, 0] = -mag[:, 0]
    return f64_to_bf16(mag)


def uniform_f64(seed: int, n: int, first: int = 0) -> np.ndarray:
    out = np.empty(n, dtype=np.float64)
    _load().synth_uniform_f64(seed, first, n, out.ctypes.data)
    return out


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def f16_to_f64(bits: np.ndarray) -> np.ndarray:
    return bits.view(np.float16).astype(np.float64)


def permutation(seed: int, n: int) -> np.ndarray:
    return np.argsort(uniform_f64(seed, n), kind="stable").astype(np.int64)


@dataclass(frozen=True)
class Workload:
    """One synthetic MoE FFN layer (or a single matrix when n_experts == 0)."""

    name: str
    cfg_id: int
    n_experts: int
    d_model: int
    d_ff: int
    p0: float            # zero probability; ignored when p0_spread is set
    n_tokens: int        # 0: derived from per-expert batch sizes
    routing: str         # "single" | "uniform" | "zipf" | "batch"
    zipf_s: float = 1.1
    p0_spread: bool = False   # per-row zero fraction 0.80 + 0.17 * Beta(2,2)
    batch_lo: int = 1
    batch_hi: int = 32

    # ---- weights -------------------------------------------------------
    def _p0_rows(self, expert: int, which: int, rows: int):
        if not self.p0_spread:
            return self.p0
        u = uniform_f64(_seed(self.cfg_id, 7, which, expert), 3 * rows).reshape(rows, 3)
        return 0.80 + 0.17 * np.median(u, axis=1)  # median of three uniforms ~ Beta(2,2)

    def wi_ternary(self, expert: int) -> np.ndarray:
        """[d_ff rows = outputs, d_model cols = inputs]"""
        return ternary(_seed(self.cfg_id, 1, expert), self.d_ff, self.d_model,
                       self._p0_rows(expert, 1, self.d_ff))

    def wo_ternary(self, expert: int) -> np.ndarray:
        """[d_model rows = outputs, d_ff cols = inputs]"""
        return ternary(_seed(self.cfg_id, 2, expert), self.d_model, self.d_ff,
                       self._p0_rows(expert, 2, self.d_model))

    def wi_scale(self, expert: int) -> np.ndarray:
        return uniform_f16(_seed(self.cfg_id, 3, expert), (self.d_ff,), 0.01, 0.1)

    def wo_scale(self, expert: int) -> np.ndarray:
        return uniform_f16(_seed(self.cfg_id, 4, expert), (self.d_model,), 0.01, 0.1)

    # (w_min, w_max) of each output row for the asymmetric grid: bfloat16 bits [rows, 2],
    # w_min in (-0.1, -0.01], w_max in [0.01, 0.1), drawn apart
    def wi_minmax(self, expert: int) -> np.ndarray:
        return minmax_bf16(_seed(self.cfg_id, 9, expert), self.d_ff, 0.01, 0.1)

    def wo_minmax(self, expert: int) -> np.ndarray:
        return minmax_bf16(_seed(self.cfg_id, 10, expert), self.d_model, 0.01, 0.1)

    def expert_idx(self) -> np.ndarray:
        E = self.n_experts
        if self.routing == "single":
            return np.zeros(self.n_tokens, dtype=np.int32)
        if self.routing == "uniform":
            u = uniform_f64(_seed(self.cfg_id, 5), self.n_tokens)
            return np.minimum((u * E).astype(np.int32), E - 1)
        if self.routing == "zipf":
            w = np.arange(1, E + 1, dtype=np.float64) ** (-self.zipf_s)
            cdf = np.cumsum(w / w.sum())
            u = uniform_f64(_seed(self.cfg_id, 5), self.n_tokens)
            rank = np.minimum(np.searchsorted(cdf, u, side="right"), E - 1)
            rank_to_expert = permutation(_seed(self.cfg_id, 6), E)
            return rank_to_expert[rank].astype(np.int32)
        if self.routing == "batch":
            u = uniform_f64(_seed(self.cfg_id, 5), E)
            span = self.batch_hi - self.batch_lo + 1
            b = self.batch_lo + np.minimum((u * span).astype(np.int64), span - 1)
            idx = np.repeat(np.arange(E, dtype=np.int32), b)
            return idx[permutation(_seed(self.cfg_id, 6), idx.size)]
        raise ValueError(self.routing)

    def tokens(self) -> np.ndarray:
        """bfloat16 bits [T, d_model], N(0,1)."""
        T = self.expert_idx().size
        return normal_bf16(_seed(self.cfg_id, 8), (T, self.d_model))

    def scaled(self, **kw) -> "Workload":
        """Same recipe at other sizes (for tests that must finish in seconds)."""
        return replace(self, **kw)


WORKLOADS = {
    "base_wi_single": Workload("base_wi_single", 1, 1, 768, 3072, 0.90, 1, "single"),
    "switch_base128": Workload("switch_base128", 2, 128, 768, 3072, 0.90, 128, "uniform"),
    "switch_large128": Workload("switch_large128", 3, 128, 1024, 4096, 0.92, 512, "uniform"),
    "c2048": Workload("c2048", 4, 2048, 2080, 6144, 0.90, 2048, "zipf"),
    "c2048_ragged256": Workload("c2048_ragged256", 5, 256, 2080, 6144, 0.885, 0, "batch",
                                p0_spread=True),
    # c2048 at the natural sparsity the paper's table of natural sparsity reports for its 2-bit model (76.5 %):
    # the densest weights the paper shows.  The values stay ternary (the paper has no code for four levels).
    "c2048_sparsity765": Workload("c2048_sparsity765", 6, 2048, 2080, 6144, 0.765, 2048, "zipf"),
}
