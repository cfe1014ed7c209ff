"""Seeded synthetic inputs for the dynamically scaled float8 linear path.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests/benchmarks.  It holds none of the method's arithmetic (no amax,
no scale, no fp8 encoding, no matmul): it only draws random numbers, shapes
them like the paper's workloads (Llama-3 linear layers, Section 4 / Table 3 of
the paper train Llama3-8B) and stores them as bfloat16 bit patterns.

Every tensor is returned as a C-contiguous ``numpy.uint16`` array holding the
raw bfloat16 bits; identical bits are handed to the oracle and to the GPU.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

# ----------------------------------------------------------------------------
# fp32 -> bfloat16 storage (round to nearest, ties to even).  Input storage
# only: bfloat16 is the container the workloads arrive in.
# ----------------------------------------------------------------------------


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round a float32 array to bfloat16 (nearest-even) and return the bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    if nan.any():
        r = np.where(nan, (u >> np.uint32(16)) | np.uint32(0x40), r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bits to float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# Distributions
# ----------------------------------------------------------------------------

_CHUNK = 1 << 24  # elements drawn per call, bounds the float32 temporaries


def _stream(seed: int, stream: int) -> np.random.Generator:
    """Independent generator for (seed, stream): PCG64 seeded from a spawn key."""
    ss = np.random.SeedSequence(entropy=seed, spawn_key=(stream,))
    return np.random.Generator(np.random.PCG64(ss))


def normal_bf16(shape, std: float, seed: int, stream: int) -> np.ndarray:
    """N(0, std^2) samples stored as bfloat16 bits."""
    rng = _stream(seed, stream)
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        v = rng.standard_normal(hi - lo, dtype=np.float32)
        if std != 1.0:
            v *= np.float32(std)
        out[lo:hi] = f32_to_bf16_bits(v)
    return out.reshape(shape)


def student_t_outlier_bf16(shape, nu: float, col_frac: float, col_gain: float,
                           seed: int, stream: int) -> np.ndarray:
    """Heavy-tailed activations: Student-t(nu) = normal / sqrt(chi2_nu / nu),
    with round(col_frac * cols) columns (chosen by the same generator)
    multiplied by ``col_gain`` before the bfloat16 rounding."""
    rows, cols = shape
    rng = _stream(seed, stream)
    n_out = int(round(col_frac * cols))
    hot = np.sort(rng.choice(cols, size=n_out, replace=False)) if n_out else np.empty(0, np.int64)
    out = np.empty((rows, cols), dtype=np.uint16)
    rows_per = max(1, _CHUNK // cols)
    for lo in range(0, rows, rows_per):
        hi = min(rows, lo + rows_per)
        z = rng.standard_normal((hi - lo, cols), dtype=np.float32)
        chi = rng.chisquare(nu, size=(hi - lo, cols)).astype(np.float32)
        v = z / np.sqrt(chi / np.float32(nu))
        if n_out:
            v[:, hot] *= np.float32(col_gain)
        out[lo:hi] = f32_to_bf16_bits(v)
    return out


def small_int_bf16(shape, seed: int, stream: int, lo: int = -2, hi: int = 2, exp: int = 0) -> np.ndarray:
    """Integers in [lo, hi] times 2^exp, exactly representable in bfloat16 and fp8."""
    rng = _stream(seed, stream)
    v = rng.integers(lo, hi + 1, size=shape).astype(np.float32) * np.float32(2.0 ** exp)
    return f32_to_bf16_bits(v)


def all_bf16_patterns() -> np.ndarray:
    """All 65 536 bfloat16 bit patterns as a [256, 256] matrix."""
    return np.arange(65536, dtype=np.uint32).astype(np.uint16).reshape(256, 256)


# ----------------------------------------------------------------------------
# Workloads (the benchmark configurations)
# ----------------------------------------------------------------------------

TENSORWISE = "tensorwise"
ROWWISE = "rowwise"


@dataclass(frozen=True)
class Workload:
    """One synthetic linear layer: X [M,K], W [N,K], dY [M,N], all bfloat16."""
    name: str
    M: int
    K: int
    N: int
    recipe: str                 # TENSORWISE or ROWWISE
    pow2: bool = False          # power-of-two scales
    x_dist: tuple = ("normal", 1.0)
    w_dist: tuple = ("normal", 0.02)
    dy_dist: tuple = ("normal", 1e-3)
    backward: bool = True
    seed: int = 0
    note: str = field(default="", compare=False)

    def _draw(self, dist, shape, stream):
        if dist[0] == "normal":
            return normal_bf16(shape, dist[1], self.seed, stream)
        if dist[0] == "student_t_outlier":
            return student_t_outlier_bf16(shape, dist[1], dist[2], dist[3], self.seed, stream)
        raise ValueError(dist)

    def x(self) -> np.ndarray:
        return self._draw(self.x_dist, (self.M, self.K), 0)

    def w(self) -> np.ndarray:
        return self._draw(self.w_dist, (self.N, self.K), 1)

    def dy(self) -> np.ndarray:
        return self._draw(self.dy_dist, (self.M, self.N), 2)

    def flop_per_gemm(self) -> int:
        return 2 * self.M * self.K * self.N


WORKLOADS = {
    # small case the oracle finishes in seconds
    "c1_tensorwise_fwd_256x512x512": Workload(
        "c1_tensorwise_fwd_256x512x512", 256, 512, 512, TENSORWISE, backward=False),
    # Llama-3-8B FFN up/gate projection, 16384 tokens: the benchmark workload
    "c2_llama3_8b_ffn_rowwise": Workload(
        "c2_llama3_8b_ffn_rowwise", 16384, 4096, 14336, ROWWISE),
    # Llama-3-8B attention projections and down projection, tensorwise
    "c3_llama3_8b_qkv_tensorwise": Workload(
        "c3_llama3_8b_qkv_tensorwise", 8192, 4096, 6144, TENSORWISE,
        w_dist=("normal", 1.0), dy_dist=("normal", 1.0)),
    "c3_llama3_8b_oproj_tensorwise": Workload(
        "c3_llama3_8b_oproj_tensorwise", 8192, 4096, 4096, TENSORWISE,
        w_dist=("normal", 1.0), dy_dist=("normal", 1.0)),
    "c3_llama3_8b_down_tensorwise": Workload(
        "c3_llama3_8b_down_tensorwise", 8192, 14336, 4096, TENSORWISE,
        w_dist=("normal", 1.0), dy_dist=("normal", 1.0)),
    # Llama-3-70B FFN shapes, rowwise with power-of-two scales
    "c4_llama3_70b_up_rowwise_pow2": Workload(
        "c4_llama3_70b_up_rowwise_pow2", 8192, 8192, 28672, ROWWISE, pow2=True),
    "c4_llama3_70b_down_rowwise_pow2": Workload(
        "c4_llama3_70b_down_rowwise_pow2", 8192, 28672, 8192, ROWWISE, pow2=True),
    # outlier-heavy activations
    "c5_outlier_rowwise": Workload(
        "c5_outlier_rowwise", 4096, 4096, 11008, ROWWISE,
        x_dist=("student_t_outlier", 3.0, 0.001, 100.0), backward=False),
    "c5_outlier_tensorwise": Workload(
        "c5_outlier_tensorwise", 4096, 4096, 11008, TENSORWISE,
        x_dist=("student_t_outlier", 3.0, 0.001, 100.0), backward=False),
}

BENCH_WORKLOAD = "c2_llama3_8b_ffn_rowwise"


def scaled_down(w: Workload, M: int, K: int, N: int, name: str | None = None) -> Workload:
    """Same distributions and recipe at a smaller shape (for parity tests the
    oracle can finish in seconds)."""
    return Workload(name or f"{w.name}_small_{M}x{K}x{N}", M, K, N, w.recipe, w.pow2,
                    w.x_dist, w.w_dist, w.dy_dist, w.backward, w.seed)


def tile_band_rows(M: int, count: int = 256, tile: int = 256, seed: int = 0) -> np.ndarray:
    """Row indices for sampled GEMM parity at full size: the first and the last row of EVERY band of `tile`
    rows (every row of output tiles, and both wavefront rows inside each, is looked at), plus seeded random rows
    up to at least `count` in all; sorted, unique."""
    fixed = set()
    for first in range(0, M, tile):
        fixed.add(first)
        fixed.add(min(first + tile, M) - 1)
    rng = _stream(seed, 98)
    pool = rng.permutation(M)
    rows = set(fixed)
    for r in pool:
        if len(rows) >= min(M, count):
            break
        rows.add(int(r))
    return np.asarray(sorted(rows), dtype=np.int64)


def stratified_rows(M: int, count: int, tile: int = 256, seed: int = 0) -> np.ndarray:
    """Row indices for sampled GEMM parity: first/last rows of the first and
    last tiles plus seeded random rows, sorted, unique."""
    fixed = {0, 1, tile - 1, tile, M - tile - 1, M - tile, M - 2, M - 1}
    fixed = {r for r in fixed if 0 <= r < M}
    rng = _stream(seed, 99)
    extra = rng.choice(M, size=min(M, count), replace=False)
    rows = sorted(fixed | set(int(r) for r in extra))[: max(count, len(fixed))]
    # keep the fixed ones even after truncation
    rows = sorted(set(rows) | fixed)
    return np.asarray(rows, dtype=np.int64)
