"""Helpers shared by the GPU parity tests: host numpy <-> device torch."""
import contextlib

import numpy as np
import torch

import paper_2507_16099_amd as fp8


@contextlib.contextmanager
def knobs(**values):
    """Force tuning / test switches of the library (e.g. GEMM_VARIANT=4) inside the block, defaults afterwards."""
    for k, v in values.items():
        fp8.set_knob(k, v)
    try:
        yield
    finally:
        for k in values:
            fp8.set_knob(k, None)


def dev_bf16(bits: np.ndarray, ld: int | None = None) -> torch.Tensor:
    """uint16 bfloat16 bits -> CUDA bfloat16 tensor (optionally with a padded
    leading dimension; the padding is filled with a large value so that a
    kernel that reads it by mistake is caught)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    rows, cols = bits.shape
    if ld is None:
        ld = (cols + 7) // 8 * 8
    t = torch.from_numpy(bits.view(np.int16)).cuda()
    if ld == cols:
        return t.view(torch.bfloat16)
    full = torch.full((rows, ld), 0x7F00, dtype=torch.int16, device="cuda")  # 1.7e38
    full[:, :cols] = t
    return full.view(torch.bfloat16)[:, :cols]


def dev_u8(codes: np.ndarray, ld: int | None = None) -> torch.Tensor:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    rows, cols = codes.shape
    if ld is None:
        ld = (cols + 15) // 16 * 16
    t = torch.from_numpy(codes).cuda()
    if ld == cols:
        return t
    full = torch.full((rows, ld), 0x7E, dtype=torch.uint8, device="cuda")
    full[:, :cols] = t
    return full[:, :cols]


def dev_f32(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def host_u8(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().cpu().numpy()


def host_f32(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().cpu().numpy()


def host_bf16_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def same_codes(got: np.ndarray, want: np.ndarray, nan_mask: np.ndarray | None, fmt_is_e4m3: bool) -> bool:
    """Bit-exact except where the input was NaN: there only the NaN class is
    compared (any NaN code of the format is accepted)."""
    if nan_mask is None or not nan_mask.any():
        return bool((got == want).all())
    ok = (got[~nan_mask] == want[~nan_mask]).all()
    g = got[nan_mask] & 0x7F
    is_nan = (g == 0x7F) if fmt_is_e4m3 else (g > 0x7C)
    return bool(ok and is_nan.all())


def bf16_ulp_distance(got_bits: np.ndarray, want_bits: np.ndarray) -> np.ndarray:
    """Distance in bfloat16 steps between two arrays of finite bfloat16 bit patterns (0 = identical, 1 = neighbours;
    +0 and -0 coincide)."""
    def order(b):
        b = b.astype(np.int32)
        mag = b & 0x7FFF
        return np.where(b & 0x8000, -mag, mag)
    return np.abs(order(got_bits) - order(want_bits))


def elementwise_report(got_bits: np.ndarray, want_bits: np.ndarray, want32: np.ndarray, mag32: np.ndarray | None = None) -> dict:
    """Per-element comparison of a bfloat16 GEMM result with the reference's.  The matrix cores add the products
    in their own order (and align the 128 products of one instruction to a common exponent: measured ~3e-5
    relative on one instruction), so an output carries an ABSOLUTE error proportional to the size of the
    products that went into it, before the bfloat16 rounding.  An element counts as close when it is within one
    bfloat16 step of the reference, or - for outputs that cancel to nearly zero, whose own step is smaller than
    that absolute error - within 2^-12 of the row's rms, or (mag32 given: the same product of the operands'
    absolute values, i.e. sum_k |a_k b_k| / (sa sb)) within 2^-13 of that sum.  The last form is the one that
    holds whatever the data: heavy-tailed rows have outputs far below their largest products, and the alignment
    error of an instruction scales with its LARGEST product (largest deviation seen on the outlier workload:
    about 2^-15 of the magnitude sum, on 5 of 2.8 million sampled outputs)."""
    d = bf16_ulp_distance(got_bits, want_bits)
    got = (got_bits.astype(np.uint32) << 16).view(np.float32)
    want = (want_bits.astype(np.uint32) << 16).view(np.float32)
    rms = np.sqrt((want32.astype(np.float64) ** 2).mean(axis=1, keepdims=True))
    delta = np.abs(got.astype(np.float64) - want.astype(np.float64))
    small = delta <= rms * 2.0 ** -12
    if mag32 is not None:
        small |= delta <= mag32.astype(np.float64) * 2.0 ** -13
    close1 = (d <= 1) | small
    close2 = (d <= 2) | small
    return {"identical": float((d == 0).mean()), "within_1_step": float(close1.mean()),
            "within_2_steps": float(close2.mean()), "max_steps_outside_abs": int(d[~small].max()) if (~small).any() else 0}


def assert_elementwise(got_bits, want_bits, want32, min_within1=0.999, mag32=None):
    rep = elementwise_report(got_bits, want_bits, want32, mag32)
    assert rep["within_1_step"] >= min_within1 and rep["within_2_steps"] == 1.0, rep
    return rep
