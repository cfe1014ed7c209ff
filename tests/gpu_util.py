"""Helpers shared by the GPU parity tests: host numpy <-> device torch."""
import numpy as np
import torch


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
