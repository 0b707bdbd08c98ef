"""Plain CPU oracle (numpy, fp64) of MoBiSlice for GENERAL slice configurations.

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library and is never imported by the product path.

Sec. 4.1 states the method for E slices of b_e bits each ("slice_bits_list" in App. C.1, group size g); the default
configuration of the paper, and of ``mbq_oracle``, is E = 4, b_e = 2, g = 128.  This module is the literal recursion for
any list of widths and any group size:

    slice 0:   s_0 = (max - min) / 2^{b_0},  z_0 = -min / s_0          (min/max fit, continuous zero point; App. B)
    slice e:   s_e = s_{e-1} / 2^{b_e},      z_e = 2^{b_e - 1}          (scale refinement, centred residual zero point)
    c_e = clamp(floor(R_e / s_e + z_e), 0, 2^{b_e} - 1),   R_{e+1} = R_e - s_e ((c_e - z_e) + 0.5),   R_0 = W
    W^(p) = sum_{e <= p} s_e ((c_e - z_e) + 0.5)                        (Eq. 3),  B_p = b_0 + ... + b_p bits

with the same readings as ``mbq_oracle`` (ratio 2^{b_e} between consecutive scales; s_0, z_0 single fp32 operations
and stored fp32; range floor for constant groups; recursion in fp64 in exactly this order).
Pins (tests/test_oracle_general_pins.py): half-step bound, equivalence with the single-shot B_p-bit floor quantiser,
mixed-radix digits of the B-bit code, exact rational recursion on small inputs, reduction to ``mbq_oracle`` at the
default configuration, dense-matmul reduction of the routed linear.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np

__all__ = ["check_config", "cumulative_bits", "group_params", "encode", "slice_matrix", "dequant", "merged_code",
           "linear", "avg_bits"]


def check_config(slice_bits: Sequence[int], group: int) -> None:
    assert len(slice_bits) >= 1 and all(int(b) >= 1 for b in slice_bits), "every slice needs at least one bit"
    assert sum(slice_bits) <= 16, "codes are held in 16 bits here"
    assert group >= 1


def cumulative_bits(slice_bits: Sequence[int]) -> List[int]:
    """B_p = b_0 + ... + b_p, the bits of precision p."""
    out, acc = [], 0
    for b in slice_bits:
        acc += int(b)
        out.append(acc)
    return out


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def group_params(W: np.ndarray, b0: int, group: int):
    """(s_0, z_0) per (row, group), fp32: 2^{b_0} floor-aligned bins tile [min, max]."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    N, K = W.shape
    assert K % group == 0
    Wg = W.reshape(N, K // group, group)
    lo = Wg.min(axis=2)
    hi = Wg.max(axis=2)
    rng = (hi - lo).astype(np.float32)
    mag = np.maximum(np.abs(lo), np.abs(hi)).astype(np.float32)
    floor_rng = np.maximum(mag * np.float32(2.0 ** -16), np.float32(2.0 ** -100)).astype(np.float32)
    rng = np.maximum(rng, floor_rng).astype(np.float32)
    s0 = (rng / np.float32(2.0 ** b0)).astype(np.float32)
    z0 = ((-lo).astype(np.float32) / s0).astype(np.float32)
    return s0, z0


def _scales(s0: np.ndarray, slice_bits: Sequence[int], group: int):
    """s_e per element, fp64, e = 0..E-1 (each an exact power-of-two fraction of s_0)."""
    s = np.repeat(s0.astype(np.float64), group, axis=1)
    out = [s]
    for b in slice_bits[1:]:
        s = s / float(1 << int(b))
        out.append(s)
    return out


def encode(W: np.ndarray, slice_bits: Sequence[int], group: int):
    """Returns (codes: list of E uint16 arrays [N, K], s0 fp32 [N, K/group], z0 fp32 [N, K/group])."""
    check_config(slice_bits, group)
    W = np.ascontiguousarray(W, dtype=np.float32)
    s0, z0 = group_params(W, int(slice_bits[0]), group)
    scales = _scales(s0, slice_bits, group)
    z0d = np.repeat(z0.astype(np.float64), group, axis=1)
    R = W.astype(np.float64)
    codes = []
    for e, b in enumerate(slice_bits):
        s_e = scales[e]
        z_e = z0d if e == 0 else float(1 << (int(b) - 1))
        c = np.clip(np.floor(R / s_e + z_e), 0.0, float((1 << int(b)) - 1))
        codes.append(c.astype(np.uint16))
        R = R - s_e * ((c - z_e) + 0.5)
    return codes, s0, z0


def slice_matrix(codes, s0, z0, slice_bits: Sequence[int], group: int, e: int) -> np.ndarray:
    """W_e = s_e ((c_e - z_e) + 0.5), fp64 [N, K]."""
    s_e = _scales(s0, slice_bits, group)[e]
    z_e = np.repeat(z0.astype(np.float64), group, axis=1) if e == 0 else float(1 << (int(slice_bits[e]) - 1))
    return s_e * ((codes[e].astype(np.float64) - z_e) + 0.5)


def dequant(codes, s0, z0, slice_bits: Sequence[int], group: int, p: int) -> np.ndarray:
    """W^(p) = sum_{e <= p} W_e (Eq. 3)."""
    out = slice_matrix(codes, s0, z0, slice_bits, group, 0)
    for e in range(1, p + 1):
        out = out + slice_matrix(codes, s0, z0, slice_bits, group, e)
    return out


def merged_code(codes, slice_bits: Sequence[int], p: int) -> np.ndarray:
    """I_p: the B_p-bit code whose mixed-radix digits are the codes of slices 0..p."""
    I = np.zeros(codes[0].shape, dtype=np.int64)
    for e in range(p + 1):
        I = (I << int(slice_bits[e])) + codes[e].astype(np.int64)
    return I


def linear(x_bits: np.ndarray, codes, s0, z0, slice_bits: Sequence[int], group: int, prec: np.ndarray) -> np.ndarray:
    """Routed output (Eq. 6 with the prefix mask): Y_i = sum_{e <= p_i} W_e^T X_i, fp64 [T, N]."""
    X = bf16_bits_to_f64(x_bits)
    T = X.shape[0]
    N = codes[0].shape[0]
    Y = np.zeros((T, N), dtype=np.float64)
    for e in range(len(slice_bits)):
        gate = (np.asarray(prec) >= e).astype(np.float64)[:, None]
        if not gate.any():
            continue
        Y += (gate * X) @ slice_matrix(codes, s0, z0, slice_bits, group, e).T
    return Y


def avg_bits(prec: np.ndarray, slice_bits: Sequence[int]) -> float:
    """AvgBits (Eq. 8): mean over tokens of the bits of their active slices."""
    prec = np.asarray(prec)
    if prec.size == 0:
        return 0.0
    B = np.asarray(cumulative_bits(slice_bits), dtype=np.float64)
    return float(np.mean(B[prec]))
