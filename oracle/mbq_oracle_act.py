"""Plain CPU oracle (numpy) of the activation-quantised variant of the layer (App. E.4; `abits` of App. C.1).

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library and is never imported by the product path.

What App. E.4 fixes: the equivalent transform of the main path,
    X~ = (X - delta) / s,   W~ = s (.) W,   B~ = B + delta W          (per input channel: shift delta, scale s)
so that X~ W~ + B~ = X W + B, and the router's input, rebuilt in the original space from what the main path sees,
    X_r = X~ (.) s + delta.
What it leaves to the pipeline it builds on is the activation quantiser itself.  The reading taken here (listed with
the others in the design notes) is the usual dynamic per-token asymmetric uniform quantiser with an integer zero point:
for one token's row t = X~[i, :] and b = abits,
    lo = min(min t, 0),  hi = max(max t, 0)                 (zero lies in the range, so the zero point is a code)
    scale = max(hi - lo, 2^-100) / (2^b - 1)
    zp    = clamp(rint(-lo / scale), 0, 2^b - 1)
    q     = clamp(rint(t / scale) + zp, 0, 2^b - 1)          (rint: to nearest, ties to even)
    t^    = (q - zp) scale
Every operation above is ONE fp32 operation in exactly this order (the codes are decided in the precision of the
kernel that writes them, so both sides can be compared bit for bit); what is built from the codes - the
reconstruction error, the layer output - is fp64.
The main path then multiplies the INTEGERS q - zp (|q - zp| <= 2^b - 1, exact in bf16 for b <= 8) with the sliced
weights of W~ and scales the token's output row afterwards:
    Y[i, :] = scale_i ((q_i - zp_i) W~^(p_i)^T) + B~.
The router's input is rounded to bf16 (the router reads bf16): X_r = bf16(((q - zp) scale) s + delta), again one fp32
operation per step, then round to nearest even.
Pins (tests/test_oracle_act_pins.py): the transform leaves X W + B unchanged and is undone exactly by X_r's formula; the
half-step bound and the code range; exact reproduction of rows that lie on the grid; a rational-arithmetic
re-computation on rows where fp32 is exact; reduction of the layer output to a dense matmul; planted mistakes.
Parity against values printed in the paper: none exist for this variant (its figure reports perplexities of trained
models), so that part is parity unpinned.
"""
from __future__ import annotations

import numpy as np

__all__ = ["let_fold", "let_transform", "undo_let", "act_quant", "router_input_bits", "w_a_linear"]

F32 = np.float32


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32)


def f32_to_bf16_bits_rne(x: np.ndarray) -> np.ndarray:
    """Round to nearest even on the upper 16 bits (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))
    return (u >> np.uint64(16)).astype(np.uint16)


def let_fold(W: np.ndarray, B: np.ndarray, delta: np.ndarray, s: np.ndarray):
    """(W~, B~) of App. E.4 for W stored [N, K] (output features x input features): W~ = W s, B~ = B + W delta."""
    W = np.asarray(W, dtype=np.float64)
    return W * np.asarray(s, dtype=np.float64)[None, :], np.asarray(B, dtype=np.float64) + W @ np.asarray(
        delta, dtype=np.float64)


def let_transform(x_bits: np.ndarray, delta: np.ndarray, s: np.ndarray) -> np.ndarray:
    """X~ = (X - delta) / s, fp32 [T, K]: one subtraction and one division per element."""
    X = bf16_bits_to_f32(x_bits)
    return ((X - np.asarray(delta, dtype=F32)[None, :]).astype(F32) / np.asarray(s, dtype=F32)[None, :]).astype(F32)


def undo_let(Xt: np.ndarray, delta: np.ndarray, s: np.ndarray) -> np.ndarray:
    """X_r = X~ s + delta, fp32: one multiplication and one addition per element."""
    Xt = np.asarray(Xt, dtype=F32)
    return ((Xt * np.asarray(s, dtype=F32)[None, :]).astype(F32) + np.asarray(delta, dtype=F32)[None, :]).astype(F32)


def act_quant(Xt: np.ndarray, abits: int):
    """Per-token quantiser described in the header.  Xt fp32 [T, K] ->
    (xint int32 [T, K] = q - zp, scale fp32 [T], zp int32 [T], q int32 [T, K])."""
    assert 2 <= abits <= 8
    Xt = np.ascontiguousarray(Xt, dtype=F32)
    T, K = Xt.shape
    top = F32((1 << abits) - 1)
    lo = np.minimum(Xt.min(axis=1), F32(0)) if K else np.zeros(T, F32)
    hi = np.maximum(Xt.max(axis=1), F32(0)) if K else np.zeros(T, F32)
    rng = np.maximum((hi - lo).astype(F32), F32(2.0 ** -100)).astype(F32)
    scale = (rng / top).astype(F32)
    zp = np.clip(np.rint(((-lo).astype(F32) / scale).astype(F32)), F32(0), top).astype(F32)
    q = np.clip((np.rint((Xt / scale[:, None]).astype(F32)) + zp[:, None]).astype(F32), F32(0), top)
    q = q.astype(np.int32)
    zp = zp.astype(np.int32)
    return q - zp[:, None], scale, zp, q


def router_input_bits(xint: np.ndarray, scale: np.ndarray, delta: np.ndarray, s: np.ndarray) -> np.ndarray:
    """bf16 bits of X_r = ((q - zp) scale) s + delta (App. E.4, the router works in the original space)."""
    xhat = (xint.astype(F32) * np.asarray(scale, dtype=F32)[:, None]).astype(F32)
    return f32_to_bf16_bits_rne(undo_let(xhat, delta, s))


def w_a_linear(xint: np.ndarray, scale: np.ndarray, Wp_of_token, bias: np.ndarray = None) -> np.ndarray:
    """Y[i] = scale_i (xint_i W^(p_i)^T) + B~, fp64.  Wp_of_token(i) -> fp64 [N, K], the sliced weights of token i."""
    T = xint.shape[0]
    rows = []
    for i in range(T):
        y = np.float64(scale[i]) * (Wp_of_token(i) @ xint[i].astype(np.float64))
        rows.append(y if bias is None else y + np.asarray(bias, dtype=np.float64))
    return np.stack(rows) if rows else np.zeros((0, 0))
