"""Pins for the oracle of the activation-quantised variant (App. E.4): the equivalent transform against the identity it
is defined by, the quantiser against its bounds, grid rows, exact rational arithmetic and a dense matmul; one test plants
mistakes."""
from fractions import Fraction

import numpy as np
import pytest

import oracle as O
from oracle import mbq_oracle_act as A
from workloads import f32_to_bf16_bits, make_weight


def activations(T, K, seed, offset=0.0):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, K)).astype(np.float32) + np.float32(offset)
    x[:, rng.choice(K, max(1, K // 100), replace=False)] *= 12.0
    return f32_to_bf16_bits(x)


def let_params(K, seed):
    rng = np.random.default_rng(seed)
    s = np.exp2(rng.uniform(-1.5, 1.5, size=K)).astype(np.float32)
    delta = rng.normal(0, 0.5, size=K).astype(np.float32)
    return delta, s


def test_transform_leaves_the_layer_output_unchanged():
    """X W + B = X~ W~ + B~ (App. E.4): a wrong sign of delta, a scale on the wrong side or a bias folded with W~
    instead of W breaks it."""
    K, N, T = 256, 24, 7
    delta, s = let_params(K, 3)
    rng = np.random.default_rng(4)
    W = rng.standard_normal((N, K))
    B = rng.standard_normal(N)
    xb = activations(T, K, 5)
    X = A.bf16_bits_to_f32(xb).astype(np.float64)
    Wt, Bt = A.let_fold(W, B, delta, s)
    Xt = (X - delta.astype(np.float64)) / s.astype(np.float64)              # the transform in fp64, for the identity
    np.testing.assert_allclose(Xt @ Wt.T + Bt, X @ W.T + B, rtol=1e-11, atol=1e-11)
    # the oracle's fp32 transform is that, rounded twice
    np.testing.assert_allclose(A.let_transform(xb, delta, s), Xt, rtol=3e-7, atol=1e-30)


def test_router_input_formula_undoes_the_transform():
    K, T = 384, 5
    delta, s = let_params(K, 8)
    xb = activations(T, K, 9)
    X = A.bf16_bits_to_f32(xb)
    back = A.undo_let(A.let_transform(xb, delta, s), delta, s)
    np.testing.assert_allclose(back, X, rtol=0, atol=6e-7 * (np.abs(X) + np.abs(delta)[None, :]).max())


@pytest.mark.parametrize("abits", [2, 3, 4, 6, 8])
@pytest.mark.parametrize("offset", [0.0, 3.0, -40.0])
def test_quantiser_bounds(abits, offset):
    """Codes and zero point are b-bit; the error is at most half a step wherever the code is not clamped, and at most
    a step anywhere; zero is a grid point; the row's extremes (with zero) span the grid."""
    T, K = 9, 512
    Xt = A.bf16_bits_to_f32(activations(T, K, [abits, 1], offset))
    xint, scale, zp, q = A.act_quant(Xt, abits)
    top = (1 << abits) - 1
    assert q.min() >= 0 and q.max() <= top and zp.min() >= 0 and zp.max() <= top
    assert np.abs(xint).max() <= top
    xhat = xint.astype(np.float64) * scale.astype(np.float64)[:, None]
    err = np.abs(Xt.astype(np.float64) - xhat)
    s64 = scale.astype(np.float64)[:, None]
    inner = (q > 0) & (q < top)
    assert np.all(err[inner] <= 0.5 * s64.repeat(K, 1)[inner] * (1 + 1e-6))
    assert np.all(err <= s64 * (1 + 1e-6))
    lo = np.minimum(Xt.min(axis=1), 0).astype(np.float64)
    hi = np.maximum(Xt.max(axis=1), 0).astype(np.float64)
    np.testing.assert_allclose(scale, (hi - lo) / top, rtol=2e-7)
    if abits == 8 and offset == 0.0:
        assert np.mean(err / s64) > 0.15            # a quantiser that does nothing would also satisfy the bounds


def test_rows_on_the_grid_are_reproduced_exactly():
    """Values k / 4 for k = -7 .. 8: range 3.75, 15 steps of exactly 0.25, zero point 7."""
    row = (np.arange(-7, 9, dtype=np.float32) * np.float32(0.25))
    Xt = np.stack([row, row[::-1], -row]).astype(np.float32)
    xint, scale, zp, q = A.act_quant(Xt, 4)
    assert np.all(scale[:2] == np.float32(0.25)) and list(zp) == [7, 7, 8]
    assert np.array_equal(xint[0], np.arange(-7, 9)) and np.array_equal(xint[1], np.arange(-7, 9)[::-1])
    assert np.array_equal(xint.astype(np.float32) * scale[:, None], Xt)
    # all zeros: scale floored, every code zero
    xint, scale, zp, q = A.act_quant(np.zeros((1, 128), dtype=np.float32), 4)
    assert not xint.any() and zp[0] == 0 and scale[0] > 0


def round_half_even(fr: Fraction) -> int:
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


def test_against_rational_arithmetic_where_fp32_is_exact():
    """Rows of dyadic values whose range is 15 x a power of two: every fp32 operation of the oracle is exact, so the
    textbook affine quantiser in rational arithmetic must give the same codes."""
    rng = np.random.default_rng(11)
    for step_log2 in (-3, 0, 2):
        step = 2.0 ** step_log2
        lo_k = int(rng.integers(-12, -2))
        vals = rng.integers(lo_k * 8, (lo_k + 15) * 8 + 1, size=64)           # eighths of a step
        vals[0], vals[1] = lo_k * 8, (lo_k + 15) * 8                            # the extremes: range = 15 steps
        Xt = (vals.astype(np.float64) * step / 8).astype(np.float32)[None, :]
        xint, scale, zp, q = A.act_quant(Xt, 4)
        assert float(scale[0]) == step and int(zp[0]) == -lo_k
        for k, v in enumerate(vals):
            want = min(15, max(0, round_half_even(Fraction(int(v), 8)) - lo_k))
            assert int(q[0, k]) == want, (step_log2, k)


def test_layer_output_reduces_to_a_dense_matmul():
    """scale_i ((q - zp) W^(p)^T) + B~ is X^ W^(p)^T + B~ with X^ the dequantised activations: a library matmul on the
    reconstructed operands, per precision."""
    N, K, T = 20, 256, 6
    W = make_weight(N, K, [5, 1], 4.0)
    codes, s0, z0 = O.encode(W)
    delta, s = let_params(K, 2)
    Xt = A.let_transform(activations(T, K, 3), delta, s)
    xint, scale, zp, q = A.act_quant(Xt, 4)
    bias = np.random.default_rng(6).standard_normal(N)
    prec = np.array([0, 1, 2, 3, 3, 1])
    Y = A.w_a_linear(xint, scale, lambda i: O.dequant(codes, s0, z0, int(prec[i])), bias)
    xhat = xint.astype(np.float64) * scale.astype(np.float64)[:, None]
    for i in range(T):
        np.testing.assert_allclose(Y[i], O.dequant(codes, s0, z0, int(prec[i])) @ xhat[i] + bias, rtol=1e-12,
                                   atol=1e-12)
    # and through the routed linear of the weight-only oracle, fed the integers as bf16 (they are exact there)
    Yint = O.linear(f32_to_bf16_bits(xint.astype(np.float32)), codes, s0, z0, prec.astype(np.int32))
    np.testing.assert_allclose(Y, Yint * scale.astype(np.float64)[:, None] + bias, rtol=1e-12, atol=1e-12)


def test_router_input_is_the_dequantised_activation_in_the_original_space():
    K, T = 256, 4
    delta, s = let_params(K, 12)
    xb = activations(T, K, 13)
    Xt = A.let_transform(xb, delta, s)
    xint, scale, zp, q = A.act_quant(Xt, 8)
    xr = A.bf16_bits_to_f32(A.router_input_bits(xint, scale, delta, s)).astype(np.float64)
    X = A.bf16_bits_to_f32(xb).astype(np.float64)
    # at 8 bits the router sees the original activations up to half a quantisation step (times s) and bf16 rounding
    bound = 0.5 * scale.astype(np.float64)[:, None] * s.astype(np.float64)[None, :] + 2.0 ** -8 * np.abs(X) + 1e-6
    assert np.all(np.abs(xr - X) <= bound * 1.01)


@pytest.mark.parametrize("mistake", ["floor", "zp_sign", "no_zero", "levels"])
def test_pins_detect_planted_mistakes(mistake):
    T, K, abits = 6, 256, 4
    top = np.float32(15)

    def broken(Xt):
        lo, hi = Xt.min(axis=1), Xt.max(axis=1)
        if mistake != "no_zero":
            lo, hi = np.minimum(lo, 0), np.maximum(hi, 0)
        scale = ((hi - lo) / (np.float32(16) if mistake == "levels" else top)).astype(np.float32)
        zp = np.clip(np.rint((lo if mistake == "zp_sign" else -lo) / scale), 0, top)
        r = np.floor(Xt / scale[:, None]) if mistake == "floor" else np.rint(Xt / scale[:, None])
        q = np.clip(r + zp[:, None], 0, top)
        return (q - zp[:, None]).astype(np.int32), scale, zp.astype(np.int32), q.astype(np.int32)

    offset = 3.0 if mistake == "no_zero" else 0.0
    Xt = A.bf16_bits_to_f32(activations(T, K, 21, offset))
    xint, scale, zp, q = broken(Xt)
    good = A.act_quant(Xt, abits)
    err = np.abs(Xt.astype(np.float64) - xint.astype(np.float64) * scale.astype(np.float64)[:, None])
    inner = (q > 0) & (q < 15)
    s64 = scale.astype(np.float64)[:, None].repeat(K, 1)
    broke_bound = np.any(err[inner] > 0.5 * s64[inner] * (1 + 1e-6)) or np.any(err > s64 * (1 + 1e-6))
    lo = np.minimum(Xt.min(axis=1), 0).astype(np.float64)
    hi = np.maximum(Xt.max(axis=1), 0).astype(np.float64)
    broke_scale = not np.allclose(scale, (hi - lo) / 15, rtol=2e-7)
    broke_range = np.abs(xint).max() > 15
    assert broke_bound or broke_scale or broke_range, mistake
    assert not np.array_equal(good[0], xint)
