"""Pins for the general-configuration oracle (other slice widths and group sizes, Sec. 4.1 / App. C.1): each check ties
it to something other than itself - the paper's half-step bound, a textbook uniform quantiser written here, exact
rational arithmetic, the default-configuration oracle, a library matmul - and one test plants mistakes."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle as O
from oracle import mbq_oracle_general as G
from workloads import f32_to_bf16_bits, make_weight

CONFIGS = [((2, 2, 2, 2), 128), ((4, 2, 2), 128), ((2, 4, 2), 128), ((4, 4), 128), ((6, 2), 128), ((8,), 128),
           ((2, 2, 2), 128), ((3, 1, 2, 2), 128), ((3, 2, 1), 64), ((4, 1, 1, 1, 1), 32), ((1, 1, 2), 128)]


def weight(N=24, K=512, seed=5):
    return make_weight(N, K, [77, seed], 4.0)


@pytest.mark.parametrize("slice_bits,group", CONFIGS)
def test_half_step_bound_every_precision(slice_bits, group):
    """|W - W^(p)| <= s_p / 2 (App. B error analysis) with s_p = s_0 / 2^{B_p - b_0}; the bound is tight."""
    W = weight(seed=len(slice_bits) + group)
    codes, s0, z0 = G.encode(W, slice_bits, group)
    B = G.cumulative_bits(slice_bits)
    s0d = np.repeat(s0.astype(np.float64), group, axis=1)
    z0d = np.repeat(z0.astype(np.float64), group, axis=1)
    for p in range(len(slice_bits)):
        err = np.abs(W.astype(np.float64) - G.dequant(codes, s0, z0, slice_bits, group, p))
        s_p = s0d / 2.0 ** (B[p] - B[0])
        slack = (np.abs(z0d) + 2.0 ** B[0]) * s0d * 2.0 ** -22   # fp32 rounding of z0 at the two clamped extremes
        assert np.all(err <= 0.5 * s_p + slack), p
        assert np.max(err / s_p) > 0.45
        for e in range(p + 1):
            assert codes[e].max() <= 2 ** slice_bits[e] - 1


def uniform_floor_quantiser(x, s, z, bits):
    """Written independently of the oracle: the App. B quantiser applied once at `bits` bits."""
    q = np.clip(np.floor(x / s + z), 0, 2 ** bits - 1)
    return q.astype(np.int64), s * (q - z + 0.5)


@pytest.mark.parametrize("slice_bits,group", CONFIGS)
def test_sliced_code_equals_single_shot_quantiser(slice_bits, group):
    """The digits of slices 0..p are the B_p-bit code of ONE floor quantiser with scale s_0 / 2^{B_p - b_0} and zero
    point 2^{B_p - b_0} z_0 (App. B, merged-code identity, for any widths), and lower precisions are its high bits."""
    W = weight(seed=3 * len(slice_bits) + group)
    codes, s0, z0 = G.encode(W, slice_bits, group)
    B = G.cumulative_bits(slice_bits)
    I_top = G.merged_code(codes, slice_bits, len(slice_bits) - 1)
    for p in range(len(slice_bits)):
        k = B[p] - B[0]
        s = np.repeat(s0.astype(np.float64), group, axis=1) / 2.0 ** k
        z = np.repeat(z0.astype(np.float64), group, axis=1) * 2.0 ** k
        q, deq = uniform_floor_quantiser(W.astype(np.float64), s, z, B[p])
        I = G.merged_code(codes, slice_bits, p)
        frac = (W.astype(np.float64) / s + z) % 1.0
        edge = np.minimum(frac, 1 - frac) < 1e-9
        assert np.all((q == I) | edge)
        assert np.mean(q != I) < 1e-3
        ok = q == I
        np.testing.assert_allclose(G.dequant(codes, s0, z0, slice_bits, group, p)[ok], deq[ok], rtol=0, atol=1e-15)
        assert np.array_equal(I, I_top >> (B[-1] - B[p]))      # nesting


def exact_encode_one(w, s0, z0, slice_bits):
    """The recursion of Sec. 4.1 Eq. 2 / App. B in exact rational arithmetic, any widths."""
    R, s = Fraction(float(w)), Fraction(float(s0))
    codes, recon, total = [], [], Fraction(0)
    for e, b in enumerate(slice_bits):
        if e > 0:
            s = s / 2 ** b
        z_e = Fraction(float(z0)) if e == 0 else Fraction(2 ** (b - 1))
        c = min(2 ** b - 1, max(0, math.floor(R / s + z_e)))
        w_e = s * (c - z_e + Fraction(1, 2))
        R -= w_e
        total += w_e
        codes.append(c)
        recon.append(total)
    return codes, recon


@pytest.mark.parametrize("slice_bits,group", [((4, 2, 2), 128), ((3, 1, 2, 2), 128), ((3, 2, 1), 64), ((8,), 128)])
def test_encode_against_exact_rational_recursion(slice_bits, group):
    W = weight(N=2, K=256, seed=21)
    W[0, 5] = W[0, :group].max()
    W[1, 130] = W[1, 128:128 + group].min()
    codes, s0, z0 = G.encode(W, slice_bits, group)
    for n in range(2):
        for k in range(256):
            g = k // group
            want_codes, want_rec = exact_encode_one(W[n, k], s0[n, g], z0[n, g], slice_bits)
            assert [int(codes[e][n, k]) for e in range(len(slice_bits))] == want_codes, (n, k)
            for p in range(len(slice_bits)):
                got = G.dequant(codes, s0, z0, slice_bits, group, p)[n, k]
                assert abs(Fraction(float(got)) - want_rec[p]) < Fraction(1, 10 ** 13)


def test_group_params_against_hand_values():
    """s_0 = (max - min) / 2^{b_0}, z_0 = -min / s_0 on a group with known extremes."""
    W = np.linspace(-1.0, 3.0, 64, dtype=np.float32).reshape(1, 64)
    for b0, want_s in ((1, 2.0), (2, 1.0), (3, 0.5), (4, 0.25)):
        s0, z0 = G.group_params(W, b0, 64)
        assert float(s0[0, 0]) == want_s and float(z0[0, 0]) == 1.0 / want_s
    s0, z0 = G.group_params(np.full((1, 32), 0.75, dtype=np.float32), 3, 32)       # constant group: floored range
    assert np.isfinite(z0).all() and s0[0, 0] > 0


def test_default_configuration_reduces_to_the_default_oracle():
    W = weight(seed=9)
    codes, s0, z0 = G.encode(W, (2, 2, 2, 2), 128)
    c4, s4, z4 = O.encode(W)
    assert np.array_equal(np.stack(codes).astype(np.uint8), c4)
    assert np.array_equal(s0, s4) and np.array_equal(z0, z4)
    for p in range(4):
        np.testing.assert_array_equal(G.dequant(codes, s0, z0, (2, 2, 2, 2), 128, p), O.dequant(c4, s4, z4, p))


@pytest.mark.parametrize("slice_bits", [(4, 2, 2), (2, 4, 2), (4, 4), (6, 2), (8,), (2, 2, 2), (2, 6)])
def test_even_widths_are_cuts_of_the_default_eight_bit_code(slice_bits):
    """A configuration whose cumulative widths are even cuts the SAME digit stream as four 2-bit slices at other
    places: its codes are the default oracle's base-4 digits merged, its (s_0, z_0) the default ones scaled by a power
    of two, and its reconstruction at precision p the default one at B_p / 2 digits - exactly, since every scale is a
    power-of-two multiple of the other."""
    W = weight(seed=13)
    codes, s0, z0 = G.encode(W, slice_bits, 128)
    c4, s4, z4 = O.encode(W)
    B = G.cumulative_bits(slice_bits)
    k = slice_bits[0] - 2
    assert np.array_equal(s0, (s4.astype(np.float64) / 2.0 ** k).astype(np.float32))
    assert np.array_equal(z0, (z4.astype(np.float64) * 2.0 ** k).astype(np.float32))
    for p in range(len(slice_bits)):
        d = B[p] // 2                                  # base-4 digits of precision p
        assert np.array_equal(G.merged_code(codes, slice_bits, p), O.merged_code(c4, d - 1))
        np.testing.assert_allclose(G.dequant(codes, s0, z0, slice_bits, 128, p), O.dequant(c4, s4, z4, d - 1),
                                   rtol=0, atol=1e-15)


@pytest.mark.parametrize("slice_bits,group", [((4, 2, 2), 128), ((3, 1, 2, 2), 128), ((3, 2, 1), 64)])
def test_uniform_routing_reduces_to_dense_matmul_and_slices_add(slice_bits, group):
    rng = np.random.default_rng(5)
    W = weight(N=20, K=256, seed=31)
    codes, s0, z0 = G.encode(W, slice_bits, group)
    xb = f32_to_bf16_bits(rng.standard_normal((9, 256)).astype(np.float32))
    X = G.bf16_bits_to_f64(xb)
    E = len(slice_bits)
    for p in range(E):
        Y = G.linear(xb, codes, s0, z0, slice_bits, group, np.full(9, p, dtype=np.int32))
        np.testing.assert_allclose(Y, X @ G.dequant(codes, s0, z0, slice_bits, group, p).T, rtol=1e-13, atol=1e-13)
    prec = rng.integers(0, E, size=9).astype(np.int32)
    Y = G.linear(xb, codes, s0, z0, slice_bits, group, prec)
    for i in range(9):
        want = X[i] @ G.dequant(codes, s0, z0, slice_bits, group, int(prec[i])).T
        np.testing.assert_allclose(Y[i], want, rtol=1e-13, atol=1e-13)
    B = G.cumulative_bits(slice_bits)
    assert G.avg_bits(prec, slice_bits) == float(np.mean([B[p] for p in prec]))


@pytest.mark.parametrize("mistake", ["ratio", "zero_point", "half", "first_scale"])
def test_pins_detect_planted_mistakes(monkeypatch, mistake):
    """A plausible slip in the general recursion must break the bound or the single-shot equivalence."""
    slice_bits, group = (3, 1, 2, 2), 128
    W = weight(seed=17)

    def broken_encode(W, slice_bits, group):
        W = np.ascontiguousarray(W, dtype=np.float32)
        b0 = slice_bits[0]
        s0, z0 = G.group_params(W, b0 + (1 if mistake == "first_scale" else 0), group)
        s = np.repeat(s0.astype(np.float64), group, axis=1)
        z0d = np.repeat(z0.astype(np.float64), group, axis=1)
        R = W.astype(np.float64)
        codes = []
        for e, b in enumerate(slice_bits):
            if e > 0:
                s = s / float(1 << (b - 1 if mistake == "ratio" else b))
            z_e = z0d if e == 0 else float(1 << (b - 1)) + (1.0 if mistake == "zero_point" else 0.0)
            c = np.clip(np.floor(R / s + z_e), 0.0, float((1 << b) - 1))
            codes.append(c.astype(np.uint16))
            R = R - s * ((c - z_e) + (0.0 if mistake == "half" else 0.5))
        return codes, s0, z0

    codes, s0, z0 = broken_encode(W, slice_bits, group)
    B = G.cumulative_bits(slice_bits)
    s0d = np.repeat(s0.astype(np.float64), group, axis=1)
    bad = False
    for p in range(len(slice_bits)):
        err = np.abs(W.astype(np.float64) - G.dequant(codes, s0, z0, slice_bits, group, p))
        if np.any(err > 0.5 * s0d / 2.0 ** (B[p] - B[0]) * 1.001 + 1e-6 * s0d):
            bad = True
    # the first-scale slip keeps a (looser) bound but no longer spans the range: the top codes are never used
    if mistake == "first_scale":
        bad = bad or codes[0].max() < 2 ** slice_bits[0] - 1
    assert bad, mistake
