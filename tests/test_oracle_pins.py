"""Pins for the CPU oracle: each check ties an oracle function to something other than
itself - the paper's error bound, a textbook uniform quantiser, exact rational
arithmetic, library matmul/sort routines, a hand-worked example."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle as O
from workloads import f32_to_bf16_bits, make_weight

HERE = os.path.dirname(os.path.abspath(__file__))


def student_matrix(N=48, K=512, seed=7, df=4.0):
    return make_weight(N, K, [99, seed], df)


# ------------------------------------------------------------------ worked example
def load_worked_example():
    rows, ys = [], []
    with open(os.path.join(HERE, "golden", "worked_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            tok = line.split()
            if tok[0] == "Y":
                ys.append((int(tok[1]), float(tok[2])))
            else:
                rows.append((int(tok[0]), float(tok[1]), [int(t) for t in tok[2:6]],
                             [float(t) for t in tok[6:10]]))
    return rows, ys


def worked_weight(rows):
    W = np.full((1, 128), 0.5, dtype=np.float32)
    for idx, w, _, _ in rows:
        W[0, idx] = w
    return W


def test_worked_example_codes_and_reconstruction():
    rows, _ = load_worked_example()
    W = worked_weight(rows)
    codes, s0, z0 = O.encode(W)
    assert s0[0, 0] == 1.0 and z0[0, 0] == 1.0
    for idx, _, want_codes, want_rec in rows:
        assert [int(codes[e, 0, idx]) for e in range(4)] == want_codes
        for p in range(4):
            assert O.dequant(codes, s0, z0, p)[0, idx] == pytest.approx(want_rec[p], abs=1e-12)
    # every filler weight behaves like row 4 of the table
    assert (codes[:, 0, 5:] == codes[:, 0, 4:5]).all()


def test_worked_example_routed_output():
    rows, ys = load_worked_example()
    W = worked_weight(rows)
    codes, s0, z0 = O.encode(W)
    x = np.zeros((1, 128), dtype=np.float32)
    x[0, 0], x[0, 2] = 1.0, 2.0
    xb = f32_to_bf16_bits(x)
    for p, want in ys:
        y = O.linear(xb, codes, s0, z0, np.array([p], dtype=np.int32))
        assert y.shape == (1, 1)
        assert y[0, 0] == pytest.approx(want, abs=1e-12)


# ----------------------------------------------------------------------- bf16 input
def test_bf16_decoding_against_known_patterns():
    bits = np.array([0x3F80, 0xC020, 0x0000, 0x8000, 0x4049, 0x3C00, 0x7F7F], dtype=np.uint16)
    want = [1.0, -2.5, 0.0, -0.0, 3.140625, 2.0 ** -7, (2 - 2 ** -7) * 2.0 ** 127]
    got = O.bf16_bits_to_f64(bits)
    assert got.tolist() == want
    # and the generator's rounding is round-to-nearest-even onto that grid
    x = np.array([1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20], dtype=np.float32)
    assert O.bf16_bits_to_f64(f32_to_bf16_bits(x)).tolist() == [1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7]


# ------------------------------------------------------------------- base-slice fit
def test_group_params_minmax_fit():
    W = student_matrix()
    s0, z0 = O.group_params(W)
    Wg = W.reshape(W.shape[0], -1, 128).astype(np.float64)
    lo, hi = Wg.min(axis=2), Wg.max(axis=2)
    assert s0.dtype == np.float32 and z0.dtype == np.float32
    np.testing.assert_allclose(4.0 * s0.astype(np.float64), hi - lo, rtol=2e-7)
    # lo lands in code 0, hi on the top edge (u = 4 up to fp32 rounding of z0)
    u_lo = lo / s0 + z0
    u_hi = hi / s0 + z0
    assert np.all(np.abs(u_lo) < 1e-5) and np.all(np.abs(u_hi - 4.0) < 1e-5)


def test_group_params_degenerate_groups():
    W = np.zeros((3, 256), dtype=np.float32)
    W[1, :128] = 0.75          # constant non-zero group
    W[2, 128:] = -3.0e-30      # tiny constant group
    codes, s0, z0 = O.encode(W)
    assert np.all(np.isfinite(s0)) and np.all(s0 > 0) and np.all(np.isfinite(z0))
    assert np.all(np.abs(z0) <= 2.0 ** 18 + 1)
    for p in range(4):
        err = np.abs(O.dequant(codes, s0, z0, p) - W)
        bound = np.repeat(s0.astype(np.float64), 128, axis=1) / 4 ** p * 0.5
        slack = np.repeat((np.abs(z0) + 4.0) * s0 * 2.0 ** -22, 128, axis=1)
        assert np.all(err <= bound + slack)


# ------------------------------------------------- paper's half-step bound (App. B)
@pytest.mark.parametrize("df", [3.0, 4.0])
def test_half_step_bound_every_precision(df):
    W = student_matrix(seed=3, df=df)
    codes, s0, z0 = O.encode(W)
    s0d = np.repeat(s0.astype(np.float64), 128, axis=1)
    z0d = np.repeat(z0.astype(np.float64), 128, axis=1)
    for p in range(4):
        err = np.abs(W.astype(np.float64) - O.dequant(codes, s0, z0, p))
        s_p = s0d / 4 ** p
        # slack: fp32 rounding of z0 can push the two extreme elements of a group past the clamp
        slack = (np.abs(z0d) + 4.0) * s0d * 2.0 ** -22
        assert np.all(err <= 0.5 * s_p + slack), p
        # bound is tight (some element within 2% of it) and not trivially loose
        assert np.max(err / s_p) > 0.49


# ------------------------- textbook single-shot quantiser at 2(p+1) bits (App. B end)
def uniform_floor_quantiser(x, s, z, bits):
    """Written independently of the oracle: the App. B quantiser applied once."""
    q = np.clip(np.floor(x / s + z), 0, 2 ** bits - 1)
    return q.astype(np.int64), s * (q - z + 0.5)


@pytest.mark.parametrize("p", [0, 1, 2, 3])
def test_sliced_code_equals_single_shot_quantiser(p):
    W = student_matrix(seed=5)
    codes, s0, z0 = O.encode(W)
    s = np.repeat(s0.astype(np.float64), 128, axis=1) / 4 ** p     # s' = 2^{-2p} s0
    z = np.repeat(z0.astype(np.float64), 128, axis=1) * 4 ** p     # z' = 2^{2p} z0
    q, deq = uniform_floor_quantiser(W.astype(np.float64), s, z, 2 * (p + 1))
    I = O.merged_code(codes, p)
    # codes can differ only for a weight sitting on a bin edge to within fp64 rounding
    frac = (W.astype(np.float64) / s + z) % 1.0
    edge = np.minimum(frac, 1 - frac) < 1e-9
    assert np.all((q == I) | edge)
    assert np.mean(q != I) < 1e-4
    ok = q == I
    np.testing.assert_allclose(O.dequant(codes, s0, z0, p)[ok], deq[ok], rtol=0, atol=1e-15)
    np.testing.assert_allclose(O.dequant_merged(codes, s0, z0, p)[ok], deq[ok], rtol=0, atol=1e-15)


def test_nesting_and_digit_closed_form():
    W = student_matrix(seed=11)
    codes, s0, z0 = O.encode(W)
    digits = O.encode_digits(W, s0, z0)
    assert np.mean(digits != codes) < 1e-5
    I3 = O.merged_code(codes, 3)
    for p in range(4):
        assert np.array_equal(O.merged_code(codes, p), I3 >> (6 - 2 * p))
        np.testing.assert_allclose(O.dequant(codes, s0, z0, p), O.dequant_merged(codes, s0, z0, p),
                                   rtol=0, atol=1e-15)


# ------------------------------------------- exact rational brute force, tiny inputs
def exact_encode_one(w, s0, z0):
    """The recursion of Sec. 4.1 Eq. 2 / App. B in exact rational arithmetic."""
    R = Fraction(float(w))
    s = Fraction(float(s0))
    z_first = Fraction(float(z0))
    codes, recon, total = [], [], Fraction(0)
    for e in range(4):
        s_e = s / 4 ** e
        z_e = z_first if e == 0 else Fraction(2)
        c = min(3, max(0, math.floor(R / s_e + z_e)))
        w_e = s_e * (c - z_e + Fraction(1, 2))
        R -= w_e
        total += w_e
        codes.append(c)
        recon.append(total)
    return codes, recon


def test_encode_against_exact_rational_recursion():
    W = student_matrix(N=2, K=256, seed=21)
    W[0, 5] = W[0, :128].max()        # duplicates of the extremes
    W[1, 130] = W[1, 128:].min()
    codes, s0, z0 = O.encode(W)
    for n in range(2):
        for k in range(256):
            g = k // 128
            want_codes, want_rec = exact_encode_one(W[n, k], s0[n, g], z0[n, g])
            assert [int(codes[e, n, k]) for e in range(4)] == want_codes, (n, k)
            for p in range(4):
                got = O.dequant(codes, s0, z0, p)[n, k]
                assert abs(Fraction(float(got)) - want_rec[p]) < Fraction(1, 10 ** 13)


# ------------------------------------------------ lattice statistics (zero-mean, bound)
def test_lattice_error_statistics():
    lo, hi = -0.37, 0.91
    n = 128 * 4096
    W = np.linspace(lo, hi, n, dtype=np.float64).astype(np.float32).reshape(4096, 128)
    W[:, 0], W[:, -1] = lo, hi       # every group spans the same range
    codes, s0, z0 = O.encode(W)
    prev_max, prev_rms = np.inf, np.inf
    for p in range(4):
        s_p = float(s0[0, 0]) / 4 ** p
        # columns 0 and 127 are the planted range ends, not lattice points: leave them out
        err = (O.dequant(codes, s0, z0, p) - W.astype(np.float64))[:, 1:-1].ravel()
        assert np.max(np.abs(err)) == pytest.approx(s_p / 2, rel=2e-3)
        assert np.sqrt(np.mean(err ** 2)) == pytest.approx(s_p / math.sqrt(12), rel=5e-3)
        assert abs(np.mean(err)) < 2e-3 * s_p
        assert np.max(np.abs(err)) < prev_max and np.sqrt(np.mean(err ** 2)) < prev_rms
        prev_max, prev_rms = np.max(np.abs(err)), np.sqrt(np.mean(err ** 2))


def test_adding_a_slice_refines_in_aggregate():
    W = student_matrix(seed=13)
    codes, s0, z0 = O.encode(W)
    norms = [np.linalg.norm(W - O.dequant(codes, s0, z0, p)) for p in range(4)]
    for a, b in zip(norms, norms[1:]):
        assert 3.5 < a / b < 4.6          # about 4x per 2-bit slice
    # per element the error may grow (a weight on a bin centre), but never past the new half step
    s0d = np.repeat(s0.astype(np.float64), 128, axis=1)
    for p in range(3):
        nxt = np.abs(W - O.dequant(codes, s0, z0, p + 1))
        assert np.all(nxt <= s0d / 4 ** (p + 1) * 0.5 * (1 + 1e-4) + 1e-12)


# --------------------------------------------------------------------------- packing
def test_canonical_packing_known_word_and_round_trip():
    codes = np.zeros((4, 1, 16), dtype=np.uint8)
    codes[0, 0] = np.arange(16) % 4
    codes[1, 0, 15] = 3
    words = O.pack_canonical(codes)
    assert words.shape == (4, 1, 1)
    assert int(words[0, 0, 0]) == 0xE4E4E4E4 and int(words[1, 0, 0]) == 0xC0000000
    rng = np.random.default_rng(1)
    c = rng.integers(0, 4, size=(4, 7, 384), dtype=np.uint8)
    assert np.array_equal(O.unpack_canonical(O.pack_canonical(c)), c)


def blob_reference_loops(codes, s0, z0):
    """The blob format of include/mbq.h restated element by element."""
    E, N, K = codes.shape
    nt, kb = -(-N // 16), -(-K // 256)
    words = np.zeros(E * nt * kb * 256, dtype=np.uint32)
    for e in range(E):
        for n in range(N):
            for k in range(K):
                r = k % 256
                d, step, kq, s = r // 64, (r % 64) // 32, (r % 32) // 8, r % 8
                lane = 16 * kq + n % 16
                word = (((e * nt + n // 16) * kb + k // 256) * 64 + lane) * 4 + d
                bit = (16 * (s & 1) + 4 * (s >> 1) + 2 * step + (2 - 2 * e)) % 32
                words[word] |= np.uint32(int(codes[e, n, k]) << bit)
    meta = np.zeros((nt, 2 * kb, 16, 2), dtype=np.float32)
    for n in range(N):
        for g in range(K // 128):
            meta[n // 16, g, n % 16, 0] = s0[n, g]
            meta[n // 16, g, n % 16, 1] = z0[n, g]
    return np.concatenate([words.view(np.uint8), meta.reshape(-1).view(np.uint8)])


@pytest.mark.parametrize("N,K", [(16, 256), (21, 384), (3, 128)])
def test_blob_layout_against_elementwise_statement(N, K):
    rng = np.random.default_rng(N * 1000 + K)
    codes = rng.integers(0, 4, size=(4, N, K), dtype=np.uint8)
    s0 = rng.random((N, K // 128), dtype=np.float32) + 0.1
    z0 = rng.random((N, K // 128), dtype=np.float32) * 4
    blob = O.pack_blob(codes, s0, z0)
    assert blob.dtype == np.uint8 and blob.size == O.blob_bytes(N, K)
    assert np.array_equal(blob, blob_reference_loops(codes, s0, z0))


# ----------------------------------------------------------------------------- route
def test_route_against_fsum_and_tie_rule():
    rng = np.random.default_rng(5)
    T, K = 9, 256
    x = rng.standard_normal((T, K)).astype(np.float32)
    xb = f32_to_bf16_bits(x)
    Wr = (rng.standard_normal((4, K)) / 16).astype(np.float32)
    br = np.array([0.1, -0.2, 0.05, 0.0], dtype=np.float32)
    Wr[1] = Wr[0]
    br[1] = br[0]                      # rows 0 and 1 tie exactly for every token
    S, prec, gap = O.route(xb, Wr, br)
    xv = O.bf16_bits_to_f64(xb)
    for i in range(T):
        want = [math.fsum(float(xv[i, k]) * float(Wr[q, k]) for k in range(K)) + float(br[q])
                for q in range(4)]
        np.testing.assert_allclose(S[i], want, rtol=0, atol=1e-12)
        best = max(want)
        first = min(q for q in range(4) if S[i, q] == S[i].max())
        assert prec[i] == first
        if abs(want[0] - best) < 1e-12:
            assert prec[i] == 0 and gap[i] == 0.0       # exact tie -> lowest index, zero gap
        else:
            srt = sorted(want)
            assert gap[i] == pytest.approx(srt[-1] - srt[-2], abs=1e-12)


def test_bucket_against_stable_sort():
    rng = np.random.default_rng(8)
    for T in (0, 1, 5, 64, 257):
        prec = rng.integers(0, 4, size=T).astype(np.int32)
        if T == 5:
            prec[:] = 2                                  # three empty buckets
        perm, offsets = O.bucket(prec)
        assert np.array_equal(perm, np.argsort(prec, kind="stable").astype(np.int32))
        assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(np.bincount(prec, minlength=4))]))


def test_avg_bits():
    assert O.avg_bits(np.array([0, 0, 1, 3])) == pytest.approx((2 + 2 + 4 + 8) / 4)
    assert O.avg_bits(np.array([], dtype=np.int32)) == 0.0


# ---------------------------------------------------------------------------- linear
def test_uniform_routing_reduces_to_dense_matmul():
    W = student_matrix(N=40, K=384, seed=17)
    codes, s0, z0 = O.encode(W)
    rng = np.random.default_rng(3)
    xb = f32_to_bf16_bits(rng.standard_normal((11, 384)).astype(np.float32))
    X = torch.from_numpy(O.bf16_bits_to_f64(xb))
    for p in range(4):
        # independent closed-form weight + library matmul
        s = np.repeat(s0.astype(np.float64), 128, axis=1) / 4 ** p
        z = np.repeat(z0.astype(np.float64), 128, axis=1) * 4 ** p
        What = torch.from_numpy(uniform_floor_quantiser(W.astype(np.float64), s, z, 2 * (p + 1))[1])
        want = (X @ What.T).numpy()
        got = O.linear(xb, codes, s0, z0, np.full(11, p, dtype=np.int32))
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-10 * np.abs(want).max())


def test_mixed_routing_rows_and_slice_linearity():
    W = student_matrix(N=24, K=256, seed=19)
    codes, s0, z0 = O.encode(W)
    rng = np.random.default_rng(4)
    xb = f32_to_bf16_bits(rng.standard_normal((13, 256)).astype(np.float32))
    prec = rng.integers(0, 4, size=13).astype(np.int32)
    Y = O.linear(xb, codes, s0, z0, prec)
    X = torch.from_numpy(O.bf16_bits_to_f64(xb))
    per_p = [O.linear(xb, codes, s0, z0, np.full(13, p, dtype=np.int32)) for p in range(4)]
    for i in range(13):
        np.testing.assert_allclose(Y[i], per_p[prec[i]][i], rtol=0, atol=1e-12)
    for p in range(1, 4):
        slice_p = torch.from_numpy(O.slice_matrix(codes, s0, z0, p))
        np.testing.assert_allclose(per_p[p] - per_p[p - 1], (X @ slice_p.T).numpy(), rtol=0, atol=1e-11)
    assert O.linear(xb[:0], codes, s0, z0, prec[:0]).shape == (0, 24)


# --------------------------------------------------- the pins do catch planted mistakes
@pytest.mark.parametrize("mistake", ["drop_half", "residual_zero", "scale_ratio"])
def test_pins_detect_planted_mistakes(monkeypatch, mistake):
    import oracle.mbq_oracle as M

    if mistake == "drop_half":
        real = M.slice_matrix

        def broken(codes, s0, z0, e):
            s_e = np.repeat(s0.astype(np.float64), 128, axis=1) / 4.0 ** e
            return real(codes, s0, z0, e) - 0.5 * s_e

        monkeypatch.setattr(M, "slice_matrix", broken)
    elif mistake == "residual_zero":
        monkeypatch.setattr(M, "RESIDUAL_ZERO", 1.5)
    else:
        monkeypatch.setattr(M, "LEVELS", 2)      # the 2^{b_e - 1} wording of Sec. 4.1
    rows, _ = load_worked_example()
    W = worked_weight(rows)
    codes, s0, z0 = M.encode(W)
    bad = False
    for idx, _, want_codes, want_rec in rows:
        if [int(codes[e, 0, idx]) for e in range(4)] != want_codes:
            bad = True
        for p in range(4):
            if abs(M.dequant(codes, s0, z0, p)[0, idx] - want_rec[p]) > 1e-9:
                bad = True
    assert bad


# ------------------------------------------------------------- the paper's router (2-layer MLP + threshold)
def _mlp_case(T=9, K=128, H=6, seed=3):
    from workloads import make_mlp_router, make_tokens
    xb, _ = make_tokens(T, K, [seed, T], outlier_channel_frac=0.0)
    W1, b1, W2, b2 = make_mlp_router(K, H, [seed])
    return xb, W1, b1, W2, b2


def test_route_mlp_scores_against_fsum_loops():
    """Scores of the 2-layer router (Sec. 4.2 Eq. 4) against exactly rounded Python sums, ReLU written out."""
    xb, W1, b1, W2, b2 = _mlp_case()
    S, prec, margin = O.route_mlp(xb, W1, b1, W2, b2, delta=0.0)
    X = O.bf16_bits_to_f64(xb)
    for i in range(X.shape[0]):
        hidden = []
        for j in range(W1.shape[0]):
            a = math.fsum([float(X[i, k]) * float(W1[j, k]) for k in range(X.shape[1])] + [float(b1[j])])
            hidden.append(a if a > 0.0 else 0.0)
        for e in range(W2.shape[0]):
            want = math.fsum([hidden[j] * float(W2[e, j]) for j in range(len(hidden))] + [float(b2[e])])
            assert abs(S[i, e] - want) <= 1e-12 * max(1.0, abs(want))


def test_route_mlp_prefix_closure_all_patterns():
    """Every on/off pattern of the three residual slices (threshold gate of Sec. 4.2): the precision is the number
    of LEADING active residual slices; the base slice's own score never matters (shared-expert slice)."""
    K, H = 128, 3
    # a router whose scores are chosen directly: hidden unit j = relu(x_j) with x_j = 1, score_e = sum_j W2[e, j]
    xb = f32_to_bf16_bits(np.zeros((8, K), dtype=np.float32) + np.eye(8, K, dtype=np.float32)[:, :K] * 0)
    X = np.zeros((8, K), dtype=np.float32)
    X[:, 0] = 1.0
    xb = f32_to_bf16_bits(X)
    W1 = np.zeros((H, K), dtype=np.float32)
    W1[0, 0] = 1.0                                  # hidden = [1, 0, 0] for every token
    b1 = np.zeros(H, dtype=np.float32)
    expected = {(0, 0, 0): 0, (1, 0, 0): 1, (1, 1, 0): 2, (1, 1, 1): 3,
                (0, 1, 0): 0, (0, 1, 1): 0, (1, 0, 1): 1, (0, 0, 1): 0}
    for base_score in (-5.0, 5.0):                   # slice 0's score is ignored
        for pattern, want in expected.items():
            W2 = np.zeros((4, H), dtype=np.float32)
            b2 = np.array([base_score] + [1.0 if on else -1.0 for on in pattern], dtype=np.float32)
            S, prec, margin = O.route_mlp(xb, W1, b1, W2, b2, delta=0.25)
            assert (prec == want).all(), (pattern, prec)
            assert np.allclose(S[:, 1:], np.array(b2[1:], dtype=np.float64)[None, :])
    # the comparison is strict: a score equal to the threshold is inactive
    b2 = np.array([0.0, 0.25, 9.0, 9.0], dtype=np.float32)
    S, prec, margin = O.route_mlp(xb, W1, b1, np.zeros((4, H), dtype=np.float32), b2, delta=0.25)
    assert (prec == 0).all() and (margin == 0.0).all()


def test_route_mlp_threshold_is_monotone_and_switches_precision():
    """Raising delta never raises a token's precision (Sec. 4.2: a larger threshold activates fewer slices), and the
    two ends of the sweep are all-2-bit and (for scores that allow it) up to 8-bit."""
    xb, W1, b1, W2, b2 = _mlp_case(T=64, K=256, H=8, seed=5)
    prev = None
    avg = []
    for delta in [-1e3] + list(np.linspace(-6.0, 6.0, 25)) + [1e3]:
        S, prec, margin = O.route_mlp(xb, W1, b1, W2, b2, delta=float(delta))
        if prev is not None:
            assert (prec <= prev).all()
        prev = prec
        avg.append(O.avg_bits(prec))
    assert avg[0] == 8.0 and avg[-1] == 2.0 and all(a >= b for a, b in zip(avg, avg[1:]))


def test_threshold_quantile_against_sorted_brute_force():
    """Layer-wise threshold calibration (App. C.2): exactly round(rho M) residual scores exceed the threshold."""
    rng = np.random.default_rng(11)
    S = rng.standard_normal((257, 4))
    M = 257 * 3
    for rho in (0.0, 1.0 / 6.0, 1.0 / 3.0, 0.5, 0.9, 1.0):
        d = O.threshold_quantile(S, rho)
        k = int(math.floor(rho * M + 0.5))
        assert int((S[:, 1:] - d > 0).sum()) == k
        if k < M:   # the threshold is itself one of the scores: the largest one that stays inactive
            resid = sorted(S[:, 1:].reshape(-1).tolist(), reverse=True)
            assert d == resid[k]
    # target bits -> ratio (App. C.2): rho = (target - 2) / 6; the realised average follows for independent slices only
    # when routing is a prefix, so only the activation count is pinned here


# ------------------------------------------------ encode with calibrated (external) base-slice parameters
def clipped_params(W, keep):
    """(s0, z0) of a range shrunk to `keep` of the group's min and max: what a learned clipping would hand over."""
    N, K = W.shape
    Wg = W.reshape(N, K // 128, 128)
    lo = (Wg.min(axis=2) * np.float32(keep)).astype(np.float32)
    hi = (Wg.max(axis=2) * np.float32(keep)).astype(np.float32)
    s0 = ((hi - lo) / np.float32(4.0)).astype(np.float32)
    z0 = ((-lo) / s0).astype(np.float32)
    return s0, z0


@pytest.mark.parametrize("keep", [0.6, 0.9])
def test_external_parameters_saturate_outside_and_bound_inside(keep):
    """Paper App. B: the quantiser clamps, so with a clipped range (Sec. 4.1: (s0, z0) are calibrated, not fitted)
    a weight outside the range gets code 0 (or 3) in EVERY slice and reconstructs to the centre of the lowest
    (highest) bin of the precision, lo + s_p/2 (hi - s_p/2); a weight inside keeps the half-step bound; and the
    sliced code still equals the single-shot floor quantiser with (s0/4^p, 4^p z0)."""
    W = student_matrix(seed=23)
    s0, z0 = clipped_params(W, keep)
    codes, s0_out, z0_out = O.encode(W, s0, z0)
    assert np.array_equal(s0_out, s0) and np.array_equal(z0_out, z0)        # stored as given
    S = np.repeat(s0.astype(np.float64), 128, axis=1)
    Z = np.repeat(z0.astype(np.float64), 128, axis=1)
    lo = -Z * S
    hi = lo + 4.0 * S
    Wd = W.astype(np.float64)
    below, above = Wd < lo - 1e-9 * S, Wd >= hi + 1e-9 * S
    inside = (Wd > lo + 1e-9 * S) & (Wd < hi - 1e-9 * S)
    assert below.sum() > 50 and above.sum() > 50 and inside.sum() > 1000      # the clip really cuts both tails
    for e in range(4):
        assert np.all(codes[e][below] == 0) and np.all(codes[e][above] == 3)
    for p in range(4):
        sp = S / 4 ** p
        What = O.dequant(codes, s0, z0, p)
        np.testing.assert_allclose(What[below], (lo + sp / 2)[below], rtol=0, atol=1e-12)
        np.testing.assert_allclose(What[above], (hi - sp / 2)[above], rtol=0, atol=1e-12)
        assert np.all(np.abs(Wd - What)[inside] <= (sp / 2 + 1e-12)[inside])
        q, deq = uniform_floor_quantiser(Wd, sp, Z * 4 ** p, 2 * (p + 1))
        frac = (Wd / sp + Z * 4 ** p) % 1.0
        edge = np.minimum(frac, 1 - frac) < 1e-9
        assert np.all((q == O.merged_code(codes, p)) | edge)


def test_external_parameters_equal_to_the_fit_change_nothing():
    W = student_matrix(seed=29)
    codes, s0, z0 = O.encode(W)
    codes2, _, _ = O.encode(W, s0, z0)
    assert np.array_equal(codes, codes2)
