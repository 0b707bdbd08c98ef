"""Pins of the C oracle (oracle/mbq_oracle.c, the one the CPU baseline times): the hand-worked example of
tests/golden/worked_example.txt (codes, base-slice parameters, routed output at every precision), a stable library sort,
`math.fsum` logits, and agreement with the numpy oracle (bit for bit where the result is an integer or an fp32 value)."""
import math
import os

import numpy as np
import pytest

import oracle as O
from oracle import c_oracle as C
from test_oracle_pins import load_worked_example, worked_weight
from workloads import f32_to_bf16_bits, make_router, make_tokens, make_weight


@pytest.fixture(scope="module", autouse=True)
def built():
    from oracle import build as b

    b.build()          # compiles every time, like the HIP library's build()
    assert os.path.exists(b.LIB)


def test_worked_example_codes_parameters_and_routed_output():
    rows, ys = load_worked_example()
    W = worked_weight(rows)
    codes, s0, z0 = C.encode(W)
    assert s0[0, 0] == 1.0 and z0[0, 0] == 1.0
    for idx, _, want_codes, _ in rows:
        assert [int(codes[e, 0, idx]) for e in range(4)] == want_codes
    x = np.zeros((1, 128), dtype=np.float32)
    x[0, 0], x[0, 2] = 1.0, 2.0
    xb = f32_to_bf16_bits(x)
    for p, want in ys:
        y = C.linear(xb, codes, s0, z0, np.array([p], dtype=np.int32))
        assert y.shape == (1, 1) and y[0, 0] == want        # dyadic values: exact


def test_route_matches_exact_sums_and_tie_rule():
    K, T = 384, 9
    Wr, br = make_router(K, [11], mix=None)
    xb, _ = make_tokens(T, K, [11, T], outlier_channel_frac=0.01)
    xb[3] = xb[2]                                            # two equal tokens: equal choices
    S, prec, gap = C.route(xb, Wr, br)
    X = O.bf16_bits_to_f64(xb)
    for i in range(T):
        want = [math.fsum(float(X[i, k]) * float(Wr[q, k]) for k in range(K)) + float(br[q]) for q in range(4)]
        assert np.allclose(S[i], want, rtol=0, atol=1e-12)
        assert prec[i] == int(np.argmax(S[i]))               # numpy's argmax: first maximum
        top = sorted(S[i])
        assert gap[i] == top[-1] - top[-2]
    assert prec[2] == prec[3]
    Wt = np.zeros((4, K), dtype=np.float32)                  # all logits equal: the first precision wins
    _, p0, g0 = C.route(xb, Wt, np.zeros(4, dtype=np.float32))
    assert np.all(p0 == 0) and np.all(g0 == 0.0)


def test_bucket_is_a_stable_sort():
    rng = np.random.default_rng(5)
    for T in (0, 1, 7, 300):
        prec = rng.integers(0, 4, size=T).astype(np.int32)
        perm, offsets = C.bucket(prec)
        assert np.array_equal(perm, np.argsort(prec, kind="stable").astype(np.int32))
        assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(np.bincount(prec, minlength=4))]))


@pytest.mark.parametrize("N,K,T", [(16, 256, 1), (40, 384, 5), (130, 1280, 33)])
def test_agrees_with_the_numpy_oracle(N, K, T):
    W = make_weight(N, K, [N, K], 4.0)
    W[3, :128] = 0.25                                        # a constant group: the range floor
    Wr, br = make_router(K, [N], mix=None)
    xb, _ = make_tokens(T, K, [N, T], outlier_channel_frac=0.01)
    c1, s1, z1 = O.encode(W)
    c2, s2, z2 = C.encode(W)
    assert np.array_equal(c1, c2) and np.array_equal(s1, s2) and np.array_equal(z1, z2)
    S1, p1, g1 = O.route(xb, Wr, br)
    S2, p2, g2 = C.route(xb, Wr, br)
    assert np.allclose(S1, S2, rtol=0, atol=1e-12) and np.array_equal(p1, p2)
    for a, b in zip(O.bucket(p1), C.bucket(p1)):
        assert np.array_equal(a, b)
    Y1 = O.linear(xb, c1, s1, z1, p1)
    Y2 = C.linear(xb, c1, s1, z1, p1)
    assert np.linalg.norm(Y1 - Y2) <= 1e-12 * np.linalg.norm(Y1)
    # threads only split rows: one thread gives the same bits
    threads = C.max_threads()
    C.set_threads(1)
    Y3 = C.linear(xb, c1, s1, z1, p1)
    C.set_threads(threads)
    assert np.array_equal(Y2, Y3)
