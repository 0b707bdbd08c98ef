"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same
seeded inputs, at sizes the oracle finishes in seconds.  Codes, blob bytes, routing and
permutation are compared bit for bit; outputs within the floating-point bar."""
import numpy as np
import pytest
import torch

import oracle as O
from helpers import (MAX_ABS_TOL, assert_output_close, check_bucket, compare_routing, dev, dev_bf16)
from workloads import CONFIGS, f32_to_bf16_bits, make_case, make_weight

pytestmark = pytest.mark.gpu


def tokens(T, K, seed, scale_channels=True):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, K)).astype(np.float32)
    if scale_channels and K >= 256:
        x[:, rng.choice(K, size=max(1, K // 100), replace=False)] *= 20.0
    return f32_to_bf16_bits(x)


# ----------------------------------------------------------------------------- encode
@pytest.mark.parametrize("N,K", [(16, 256), (3, 128), (40, 384), (130, 1280), (2048, 2048)])
def test_encode_blob_is_bit_exact(mbq, N, K):
    print(f"[case] encode N={N} K={K}", flush=True)
    W = make_weight(N, K, [7, N, K], 4.0)
    if N >= 40:
        W[1, :128] = 0.0                # an all-zero group
        W[2, 128:256] = 0.3125          # a constant group
    codes, s0, z0 = O.encode(W)
    blob = mbq.mbq_encode(dev(W))
    torch.cuda.synchronize()
    got = blob.cpu().numpy()
    want = O.pack_blob(codes, s0, z0)
    assert got.size == want.size
    assert np.array_equal(got, want)
    c, s, z = mbq.mbq_unpack(blob, N, K)
    assert np.array_equal(c.cpu().numpy(), codes)
    assert np.array_equal(s.cpu().numpy(), s0) and np.array_equal(z.cpu().numpy(), z0)
    for p in range(4):
        What = mbq.mbq_dequant(blob, N, K, p).cpu().numpy().astype(np.float64)
        ref = O.dequant(codes, s0, z0, p)
        np.testing.assert_allclose(What, ref, rtol=2e-7, atol=1e-12)


@pytest.mark.parametrize("N,K,keep", [(3, 128, 0.7), (130, 1280, 0.6), (272, 4096, 0.9)])
def test_encode_with_external_parameters(mbq, N, K, keep):
    """Calibrated (clipped) base-slice parameters handed in: blob bit-exact with the oracle's, weights outside the range
    saturated, and the routed linear over such a blob within tolerance of the oracle's."""
    print(f"[case] encode with params N={N} K={K} keep={keep}", flush=True)
    W = make_weight(N, K, [53, N, K], 4.0)
    Wg = W.reshape(N, K // 128, 128)
    lo = (Wg.min(axis=2) * np.float32(keep)).astype(np.float32)
    hi = (Wg.max(axis=2) * np.float32(keep)).astype(np.float32)
    s0 = ((hi - lo) / np.float32(4.0)).astype(np.float32)
    z0 = ((-lo) / s0).astype(np.float32)
    codes, _, _ = O.encode(W, s0, z0)
    blob = mbq.mbq_encode_with_params(dev(W), dev(s0), dev(z0))
    torch.cuda.synchronize()
    assert np.array_equal(blob.cpu().numpy(), O.pack_blob(codes, s0, z0))
    c, s, z = mbq.mbq_unpack(blob, N, K)
    assert np.array_equal(c.cpu().numpy(), codes)
    assert np.array_equal(s.cpu().numpy(), s0) and np.array_equal(z.cpu().numpy(), z0)
    T = 16
    xb = tokens(T, K, [N, K, 59])
    prec = np.random.default_rng([N, K]).integers(0, 4, size=T).astype(np.int32)
    perm, offsets = O.bucket(prec)
    Y = mbq.mbq_linear(dev_bf16(xb).reshape(T, K), blob, N, K, dev(prec), dev(perm), dev(offsets))
    assert_output_close(Y.cpu().numpy(), O.linear(xb, codes, s0, z0, prec), f"linear over clipped blob N={N} K={K}")


@pytest.mark.parametrize("meta", ["float16", "bfloat16"])
def test_sixteen_bit_parameter_values_through_external_parameters(mbq, meta):
    """App. C.1's pipeline may keep the per-group scale and zero point in 16 bits.  The blob stores fp32 pairs, but the
    NUMBERS of such a setting pass through unchanged: parameters rounded to fp16 / bf16 before they are handed in give
    the oracle's codes for exactly those parameters, and every stored value is a 16-bit number."""
    N, K, T = 70, 1024, 16
    print(f"[case] encode with {meta} parameter values N={N} K={K}", flush=True)
    W = make_weight(N, K, [57, N, K], 4.0)
    _, s_fit, z_fit = O.encode(W)
    if meta == "float16":
        s0, z0 = s_fit.astype(np.float16).astype(np.float32), z_fit.astype(np.float16).astype(np.float32)
    else:
        def to_bf16(a):
            u = a.view(np.uint32).astype(np.uint64)
            u = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
            return u.astype(np.uint32).view(np.float32)
        s0, z0 = to_bf16(s_fit), to_bf16(z_fit)
    codes, _, _ = O.encode(W, s0, z0)
    blob = mbq.mbq_encode_with_params(dev(W), dev(s0), dev(z0))
    torch.cuda.synchronize()
    assert np.array_equal(blob.cpu().numpy(), O.pack_blob(codes, s0, z0))
    c, s, z = mbq.mbq_unpack(blob, N, K)
    assert np.array_equal(s.cpu().numpy(), s0) and np.array_equal(z.cpu().numpy(), z0)
    xb = tokens(T, K, [N, K, 61])
    prec = np.random.default_rng([N, K, 3]).integers(0, 4, size=T).astype(np.int32)
    perm, offsets = O.bucket(prec)
    Y = mbq.mbq_linear(dev_bf16(xb).reshape(T, K), blob, N, K, dev(prec), dev(perm), dev(offsets))
    assert_output_close(Y.cpu().numpy(), O.linear(xb, codes, s0, z0, prec), f"linear, {meta} parameter values")


# ------------------------------------------------------------------------------ route
@pytest.mark.parametrize("T,K", [(0, 256), (1, 128), (5, 384), (16, 4096), (16, 11008), (28, 8192), (29, 8320),
                                 (32, 2048), (64, 4096), (65, 1024), (100, 2304), (128, 4096), (129, 512), (1023, 256), (1024, 256), (1025, 256),
                                 (4100, 512)])
def test_route_and_bucket_are_bit_exact(mbq, T, K):
    print(f"[case] route T={T} K={K}", flush=True)
    rng = np.random.default_rng([T, K])
    xb = tokens(T, K, [T, K, 1])
    Wr = (rng.standard_normal((4, K)) / np.sqrt(K)).astype(np.float32)
    br = np.array([0.3, 0.1, -0.1, -0.4], dtype=np.float32)
    S, prec_ref, gap = O.route(xb, Wr, br)
    prec, perm, offsets, logits = mbq.mbq_route(dev_bf16(xb).reshape(T, K), dev(Wr), dev(br), want_logits=True)
    torch.cuda.synchronize()
    prec, perm, offsets = prec.cpu().numpy(), perm.cpu().numpy(), offsets.cpu().numpy()
    if T:
        np.testing.assert_allclose(logits.cpu().numpy(), S, rtol=0, atol=1e-10)
    compare_routing(prec, prec_ref, gap, f"route T={T} K={K}")
    check_bucket(prec, perm, offsets)          # permutation of the GPU's own choices: unique answer
    assert offsets[4] == T


# ------------------------------------------------------------- the paper's router (2-layer MLP + threshold)
@pytest.mark.parametrize("T,K,H", [(0, 256, 8), (1, 128, 1), (16, 4096, 64), (37, 384, 13), (513, 512, 32),
                                   (2048, 1024, 64), (300, 256, 512), (290, 384, 21)])
def test_route_mlp_matches_oracle(mbq, T, K, H):
    """Scores to fp64 rounding, precisions bit-exact away from the threshold, permutation exact; a sweep of the
    threshold over one set of parameters switches precisions without touching anything else."""
    from workloads import make_mlp_router
    print(f"[case] route_mlp T={T} K={K} H={H}", flush=True)
    xb = tokens(T, K, [T, K, H])
    W1, b1, W2, b2 = make_mlp_router(K, H, [T, K, H])
    X = dev_bf16(xb).reshape(T, K)
    d = [dev(a) for a in (W1, b1, W2, b2)]
    avgs = []
    for delta in (-1e3, -0.75, 0.0, 0.4, 1e3):
        S, prec_ref, margin = O.route_mlp(xb, W1, b1, W2, b2, delta)
        prec, perm, offsets, scores = mbq.mbq_route_mlp(X, *d, delta, want_scores=True)
        torch.cuda.synchronize()
        prec, perm, offsets = prec.cpu().numpy(), perm.cpu().numpy(), offsets.cpu().numpy()
        if T:
            np.testing.assert_allclose(scores.cpu().numpy(), S, rtol=0, atol=1e-10)
        compare_routing(prec, prec_ref, margin, f"route_mlp T={T} K={K} H={H} delta={delta}")
        check_bucket(prec, perm, offsets)
        assert offsets[4] == T
        avgs.append(O.avg_bits(prec))
    if T:
        assert avgs[0] == 8.0 and avgs[-1] == 2.0 and all(a >= b for a, b in zip(avgs, avgs[1:]))


def test_threshold_quantile_is_exact(mbq):
    """The calibration quantile is an order statistic: fed the oracle's scores it must return the same double."""
    rng = np.random.default_rng(23)
    S = rng.standard_normal((1000, 4)) * 3.0
    S[5, 1] = S[9, 2]                      # a tie among the residual scores
    Sd = dev(S)
    for rho in (0.0, 1.0 / 6.0, 1.0 / 3.0, 0.5, 0.77, 1.0):
        want = O.threshold_quantile(S, rho)
        got = float(mbq.mbq_threshold_quantile(Sd, rho).cpu().numpy()[0])
        assert got == want, (rho, got, want)
    with pytest.raises(mbq.MbqError):
        mbq.mbq_threshold_quantile(Sd, 1.5)


def test_route_mlp_target_bits_and_linear(mbq):
    """Layer-wise calibration end to end (App. C.2): scores of a calibration batch -> threshold for a target of
    4 average bits -> routing of a fresh batch -> routed linear against the oracle with the same routing."""
    from workloads import make_mlp_router
    N, K, H, T = 272, 512, 16, 200
    W = make_weight(N, K, [29], 4.0)
    W1, b1, W2, b2 = make_mlp_router(K, H, [29])
    d = [dev(a) for a in (W1, b1, W2, b2)]
    cal = tokens(4096, K, [29, 1])
    *_, cal_scores = mbq.mbq_route_mlp(dev_bf16(cal).reshape(-1, K), *d, 0.0, want_scores=True)
    rho = (4.0 - 2.0) / 6.0
    delta = float(mbq.mbq_threshold_quantile(cal_scores, rho).cpu().numpy()[0])
    S_cal, _, _ = O.route_mlp(cal, W1, b1, W2, b2, 0.0)
    active = float(np.mean(S_cal[:, 1:] - delta > 0))
    assert abs(active - rho) < 2e-3                       # the requested fraction of residual slices is active
    xb = tokens(T, K, [29, 2])
    X = dev_bf16(xb).reshape(T, K)
    prec, perm, offsets = mbq.mbq_route_mlp(X, *d, delta)
    S, prec_ref, margin = O.route_mlp(xb, W1, b1, W2, b2, delta)
    compare_routing(prec.cpu().numpy(), prec_ref, margin, "route_mlp calibrated")
    blob = mbq.mbq_encode(dev(W))
    codes, s0, z0 = O.encode(W)
    for algo in (1, 3):
        Y = mbq.mbq_linear(X, blob, N, K, prec, perm, offsets, algo=algo)
        assert_output_close(Y.cpu().numpy(), O.linear(xb, codes, s0, z0, prec.cpu().numpy()), f"mlp-routed linear algo={algo}")


@pytest.mark.parametrize("T,K,n", [(1, 4096, 3), (16, 4096, 3), (28, 1280, 4), (16, 11008, 1), (40, 512, 2), (97, 4096, 2), (128, 1024, 3), (130, 512, 2),
                                   (0, 256, 2)])
def test_route_group_equals_separate_calls(mbq, T, K, n):
    """Several routers over one X: against the oracle, and bit for bit against mbq_route; called
    twice on one workspace that starts out full of ones (the call clears its counters itself)."""
    print(f"[case] route group T={T} K={K} n={n}", flush=True)
    rng = np.random.default_rng([T, K, n])
    xb = tokens(T, K, [T, K, 2])
    X = dev_bf16(xb).reshape(T, K)
    Wrs = [(rng.standard_normal((4, K)) / np.sqrt(K)).astype(np.float32) for _ in range(n)]
    brs = [rng.normal(0, 0.2, size=4).astype(np.float32) for _ in range(n)]
    ws = mbq.route_workspace(T, K, "cuda").fill_(0xFF)
    for _ in range(2):
        outs = mbq.mbq_route_group(X, [dev(w) for w in Wrs], [dev(b) for b in brs], ws=ws)
        torch.cuda.synchronize()
        for i in range(n):
            S, prec_ref, gap = O.route(xb, Wrs[i], brs[i])
            prec, perm, offsets = (t.cpu().numpy() for t in outs[i])
            compare_routing(prec, prec_ref, gap, f"group router {i}")
            check_bucket(prec, perm, offsets)
            single = mbq.mbq_route(X, dev(Wrs[i]), dev(brs[i]))
            for a, b in zip(single, outs[i]):
                assert torch.equal(a, b)


@pytest.mark.parametrize("T", [1, 16, 28, 29, 128, 129, 700])
def test_route_workspace_contents_do_not_matter(mbq, T):
    """A workspace left in any state (say by a call that was cut short) gives the same routing as a clean one,
    for the linear router, the 2-layer router and the routed stage."""
    from workloads import make_mlp_router
    K, H, N = 512, 16, 64
    print(f"[case] dirty route workspace T={T}", flush=True)
    rng = np.random.default_rng([T, 91])
    xb = tokens(T, K, [T, 91])
    X = dev_bf16(xb).reshape(T, K)
    Wr = dev((rng.standard_normal((4, K)) / np.sqrt(K)).astype(np.float32))
    br = dev(rng.normal(0, 0.2, size=4).astype(np.float32))
    clean = mbq.mbq_route(X, Wr, br, ws=mbq.route_workspace(T, K, "cuda").zero_())
    for fill in (0xFF, 0x01, 0x80):
        dirty = mbq.mbq_route(X, Wr, br, ws=mbq.route_workspace(T, K, "cuda").fill_(fill))
        torch.cuda.synchronize()
        for a, b in zip(clean, dirty):
            assert torch.equal(a, b), (T, fill)
    m = [dev(a) for a in make_mlp_router(K, H, [T, 92])]
    clean = mbq.mbq_route_mlp(X, *m, 0.1, ws=mbq.route_mlp_workspace(T, K, H, "cuda").zero_())
    dirty = mbq.mbq_route_mlp(X, *m, 0.1, ws=mbq.route_mlp_workspace(T, K, H, "cuda").fill_(0xFF))
    torch.cuda.synchronize()
    for a, b in zip(clean, dirty):
        assert torch.equal(a, b), T
    blob = mbq.mbq_encode(dev(make_weight(N, K, [T, 93])))
    outs = []
    for fill in (0x00, 0xFF):
        ws = mbq.route_workspace(T, K, "cuda").fill_(fill)
        outs.append(mbq.mbq_routed_linear_group(X, [Wr], [br], [blob], [N], ws_route=ws))
        torch.cuda.synchronize()
    for a, b in zip(outs[0][0][0] + (outs[0][1][0],), outs[1][0][0] + (outs[1][1][0],)):
        assert torch.equal(a, b), T


def test_route_small_and_general_kernels_agree(mbq):
    T, K = 16, 4096
    xb = tokens(T, K, 77)
    rng = np.random.default_rng(77)
    Wr = (rng.standard_normal((4, K)) / np.sqrt(K)).astype(np.float32)
    br = np.zeros(4, dtype=np.float32)
    a = mbq.mbq_route(dev_bf16(xb), dev(Wr), dev(br), want_logits=True)
    mbq.set_knob(4, 1)
    try:
        b = mbq.mbq_route(dev_bf16(xb), dev(Wr), dev(br), want_logits=True)
    finally:
        mbq.set_knob(4, 0)
    for u, v in zip(a[:3], b[:3]):
        assert torch.equal(u, v)
    np.testing.assert_allclose(a[3].cpu().numpy(), b[3].cpu().numpy(), rtol=0, atol=1e-10)


def test_route_ties_and_single_bucket(mbq):
    T, K = 70, 256
    xb = tokens(T, K, 3)
    Wr = np.zeros((4, K), dtype=np.float32)
    br = np.zeros(4, dtype=np.float32)            # every logit ties: first index wins
    prec, perm, offsets = mbq.mbq_route(dev_bf16(xb), dev(Wr), dev(br))
    assert prec.cpu().numpy().tolist() == [0] * T
    assert offsets.cpu().numpy().tolist() == [0, T, T, T, T]
    assert perm.cpu().numpy().tolist() == list(range(T))
    br[2] = 1.0
    prec, perm, offsets = mbq.mbq_route(dev_bf16(xb), dev(Wr), dev(br))
    assert prec.cpu().numpy().tolist() == [2] * T
    assert offsets.cpu().numpy().tolist() == [0, 0, 0, T, T]


# ----------------------------------------------------------------------------- linear
def run_linear(mbq, W, xb, prec, algo):
    N, K = W.shape
    T = xb.shape[0]
    blob = mbq.mbq_encode(dev(W))
    perm, offsets = O.bucket(prec)
    Y = mbq.mbq_linear(dev_bf16(xb).reshape(T, K), blob, N, K, dev(prec.astype(np.int32)), dev(perm),
                       dev(offsets), algo=algo)
    torch.cuda.synchronize()
    return Y.cpu().numpy()


ALGOS = {"simple": 1, "decode": 2, "prefill": 3}


@pytest.mark.parametrize("algo", ["simple", "decode", "prefill"])
@pytest.mark.parametrize("N,K,T", [(16, 256, 1), (40, 384, 5), (130, 1280, 16), (272, 512, 33), (64, 2048, 64)])
def test_linear_small_shapes(mbq, algo, N, K, T):
    print(f"[case] linear {algo} N={N} K={K} T={T}", flush=True)
    W = make_weight(N, K, [11, N, K], 4.0)
    xb = tokens(T, K, [N, K, T])
    prec = np.random.default_rng([N, T]).integers(0, 4, size=T).astype(np.int32)
    codes, s0, z0 = O.encode(W)
    Yref = O.linear(xb, codes, s0, z0, prec)
    Y = run_linear(mbq, W, xb, prec, ALGOS[algo])
    assert_output_close(Y, Yref, f"{algo} N={N} K={K} T={T}")


@pytest.mark.parametrize("algo", ["decode", "prefill"])
@pytest.mark.parametrize("p", [0, 1, 2, 3])
def test_linear_single_precision_is_a_dense_gemm(mbq, algo, p):
    """All tokens at one precision: three empty buckets; equals X What^T (dense library matmul)."""
    N, K, T = 96, 768, 16 if algo == "decode" else 150
    print(f"[case] linear {algo} uniform p={p}", flush=True)
    W = make_weight(N, K, [13, p], 4.0)
    xb = tokens(T, K, [p, 5])
    prec = np.full(T, p, dtype=np.int32)
    codes, s0, z0 = O.encode(W)
    dense = torch.from_numpy(O.bf16_bits_to_f64(xb)) @ torch.from_numpy(O.dequant_merged(codes, s0, z0, p)).T
    Y = run_linear(mbq, W, xb, prec, ALGOS[algo])
    assert_output_close(Y, dense.numpy(), f"{algo} uniform p={p}")


@pytest.mark.parametrize("N,K,T,mix", [
    (300, 128, 70, None),            # one group (no rescale), N not a multiple of 16 or 256, one ragged tile per bucket
    (520, 1152, 513, None),          # odd group count (tail pairs end on a single group), three column tiles
    (272, 512, 300, (0.9, 0.1, 0.0, 0.0)),   # one full 256-row tile plus ragged rest in bucket 0, an empty bucket
    (256, 768, 600, (0.0, 0.0, 0.5, 0.5)),   # full tiles at precisions 2 and 3 (8-bit operand path)
])
def test_prefill_tile_shapes(mbq, N, K, T, mix):
    """Full and ragged 256-row tiles, group-boundary rescale, the fp32 zero-point tail, column padding."""
    print(f"[case] prefill tiles N={N} K={K} T={T} mix={mix}", flush=True)
    W = make_weight(N, K, [17, N, K], 4.0)
    xb = tokens(T, K, [N, K, T, 1])
    rng = np.random.default_rng([N, T, 3])
    prec = (rng.integers(0, 4, size=T) if mix is None else rng.choice(4, size=T, p=mix)).astype(np.int32)
    codes, s0, z0 = O.encode(W)
    Yref = O.linear(xb, codes, s0, z0, prec)
    Y = run_linear(mbq, W, xb, prec, ALGOS["prefill"])
    assert_output_close(Y, Yref, f"prefill N={N} K={K} T={T}")


@pytest.mark.parametrize("splits", [2, 3, 4, 7])
def test_prefill_k_split(mbq, splits):
    """The K range of a tile cut into workgroups that add their partial sums into a zeroed Y."""
    N, K, T = 272, 2304, 300     # 18 groups: uneven split ranges
    print(f"[case] prefill K split {splits}", flush=True)
    W = make_weight(N, K, [19, splits], 4.0)
    xb = tokens(T, K, [N, K, T, 2])
    prec = np.random.default_rng([splits, 5]).integers(0, 4, size=T).astype(np.int32)
    codes, s0, z0 = O.encode(W)
    Yref = O.linear(xb, codes, s0, z0, prec)
    mbq.set_knob(5, splits)
    try:
        Y = run_linear(mbq, W, xb, prec, ALGOS["prefill"])
    finally:
        mbq.set_knob(5, 0)
    assert_output_close(Y, Yref, f"prefill K split {splits}")


@pytest.mark.parametrize("K", [768, 2048, 4096, 5120, 11008])
@pytest.mark.parametrize("pmax", [0, 1, 2, 3])
@pytest.mark.parametrize("T", [7, 16, 40])
def test_decode_every_highest_precision(mbq, K, pmax, T):
    """The decode kernels are specialised on the highest precision present and on the number of
    column blocks (4, 8 or 16 wavefronts, one or several K chunks): cover every combination."""
    N = 80
    print(f"[case] decode pmax={pmax} K={K} T={T}", flush=True)
    W = make_weight(N, K, [19, K], 4.0)
    xb = tokens(T, K, [K, pmax, T])
    prec = np.random.default_rng([K, pmax, T]).integers(0, pmax + 1, size=T).astype(np.int32)
    prec[T // 2] = pmax
    codes, s0, z0 = O.encode(W)
    Yref = O.linear(xb, codes, s0, z0, prec)
    Y = run_linear(mbq, W, xb, prec, ALGOS["decode"])
    assert_output_close(Y, Yref, f"decode pmax={pmax} K={K} T={T}")


@pytest.mark.parametrize("K,N,T,pmax", [(8448, 80, 16, 3), (11008, 272, 16, 3), (11008, 4096, 13, 2), (14336, 130, 1, 3),
                                        (16384, 64, 16, 1), (9216, 2064, 7, 3), (12288, 16, 16, 0), (16384, 16500, 5, 3)])
def test_decode_one_token_tile_long_rows(mbq, K, N, T, pmax):
    """8192 < K <= 16384 at up to 16 tokens: the loader kernel works through each of its two parts in two chunks and
    keeps the tiles' sums of the first chunk in LDS (few enough tiles per workgroup), else the kernel that streams the
    activations with the weights takes over (the last case: 1032 row tiles); outputs also identical from call to call."""
    print(f"[case] decode long rows K={K} N={N} T={T} pmax={pmax}", flush=True)
    W = make_weight(N, K, [53, N, K], 4.0)
    xb = tokens(T, K, [K, N, T])
    prec = np.random.default_rng([K, N, T]).integers(0, pmax + 1, size=T).astype(np.int32)
    prec[T // 2] = pmax
    blob = mbq.mbq_encode(dev(W))
    perm, offsets = O.bucket(prec)
    X = dev_bf16(xb).reshape(T, K)
    args = (X, blob, N, K, dev(prec), dev(perm), dev(offsets))
    Y = mbq.mbq_linear(*args, algo=ALGOS["decode"])
    Y2 = mbq.mbq_linear(*args, algo=ALGOS["decode"])
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2)
    rows = np.arange(N) if N <= 4096 else np.random.default_rng(3).choice(N, 2048, replace=False)
    codes, s0, z0 = O.encode(W[rows])
    assert_output_close(Y.cpu().numpy()[:, rows], O.linear(xb, codes, s0, z0, prec), f"long rows K={K} N={N} T={T}")


@pytest.mark.parametrize("T,K,N", [(17, 4096, 130), (31, 2304, 48), (32, 4096, 64), (33, 1024, 272), (48, 4096, 40),
                                   (49, 2048, 130), (64, 4096, 2064), (64, 256, 16)])
def test_decode_several_token_tiles(mbq, T, K, N):
    """17..64 tokens: one pass over the weights per 16 precision-sorted tokens, each reading the slices of
    ITS highest precision; mixes chosen so that the passes differ."""
    print(f"[case] decode token tiles T={T} K={K} N={N}", flush=True)
    W = make_weight(N, K, [37, N, K], 4.0)
    xb = tokens(T, K, [T, K, 41])
    rng = np.random.default_rng([T, K, N])
    prec = rng.integers(0, 4, size=T).astype(np.int32)
    prec[:32] = np.minimum(prec[:32], 2)      # first window: at most 6 bits
    prec[5] = 2
    if T > 40:
        prec[40] = 3
    codes, s0, z0 = O.encode(W)
    Yref = O.linear(xb, codes, s0, z0, prec)
    Y = run_linear(mbq, W, xb, prec, ALGOS["decode"])
    assert_output_close(Y, Yref, f"decode token tiles T={T} K={K} N={N}")


@pytest.mark.parametrize("K,T,Ns", [(4096, 16, (96, 32, 130)), (4096, 1, (64, 64)), (2048, 7, (80, 48, 16, 33)),
                                    (768, 16, (40,)), (3072, 5, (48, 96)), (5120, 16, (48, 32)), (1024, 40, (48, 32)),
                                    (4096, 64, (1040, 130, 256)), (2304, 33, (272, 48, 16, 640)), (4352, 48, (2064, 16))])
def test_linear_group_equals_separate_calls(mbq, K, T, Ns):
    """Several matrices over one X, each with its own routing: against the oracle and bit for bit
    against mbq_linear (17..64 tokens: one launch of the register-stationary kernel for all matrices when
    each would take it, else per-matrix kernels inside the group call - the last shape)."""
    print(f"[case] linear group K={K} T={T} Ns={Ns}", flush=True)
    xb = tokens(T, K, [K, T, 9])
    X = dev_bf16(xb).reshape(T, K)
    blobs, routing, refs = [], [], []
    for i, N in enumerate(Ns):
        W = make_weight(N, K, [23, N, K, i], 4.0)
        codes, s0, z0 = O.encode(W)
        rng = np.random.default_rng([K, T, i])
        prec = rng.integers(0, (i % 4) + 1 if i else 4, size=T).astype(np.int32)   # different highest precisions
        perm, offsets = O.bucket(prec)
        blobs.append(mbq.mbq_encode(dev(W)))
        routing.append((dev(prec), dev(perm), dev(offsets)))
        refs.append(O.linear(xb, codes, s0, z0, prec))
    Ys = mbq.mbq_linear_group(X, blobs, list(Ns), K, routing)
    torch.cuda.synchronize()
    for i, N in enumerate(Ns):
        assert_output_close(Ys[i].cpu().numpy(), refs[i], f"group matrix {i}")
        single = mbq.mbq_linear(X, blobs[i], N, K, *routing[i])
        assert torch.equal(single, Ys[i])


@pytest.mark.parametrize("K,T,Ns", [(4096, 16, (96, 32, 130)), (2048, 1, (64, 48)), (1280, 9, (40,)), (5120, 16, (48, 32)),
                                    (1024, 40, (48, 32)),
                                    # 29..64 tokens: the linear launch sorts the tokens; last shape: one matrix takes
                                    # another kernel, so the stage falls back to the two calls
                                    (4096, 64, (1040, 130)), (2304, 33, (272, 48, 16)), (512, 17, (40,)), (4352, 48, (2064, 16)),
                                    # 65..128 tokens under the automatic choice: the same path, two tokens per sorting lane
                                    (4096, 65, (272, 130)), (2304, 128, (1040, 48, 16)), (1024, 100, (40, 300)),
                                    # many row tiles: the whole chip takes part, K in one part, two parts and streamed
                                    (1024, 5, (1024, 528)), (4096, 16, (1040, 512, 512)), (9216, 3, (1600,)), (2304, 16, (640, 130))])
def test_routed_linear_stage_equals_route_then_linear(mbq, K, T, Ns):
    """One block stage in one call: same routing and the same outputs, bit for bit, as mbq_route_group
    followed by mbq_linear_group, and within tolerance of the oracle; run twice on the same workspaces,
    which the calls must leave zeroed."""
    print(f"[case] stage K={K} T={T} Ns={Ns}", flush=True)
    rng = np.random.default_rng([K, T, len(Ns)])
    xb = tokens(T, K, [K, T, 31])
    X = dev_bf16(xb).reshape(T, K)
    Wrs = [(rng.standard_normal((4, K)) / np.sqrt(K)).astype(np.float32) for _ in Ns]
    brs = [rng.normal(0, 0.3, size=4).astype(np.float32) for _ in Ns]
    Ws = [make_weight(N, K, [29, N, K, i], 4.0) for i, N in enumerate(Ns)]
    blobs = [mbq.mbq_encode(dev(W)) for W in Ws]
    ws_r = mbq.route_workspace(T, K, "cuda").fill_(0xA5)
    ws_l = mbq.linear_workspace(T, max(Ns), K, "cuda")
    dWr, dbr = [dev(w) for w in Wrs], [dev(b) for b in brs]
    for _ in range(2):
        routing, Ys = mbq.mbq_routed_linear_group(X, dWr, dbr, blobs, list(Ns), ws_route=ws_r, ws_linear=ws_l)
        torch.cuda.synchronize()
        routing2 = mbq.mbq_route_group(X, dWr, dbr)
        Ys2 = mbq.mbq_linear_group(X, blobs, list(Ns), K, routing2)
        for i, N in enumerate(Ns):
            for a, b in zip(routing[i], routing2[i]):
                assert torch.equal(a, b)
            assert torch.equal(Ys[i], Ys2[i])
            S, prec_ref, gap = O.route(xb, Wrs[i], brs[i])
            prec = routing[i][0].cpu().numpy()
            compare_routing(prec, prec_ref, gap, f"stage router {i}")
            check_bucket(prec, routing[i][1].cpu().numpy(), routing[i][2].cpu().numpy())
            codes, s0, z0 = O.encode(Ws[i])
            assert_output_close(Ys[i].cpu().numpy(), O.linear(xb, codes, s0, z0, prec), f"stage matrix {i}")


@pytest.mark.parametrize("algo,T", [("decode", 12), ("decode", 40), ("prefill", 300)])
def test_linear_special_activation_rows(mbq, algo, T):
    """Rows that stress the activation handling: all zeros, all tiny (1e-30), one element 2^20 times the rest of
    its block, negative zeros, a constant row, an outlier in another 256-column block than the small values, bf16
    subnormals (alone in their block and next to normal values); every row is held to the bar on its own as well."""
    N, K = 130, 1280
    print(f"[case] special rows {algo} T={T}", flush=True)
    W = make_weight(N, K, [43, T], 4.0)
    rng = np.random.default_rng([43, T])
    x = rng.standard_normal((T, K)).astype(np.float32)
    x[0] = 0.0
    x[1] *= 1e-30
    x[2] *= 1e-3
    x[2, 300] = 1e3
    x[3, ::2] = -0.0
    x[4] = 0.75
    x[5] *= 1e-4
    x[5, 256:512] *= 1e8                      # block 1 of the row is 10^8 times its other blocks
    x[6] *= 1e-3
    x[6, :256] = rng.standard_normal(256) * 2.0 ** -130      # a block of subnormals only (bf16 keeps 2^-133)
    x[6, 600:640] = rng.standard_normal(40) * 2.0 ** -128    # subnormals among normal values
    x[7] = rng.standard_normal(K) * 2.0 ** -131               # a whole row of subnormals
    xb = f32_to_bf16_bits(x)
    assert (xb[7] & 0x7F80).max() == 0 and (xb[7] & 0x7F).max() > 0   # really subnormal, and not all zero
    prec = rng.integers(0, 4, size=T).astype(np.int32)
    prec[:8] = [3, 2, 3, 1, 0, 3, 3, 2]
    codes, s0, z0 = O.encode(W)
    Yref = O.linear(xb, codes, s0, z0, prec)
    Y = run_linear(mbq, W, xb, prec, ALGOS[algo])
    assert np.all(np.isfinite(Y))
    assert_output_close(Y, Yref, f"special rows {algo} T={T}")
    assert not Y[0].any(), "an all-zero token must give an all-zero output row"
    for i in range(1, 7):
        assert_output_close(Y[i:i + 1], Yref[i:i + 1], f"special row {i}")
    if algo == "decode" and T <= 16:
        # The two-FP8-piece split cannot scale a block below 2^-122 (the block scale is an 8-bit exponent and the
        # second piece sits 4 binades lower): elements of a block whose largest is under 2^-115 are rounded to
        # multiples of 2^-135, an eighth of bf16's subnormal spacing.  Row 7 is held to that bound element by
        # element: |dY[n]| <= 2^-136 sum_k |W^(p)[n, k]|, plus the ordinary bar for the fp32 accumulation.
        What = O.dequant(codes, s0, z0, int(prec[7]))
        bound = 2.0 ** -136 * np.abs(What).sum(axis=1) + MAX_ABS_TOL * np.sqrt(np.mean(Yref[7] ** 2))
        err = np.abs(Y[7].astype(np.float64) - Yref[7])
        print(f"[parity] special row 7 (subnormals): max err/bound {float((err / bound).max()):.3f}", flush=True)
        assert np.all(err <= bound)
    else:
        assert_output_close(Y[7:8], Yref[7:8], "special row 7")


@pytest.mark.parametrize("T", [16, 64])
def test_stage_call_replays_from_a_hip_graph(mbq, T):
    """The stage call captured once and replayed with new activations in the same buffers (eager work and
    synchronisation between the replays): every replay equals the eager call bit for bit.  K = 4096 takes the
    two-part kernels at both token counts, whose outputs the router launch zeroes with a kernel (not a memset
    node); at 64 tokens the linear launch also sorts the tokens."""
    K, Ns = 4096, (272, 130)
    print(f"[case] stage call under graph replay T={T}", flush=True)
    rng = np.random.default_rng(47)
    Wrs = [dev((rng.standard_normal((4, K)) / np.sqrt(K)).astype(np.float32)) for _ in Ns]
    brs = [dev(rng.normal(0, 0.3, size=4).astype(np.float32)) for _ in Ns]
    blobs = [mbq.mbq_encode(dev(make_weight(N, K, [47, N], 4.0))) for N in Ns]
    X = dev_bf16(tokens(T, K, [47, 0])).reshape(T, K)
    ws_r = mbq.route_workspace(T, K, "cuda")
    ws_l = mbq.linear_workspace(T, max(Ns), K, "cuda")
    routing = [(torch.empty(T, dtype=torch.int32, device="cuda"), torch.empty(T, dtype=torch.int32, device="cuda"),
                torch.empty(5, dtype=torch.int32, device="cuda")) for _ in Ns]
    Ys = [torch.empty((T, N), dtype=torch.float32, device="cuda") for N in Ns]

    def call():
        mbq.mbq_routed_linear_group(X, Wrs, brs, blobs, list(Ns), routing=routing, Y=Ys, ws_route=ws_r, ws_linear=ws_l)

    call()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call()
    for rep in range(4):
        X.copy_(dev_bf16(tokens(T, K, [47, rep + 1])).reshape(T, K))
        call()
        torch.cuda.synchronize()
        want = [[t.clone() for t in r] for r in routing], [y.clone() for y in Ys]
        for y in Ys:
            y.fill_(float("nan"))
        for r in routing:
            for t in r:
                t.fill_(-7)
        g.replay()
        torch.cuda.synchronize()
        for i in range(len(Ns)):
            for a, b in zip(want[0][i], routing[i]):
                assert torch.equal(a, b), (rep, i)
            assert torch.equal(want[1][i], Ys[i]), (rep, i)


def test_stage_calls_on_drawn_shapes(mbq):
    """Stage calls on seeded random shapes (1..4 matrices, 1..64 tokens, K up to 6144, ragged N): routing,
    permutation and outputs against the oracle.  Covers the launch arithmetic of the grouped kernels (shares of
    workgroups per matrix, K parts, token passes) beyond the hand-picked shapes above."""
    rng = np.random.default_rng(2027)
    for case in range(14):
        n = int(rng.integers(1, 5))
        T = int(rng.choice([1, 7, 16, 17, 29, 33, 48, 63, 64]))
        K = 128 * int(rng.integers(1, 49))
        Ns = [int(rng.integers(1, 700)) for _ in range(n)]
        print(f"[case] drawn stage {case}: T={T} K={K} Ns={Ns}", flush=True)
        xb = tokens(T, K, [2027, case])
        X = dev_bf16(xb).reshape(T, K)
        Wrs = [(rng.standard_normal((4, K)) / np.sqrt(K)).astype(np.float32) for _ in Ns]
        brs = [rng.normal(0, 0.3, size=4).astype(np.float32) for _ in Ns]
        Ws = [make_weight(N, K, [53, case, i], 4.0) for i, N in enumerate(Ns)]
        blobs = [mbq.mbq_encode(dev(W)) for W in Ws]
        routing, Ys = mbq.mbq_routed_linear_group(X, [dev(w) for w in Wrs], [dev(b) for b in brs], blobs, Ns)
        torch.cuda.synchronize()
        for i, N in enumerate(Ns):
            S, prec_ref, gap = O.route(xb, Wrs[i], brs[i])
            prec = routing[i][0].cpu().numpy()
            compare_routing(prec, prec_ref, gap, f"drawn stage {case} router {i}")
            check_bucket(prec, routing[i][1].cpu().numpy(), routing[i][2].cpu().numpy())
            codes, s0, z0 = O.encode(Ws[i])
            assert_output_close(Ys[i].cpu().numpy(), O.linear(xb, codes, s0, z0, prec), f"drawn stage {case} matrix {i}")


def test_prefill_on_drawn_shapes(mbq):
    """mbq_linear above 64 tokens on seeded random shapes, automatic launch choice (including the K split that
    launches with few tiles take from K = 8192 on): outputs against the oracle."""
    rng = np.random.default_rng(2029)
    shapes = [(int(rng.integers(65, 700)), int(rng.integers(1, 600)), 128 * int(rng.integers(1, 40))) for _ in range(6)]
    shapes += [(130, 272, 8192), (600, 520, 9216), (257, 40, 12288)]
    for case, (T, N, K) in enumerate(shapes):
        print(f"[case] drawn prefill {case}: T={T} N={N} K={K}", flush=True)
        W = make_weight(N, K, [59, case], 4.0)
        xb = tokens(T, K, [2029, case])
        prec = rng.choice(4, size=T, p=[0.4, 0.3, 0.2, 0.1]).astype(np.int32)
        codes, s0, z0 = O.encode(W)
        Yref = O.linear(xb, codes, s0, z0, prec)
        Y = run_linear(mbq, W, xb, prec, 0)
        assert_output_close(Y, Yref, f"drawn prefill {case}")


@pytest.mark.parametrize("T,K,Ns", [(65, 4096, (130,)), (96, 2304, (48,)), (128, 4096, (272,)), (100, 1024, (40,)),
                                    (128, 4352, (2064,)), (96, 4096, (272, 130, 16)), (127, 512, (48, 300)),
                                    (80, 4352, (2064, 16)), (192, 4096, (130, 272)), (161, 2304, (48,)), (500, 1024, (300,))])
def test_automatic_choice_above_64_tokens(mbq, T, K, Ns):
    """Above 64 tokens the automatic choice still takes the register-stationary kernel (one pass per 32 sorted
    tokens, the tokens dealt evenly to the passes) up to 128 tokens, 512 for small matrices, alone or as one launch
    for a group; (80, 4352, (2064, 16)) mixes it with the prefill kernel inside one group call.  Group and single
    calls against the oracle."""
    print(f"[case] automatic choice T={T} K={K} Ns={Ns}", flush=True)
    xb = tokens(T, K, [T, K, 61])
    X = dev_bf16(xb).reshape(T, K)
    blobs, routing, refs = [], [], []
    for i, N in enumerate(Ns):
        W = make_weight(N, K, [61, N, K, i], 4.0)
        codes, s0, z0 = O.encode(W)
        prec = np.random.default_rng([T, K, i]).integers(0, 4, size=T).astype(np.int32)
        perm, offsets = O.bucket(prec)
        blobs.append(mbq.mbq_encode(dev(W)))
        routing.append((dev(prec), dev(perm), dev(offsets)))
        refs.append(O.linear(xb, codes, s0, z0, prec))
    Ys = mbq.mbq_linear_group(X, blobs, list(Ns), K, routing)
    torch.cuda.synchronize()
    for i, N in enumerate(Ns):
        assert_output_close(Ys[i].cpu().numpy(), refs[i], f"automatic choice matrix {i}")
        single = mbq.mbq_linear(X, blobs[i], N, K, *routing[i])
        # (no bit-for-bit claim here: a matrix that goes to the prefill kernel may be cut into more than two parts
        # along K, whose float atomic adds land in any order)
        assert_output_close(single.cpu().numpy(), refs[i], f"automatic choice matrix {i}, single call")


@pytest.mark.parametrize("T", [129, 200, 256])
@pytest.mark.parametrize("mix", [(0.8, 0.15, 0.05, 0.0), (0.25, 0.25, 0.25, 0.25), (0.0, 0.0, 0.1, 0.9)])
def test_choice_by_precision_mix_from_129_to_256_tokens(mbq, T, mix):
    """129..256 tokens on a matrix that is not small: the stationary kernel and the prefill kernel are both
    launched and the device lets one of them work, by the slices the sorted passes would read; a skewed mix
    takes the first, a uniform or high-precision mix the second.  Either way against the oracle."""
    N, K = 2064, 4352
    print(f"[case] choice by mix T={T} mix={mix}", flush=True)
    W = make_weight(N, K, [67, T], 4.0)
    xb = tokens(T, K, [67, T, 1])
    prec = np.random.default_rng([67, T]).choice(4, size=T, p=mix).astype(np.int32)
    codes, s0, z0 = O.encode(W)
    Yref = O.linear(xb, codes, s0, z0, prec)
    Y = run_linear(mbq, W, xb, prec, 0)
    assert_output_close(Y, Yref, f"choice by mix T={T} mix={mix}")


def test_linear_zero_tokens_and_bad_arguments(mbq):
    N, K = 32, 256
    W = make_weight(N, K, [17], 4.0)
    blob = mbq.mbq_encode(dev(W))
    empty = torch.empty((0, K), dtype=torch.bfloat16, device="cuda")
    z32 = torch.zeros(0, dtype=torch.int32, device="cuda")
    off = torch.zeros(5, dtype=torch.int32, device="cuda")
    Y = mbq.mbq_linear(empty, blob, N, K, z32, z32, off)
    assert Y.shape == (0, N)
    xb = tokens(70, K, 1)
    prec = np.zeros(70, dtype=np.int32)
    perm, offsets = O.bucket(prec)
    with pytest.raises(mbq.MbqError):       # the decode kernel refuses more than 64 tokens
        mbq.mbq_linear(dev_bf16(xb), blob, N, K, dev(prec), dev(perm), dev(offsets), algo=2)
    with pytest.raises(mbq.MbqError):       # workspace too small
        mbq.mbq_linear(dev_bf16(xb), blob, N, K, dev(prec), dev(perm), dev(offsets),
                       ws=torch.empty(16, dtype=torch.uint8, device="cuda"))


def test_config0_end_to_end(mbq):
    """BASELINE config 0: 2048 x 2048, 32 tokens, {40,30,20,10}% mix; full comparison, every kernel."""
    cfg = CONFIGS[0]
    case = make_case(cfg, 0, 32)
    W, xb, Wr, br = case["W"], case["X"], case["Wr"], case["br"]
    N, K = W.shape
    codes, s0, z0 = O.encode(W)
    S, prec_ref, gap = O.route(xb, Wr, br)
    X = dev_bf16(xb)
    blob = mbq.mbq_encode(dev(W))
    assert np.array_equal(blob.cpu().numpy(), O.pack_blob(codes, s0, z0))
    prec, perm, offsets = mbq.mbq_route(X, dev(Wr), dev(br))
    compare_routing(prec.cpu().numpy(), prec_ref, gap, "config 0")
    check_bucket(prec.cpu().numpy(), perm.cpu().numpy(), offsets.cpu().numpy())
    Yref = O.linear(xb, codes, s0, z0, prec.cpu().numpy())
    for name, algo in ALGOS.items():
        Y = mbq.mbq_linear(X, blob, N, K, prec, perm, offsets, algo=algo)
        assert_output_close(Y.cpu().numpy(), Yref, f"config 0 {name}")
    # the layer fed with the oracle's routing as well
    perm_ref, off_ref = O.bucket(prec_ref)
    Y = mbq.mbq_linear(X, blob, N, K, dev(prec_ref), dev(perm_ref), dev(off_ref))
    assert_output_close(Y.cpu().numpy(), O.linear(xb, codes, s0, z0, prec_ref), "config 0 oracle routing")
