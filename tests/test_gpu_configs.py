"""GPU parity for other slice configurations (Sec. 4.1 general E and b_e, App. C.1): the library runs them as cuts of
its eight-bit code; the oracle (oracle/mbq_oracle_general.py) runs the literal recursion with the configuration's own
widths, scales and zero points.  Encode and routing bit-exact, outputs to the usual bar."""
import numpy as np
import pytest
import torch

import oracle as O
from oracle import mbq_oracle_general as G
from helpers import assert_output_close, check_bucket, compare_routing, dev, dev_bf16
from workloads import f32_to_bf16_bits, make_weight

pytestmark = pytest.mark.gpu

CONFIGS = [(2, 2, 2, 2), (4, 2, 2), (2, 4, 2), (2, 2, 4), (4, 4), (6, 2), (2, 6), (8,), (2, 2, 2), (4, 2), (2,),
           (3, 1, 2, 2), (3, 2, 1), (4, 1, 1, 2), (1, 1, 1, 1), (5, 3), (1, 2, 2, 2), (7,)]       # the last row: bit configurations


def stored_values(mbq, cfg, E):
    """What the precision arrays hold for the configuration's precisions, and the digits tokens are bucketed by."""
    values = np.array([mbq.config_precision_value(cfg, p) for p in range(E)], dtype=np.int32)
    bits = np.array([mbq.config_bits(cfg, p) for p in range(E)], dtype=np.int32)
    return values, (bits + 1) // 2 - 1


def tokens(T, K, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, K)).astype(np.float32)
    x[:, rng.choice(K, max(1, K // 100), replace=False)] *= 20.0
    return f32_to_bf16_bits(x)


@pytest.mark.parametrize("bits", CONFIGS)
def test_encode_in_the_configurations_terms_is_bit_exact(mbq, bits):
    N, K = 37, 640
    print(f"[case] config {bits}: encode / unpack / dequant N={N} K={K}", flush=True)
    cfg = mbq.Config(bits)
    mbq.config_check(cfg)
    W = make_weight(N, K, [61, len(bits), bits[0]], 4.0)
    blob = mbq.mbq_encode_cfg(dev(W), cfg)
    assert torch.equal(blob, mbq.mbq_encode(dev(W)))          # one blob for every configuration
    codes, s0, z0 = G.encode(W, bits, 128)
    c, s, z = mbq.mbq_unpack_cfg(blob, N, K, cfg)
    torch.cuda.synchronize()
    assert np.array_equal(c.cpu().numpy(), np.stack(codes).astype(np.uint8))
    assert np.array_equal(s.cpu().numpy(), s0) and np.array_equal(z.cpu().numpy(), z0)
    B = G.cumulative_bits(bits)
    for p in range(len(bits)):
        assert mbq.config_bits(cfg, p) == B[p]
        assert mbq.config_precision_value(cfg, p) == (B[p] - 1 if mbq.config_counts_bits(cfg) else B[p] // 2 - 1)
        What = mbq.mbq_dequant_cfg(blob, N, K, cfg, p).cpu().numpy()
        want = G.dequant(codes, s0, z0, bits, 128, p)
        np.testing.assert_allclose(What, want.astype(np.float32), rtol=0, atol=0)
    assert mbq.config_bits(cfg, len(bits)) == -1


@pytest.mark.parametrize("bits,T,K", [((4, 2, 2), 16, 4096), ((4, 4), 5, 384), ((2, 2, 2), 28, 1280), ((8,), 16, 256),
                                      ((6, 2), 64, 2048), ((2, 4, 2), 129, 512), ((4, 2, 2), 700, 256),
                                      ((2, 6), 0, 256), ((3, 1, 2, 2), 16, 4096), ((3, 2, 1), 40, 512),
                                      ((1, 1, 1, 1), 100, 384), ((4, 1, 1, 2), 300, 256), ((5, 3), 0, 128)])
def test_route_with_as_many_outputs_as_slices(mbq, bits, T, K):
    print(f"[case] config {bits}: route T={T} K={K}", flush=True)
    cfg = mbq.Config(bits)
    E = len(bits)
    rng = np.random.default_rng([T, K, E])
    xb = tokens(T, K, [T, K, 3])
    Wr = (rng.standard_normal((E, K)) / np.sqrt(K)).astype(np.float32)
    br = rng.normal(0, 0.2, size=E).astype(np.float32)
    S, prec_ref, gap = O.route(xb, Wr, br) if E > 1 else (None, np.zeros(T, dtype=np.int32), np.full(T, np.inf))
    values, digits = stored_values(mbq, cfg, E)
    prec, perm, offsets, logits = mbq.mbq_route_cfg(dev_bf16(xb).reshape(T, K), dev(Wr), dev(br), cfg, want_logits=True)
    torch.cuda.synchronize()
    prec, perm, offsets = prec.cpu().numpy(), perm.cpu().numpy(), offsets.cpu().numpy()
    if T and E > 1:
        np.testing.assert_allclose(logits.cpu().numpy(), S, rtol=0, atol=1e-10)
    compare_routing(prec, values[prec_ref], gap, f"route config {bits} T={T}")
    shift = 1 if mbq.config_counts_bits(cfg) else 0
    check_bucket(prec >> shift, perm, offsets)   # buckets are by the digits a token touches: five offsets as ever
    assert offsets[4] == T
    assert set(np.unique(prec)).issubset(set(values.tolist()))


@pytest.mark.parametrize("bits,T,K,Ns", [((4, 2, 2), 16, 4096, (272, 130)), ((4, 4), 12, 1280, (96,)),
                                         ((2, 2, 2), 16, 8192, (64, 48, 80)), ((6, 2), 40, 4096, (272,)),
                                         ((2, 4, 2), 64, 1024, (130, 64)), ((8,), 16, 512, (100,)),
                                         ((4, 2, 2), 300, 768, (260,)),
                                         # bit configurations: the decode kernel up to 16 tokens and K <= 8192 ...
                                         ((3, 1, 2, 2), 16, 4096, (272, 130)), ((3, 2, 1), 12, 1280, (96, 40, 64)),
                                         ((1, 1, 1, 1), 16, 8192, (48,)), ((4, 1, 1, 2), 7, 2304, (130, 66)),
                                         ((1, 2, 2, 2), 16, 768, (100,)), ((7,), 3, 512, (64,)),
                                         # ... 16 tokens per launch beyond
                                         ((3, 1, 2, 2), 40, 512, (72,)), ((5, 3), 16, 8448, (32,)),
                                         ((3, 2, 1), 300, 768, (130, 64)), ((1, 2, 2, 2), 17, 4096, (272,)),
                                         ((4, 1, 1, 2), 33, 11008, (48,))])
def test_stage_call_under_a_configuration(mbq, bits, T, K, Ns):
    """mbq_routed_linear_group_cfg against the general oracle: precisions (as digit counts) bit-exact off the near-tie
    list, outputs within the bar for the precisions the GPU chose, and identical to route_cfg + linear_group."""
    print(f"[case] config {bits}: stage T={T} K={K} Ns={Ns}", flush=True)
    cfg = mbq.Config(bits)
    E = len(bits)
    rng = np.random.default_rng([T, K, E, len(Ns)])
    xb = tokens(T, K, [T, K, 5])
    X = dev_bf16(xb).reshape(T, K)
    Wrs = [(rng.standard_normal((E, K)) / np.sqrt(K)).astype(np.float32) for _ in Ns]
    brs = [rng.normal(0, 0.3, size=E).astype(np.float32) for _ in Ns]
    Ws = [make_weight(N, K, [67, N, K, i], 4.0) for i, N in enumerate(Ns)]
    blobs = [mbq.mbq_encode_cfg(dev(W), cfg) for W in Ws]
    dWr, dbr = [dev(w) for w in Wrs], [dev(b) for b in brs]
    routing, Ys = mbq.mbq_routed_linear_group_cfg(X, dWr, dbr, cfg, blobs, list(Ns))
    torch.cuda.synchronize()
    routing2 = mbq.mbq_route_group_cfg(X, dWr, dbr, cfg)
    if mbq.config_counts_bits(cfg):
        Ys2 = [mbq.mbq_linear_cfg(X, blobs[i], N, K, cfg, *routing2[i]) for i, N in enumerate(Ns)]
    else:
        Ys2 = mbq.mbq_linear_group(X, blobs, list(Ns), K, routing2)
    values, digits = stored_values(mbq, cfg, E)
    shift = 1 if mbq.config_counts_bits(cfg) else 0
    back = {int(d): p for p, d in enumerate(values)}
    for i, N in enumerate(Ns):
        for a, b in zip(routing[i], routing2[i]):
            assert torch.equal(a, b), i
        assert torch.equal(Ys[i], Ys2[i]) or T > 64, i       # (the tiled GEMM may add K parts in any order)
        prec = routing[i][0].cpu().numpy()
        if E > 1:
            _, prec_ref, gap = O.route(xb, Wrs[i], brs[i])
        else:
            prec_ref, gap = np.zeros(T, dtype=np.int32), np.full(T, np.inf)
        compare_routing(prec, values[prec_ref], gap, f"stage router {i}")
        check_bucket(prec >> shift, routing[i][1].cpu().numpy(), routing[i][2].cpu().numpy())
        prec_cfg = np.array([back[int(d)] for d in prec], dtype=np.int32)       # the GPU's choice, as config indices
        codes, s0, z0 = G.encode(Ws[i], bits, 128)
        want = G.linear(xb, codes, s0, z0, bits, 128, prec_cfg)
        assert_output_close(Ys[i].cpu().numpy(), want, f"config {bits} matrix {i}")
        assert_output_close(Ys2[i].cpu().numpy(), want, f"config {bits} matrix {i}, two calls")


SMALL_GROUPS = [((2, 2, 2, 2), 64), ((4, 2, 2), 64), ((3, 2, 1), 64), ((2, 2, 2, 2), 32), ((4, 1, 1, 2), 32),
                ((8,), 32), ((2, 3), 64)]


@pytest.mark.parametrize("bits,group", SMALL_GROUPS)
def test_groups_of_64_and_32_columns_encode_bit_exact(mbq, bits, group):
    """App. C.1 lists the group size among the settings: codes, (s_0, z_0) per group and every W^(p) against the
    general oracle at that group size; the blob has the documented size and is written in full."""
    N, K = 37, 640
    print(f"[case] config {bits} group {group}: encode / unpack / dequant N={N} K={K}", flush=True)
    cfg = mbq.Config(bits, group)
    mbq.config_check(cfg)
    W = make_weight(N, K, [71, len(bits), bits[0], group], 4.0)
    blob = mbq.mbq_encode_cfg(dev(W), cfg)
    assert blob.numel() == mbq.blob_bytes_cfg(cfg, N, K) > mbq.blob_bytes(N, K)
    codes, s0, z0 = G.encode(W, bits, group)
    c, s, z = mbq.mbq_unpack_cfg(blob, N, K, cfg)
    torch.cuda.synchronize()
    assert s.shape == (N, K // group)
    assert np.array_equal(c.cpu().numpy(), np.stack(codes).astype(np.uint8))
    assert np.array_equal(s.cpu().numpy(), s0) and np.array_equal(z.cpu().numpy(), z0)
    for p in range(len(bits)):
        What = mbq.mbq_dequant_cfg(blob, N, K, cfg, p).cpu().numpy()
        np.testing.assert_allclose(What, G.dequant(codes, s0, z0, bits, group, p).astype(np.float32), rtol=0, atol=0)
    # rows and groups of the padding hold zeros: the blob is written in full, whatever the buffer held before
    blob2 = torch.full_like(blob, 0xA5)
    mbq.mbq_encode_cfg(dev(W), cfg, blob2)
    assert torch.equal(blob, blob2)


@pytest.mark.parametrize("bits,group,T,K,Ns", [((2, 2, 2, 2), 64, 16, 1024, (100, 48)), ((4, 2, 2), 64, 40, 512, (72,)),
                                               ((3, 2, 1), 64, 9, 768, (64, 33)), ((2, 2, 2, 2), 32, 70, 256, (96,)),
                                               ((4, 1, 1, 2), 32, 16, 640, (40,)), ((8,), 32, 3, 384, (50,)),
                                               ((2, 2, 2, 2), 64, 0, 256, (16,))])
def test_stage_call_with_groups_of_64_and_32_columns(mbq, bits, group, T, K, Ns):
    """The routed stage and route_cfg + linear_cfg on blobs with smaller groups (the one-thread-per-output kernel at
    every token count) against the general oracle at that group size."""
    print(f"[case] config {bits} group {group}: stage T={T} K={K} Ns={Ns}", flush=True)
    cfg = mbq.Config(bits, group)
    E = len(bits)
    rng = np.random.default_rng([T, K, E, group])
    xb = tokens(T, K, [T, K, 9])
    X = dev_bf16(xb).reshape(T, K)
    Wrs = [(rng.standard_normal((E, K)) / np.sqrt(K)).astype(np.float32) for _ in Ns]
    brs = [rng.normal(0, 0.3, size=E).astype(np.float32) for _ in Ns]
    Ws = [make_weight(N, K, [73, N, K, i], 4.0) for i, N in enumerate(Ns)]
    blobs = [mbq.mbq_encode_cfg(dev(W), cfg) for W in Ws]
    dWr, dbr = [dev(w) for w in Wrs], [dev(b) for b in brs]
    routing, Ys = mbq.mbq_routed_linear_group_cfg(X, dWr, dbr, cfg, blobs, list(Ns))
    torch.cuda.synchronize()
    routing2 = mbq.mbq_route_group_cfg(X, dWr, dbr, cfg)
    values, digits = stored_values(mbq, cfg, E)
    shift = 1 if mbq.config_counts_bits(cfg) else 0
    back = {int(d): p for p, d in enumerate(values)}
    for i, N in enumerate(Ns):
        for a, b in zip(routing[i], routing2[i]):
            assert torch.equal(a, b), i
        Y2 = mbq.mbq_linear_cfg(X, blobs[i], N, K, cfg, *routing2[i])
        assert torch.equal(Ys[i], Y2), i
        assert Ys[i].shape == (T, N)
        if T == 0:
            continue
        prec = routing[i][0].cpu().numpy()
        if E > 1:
            _, prec_ref, gap = O.route(xb, Wrs[i], brs[i])
        else:
            prec_ref, gap = np.zeros(T, dtype=np.int32), np.full(T, np.inf)
        compare_routing(prec, values[prec_ref], gap, f"stage router {i}")
        check_bucket(prec >> shift, routing[i][1].cpu().numpy(), routing[i][2].cpu().numpy())
        prec_cfg = np.array([back[int(d)] for d in prec], dtype=np.int32)
        codes, s0, z0 = G.encode(Ws[i], bits, group)
        want = G.linear(xb, codes, s0, z0, bits, group, prec_cfg)
        assert_output_close(Ys[i].cpu().numpy(), want, f"config {bits} group {group} matrix {i}")


def test_unsupported_configurations_are_refused(mbq):
    for bits, group in [((2, 2, 2, 2), 16), ((2, 2, 2, 2), 96), ((4, 4, 2), 128), ((3, 3, 3), 128),
                        ((2, 2, 2, 2, 2), 128), ((), 128), ((0, 2), 128)]:
        cfg = mbq.Config(bits[:4], group)
        cfg.n_slices = len(bits)
        with pytest.raises(mbq.MbqError):
            mbq.config_check(cfg)
    W = dev(make_weight(16, 256, [1], 4.0))
    with pytest.raises(mbq.MbqError):
        mbq.mbq_encode_cfg(W, mbq.Config((2, 2, 2, 2), 16))
    # P must match the configuration
    cfg = mbq.Config((4, 2, 2))
    X = dev_bf16(tokens(4, 256, 1)).reshape(4, 256)
    with pytest.raises(AssertionError):
        mbq.mbq_route_cfg(X, dev(np.zeros((4, 256), dtype=np.float32)), dev(np.zeros(4, dtype=np.float32)), cfg)
