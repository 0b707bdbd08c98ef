"""GPU parity at the full sizes of BASELINE configs 1-4 with the automatic kernel choice, per matrix
(mbq_route + mbq_linear) and, for the block the bench times, per stage call (mbq_routed_linear_group).
The decode configurations (1: Llama-2-7B block at 1, 4, 16 tokens; 3: Llama-3-8B block at 64 tokens) are checked IN
FULL: the whole packed blob byte for byte against the oracle's encoding, and every output column of every token
against the oracle (the C oracle, which is pinned to the numpy oracle and the worked example in the CPU tests, redoes
a Llama-sized matrix in about a second).  The prefill configurations (2, 4) are too large for that: there the oracle
recomputes a seeded sample of weight rows (= output columns), including the rows at tile edges - their codes and
scales bit for bit, and the outputs of ALL tokens on those columns within the floating-point bar.  Routing and the
permutation are compared in full everywhere."""
import numpy as np
import pytest
import torch

import oracle as O
from oracle import c_oracle as C
from helpers import assert_output_close, check_bucket, compare_routing, dev, dev_bf16
from workloads import CONFIGS, make_case

pytestmark = pytest.mark.gpu


def sample_rows(N, seed, n_random=160):
    edges = [0, 1, 15, 16, 17, 31, 127, 128, 129, N // 2 - 1, N // 2, N - 129, N - 128, N - 17, N - 16, N - 2, N - 1]
    rng = np.random.default_rng([seed, N])
    rows = set(int(r) for r in edges if 0 <= r < N) | set(int(r) for r in rng.integers(0, N, size=n_random))
    return np.array(sorted(rows))


def check_linear(mbq, cfg, li, full=False):
    spec = cfg.linears[li]
    N, K = spec.N, spec.K
    print(f"[case] config {cfg.index} linear {spec.name} {N}x{K} ({'all columns' if full else 'sampled columns'})", flush=True)
    first = make_case(cfg, li, cfg.token_counts[0])
    W = first["W"]
    blob = mbq.mbq_encode(dev(W))
    if full:
        codes_s, s0_s, z0_s = C.encode(W)                       # the whole matrix
        want = torch.from_numpy(O.pack_blob(codes_s, s0_s, z0_s)).cuda()
        assert blob.numel() == want.numel() and torch.equal(blob, want), "packed blob differs from the oracle's"
        del want
        idx = None
    else:
        rows = sample_rows(N, cfg.seed)
        codes_s, s0_s, z0_s = O.encode(W[rows])
        codes_d, s0_d, z0_d = mbq.mbq_unpack(blob, N, K)
        idx = torch.from_numpy(rows).cuda()
        assert np.array_equal(codes_d[:, idx, :].cpu().numpy(), codes_s)
        assert np.array_equal(s0_d[idx].cpu().numpy(), s0_s) and np.array_equal(z0_d[idx].cpu().numpy(), z0_s)
        del codes_d
    del W
    for T in cfg.token_counts:
        case = first if T == cfg.token_counts[0] else make_case(cfg, li, T, with_weight=False)
        xb, Wr, br = case["X"], case["Wr"], case["br"]
        X = dev_bf16(xb)
        prec, perm, offsets = mbq.mbq_route(X, dev(Wr), dev(br))
        S, prec_ref, gap = O.route(xb, Wr, br)
        p = prec.cpu().numpy()
        what = f"config {cfg.index} {spec.name} T={T}"
        compare_routing(p, prec_ref, gap, what)
        check_bucket(p, perm.cpu().numpy(), offsets.cpu().numpy())
        if len(case["outlier_tokens"]):
            assert (p[case["outlier_tokens"]] == 3).all()      # outlier tokens are pushed to 8 bits
        print(f"[mix] {what}: {np.bincount(p, minlength=4).tolist()} avg bits {O.avg_bits(p):.2f}", flush=True)
        Yref = C.linear(xb, codes_s, s0_s, z0_s, p) if full else O.linear(xb, codes_s, s0_s, z0_s, p)
        algos = [0] if T <= 16 or T > 64 else [2, 3]              # 17..64 tokens: both kernel families
        for algo in algos:
            Y = mbq.mbq_linear(X, blob, N, K, prec, perm, offsets, algo=algo)
            if full:
                assert_output_close(Y.cpu().numpy(), Yref, f"{what} algo={algo} (all {N} columns)")
            else:
                assert_output_close(Y[:, idx].cpu().numpy(), Yref, f"{what} algo={algo} ({len(rows)} sampled columns)")


@pytest.mark.parametrize("li", range(7))
def test_config1_llama2_7b_decode(mbq, li):
    check_linear(mbq, CONFIGS[1], li, full=True)


@pytest.mark.parametrize("li", range(3))
def test_config2_llama2_7b_prefill(mbq, li):
    check_linear(mbq, CONFIGS[2], li)


@pytest.mark.parametrize("li", range(7))
def test_config3_llama3_8b_decode64(mbq, li):
    check_linear(mbq, CONFIGS[3], li, full=True)


@pytest.mark.parametrize("li", range(3))
def test_config4_llama70b_mlp(mbq, li):
    check_linear(mbq, CONFIGS[4], li)


@pytest.mark.parametrize("names", [("q", "k", "v"), ("o",), ("gate", "up"), ("down",)])
def test_config1_block_stage_calls(mbq, names):
    """The launch form the bench times: one mbq_routed_linear_group call per stage of the Llama-2-7B-shaped
    block (projections that share their input routed and computed together), at every batch size of the
    config.  Routing in full, every output column of every projection, against the oracle."""
    cfg = CONFIGS[1]
    by_name = {s.name: i for i, s in enumerate(cfg.linears)}
    lis = [by_name[n] for n in names]
    K = cfg.linears[lis[0]].K
    Ns = [cfg.linears[li].N for li in lis]
    print(f"[case] config 1 stage {names}", flush=True)
    blobs, encoded = [], []
    for li in lis:
        W = make_case(cfg, li, 1)["W"]
        blobs.append(mbq.mbq_encode(dev(W)))
        encoded.append(C.encode(W))
        del W
    for T in cfg.token_counts:
        cases = [make_case(cfg, li, T, with_weight=False) for li in lis]
        xb = cases[0]["X"]                     # the stage's projections read the first one's activations
        X = dev_bf16(xb)
        routing, Ys = mbq.mbq_routed_linear_group(X, [dev(c["Wr"]) for c in cases], [dev(c["br"]) for c in cases],
                                                  blobs, Ns)
        torch.cuda.synchronize()
        for i, li in enumerate(lis):
            what = f"config 1 stage {names} {cfg.linears[li].name} T={T}"
            S, prec_ref, gap = O.route(xb, cases[i]["Wr"], cases[i]["br"])
            p = routing[i][0].cpu().numpy()
            compare_routing(p, prec_ref, gap, what)
            check_bucket(p, routing[i][1].cpu().numpy(), routing[i][2].cpu().numpy())
            codes_s, s0_s, z0_s = encoded[i]
            Yref = C.linear(xb, codes_s, s0_s, z0_s, p)
            assert_output_close(Ys[i].cpu().numpy(), Yref, what + f" (all {Ns[i]} columns)")
