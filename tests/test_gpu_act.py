"""GPU parity for the activation-quantised variant (App. E.4): quantiser outputs bit for bit against the oracle, and
the whole stage - quantise, route on the rebuilt activations, routed linears on the integers, row scaling and bias -
against the oracle to the usual bar."""
import numpy as np
import pytest
import torch

import oracle as O
from oracle import mbq_oracle_act as A
from helpers import assert_output_close, check_bucket, compare_routing, dev, dev_bf16
from workloads import f32_to_bf16_bits, make_weight

pytestmark = pytest.mark.gpu


def activations(T, K, seed, offset=0.0):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, K)).astype(np.float32) + np.float32(offset)
    if K:
        x[:, rng.choice(K, max(1, K // 100), replace=False)] *= 15.0
    return f32_to_bf16_bits(x)


def let_params(K, seed):
    rng = np.random.default_rng(seed)
    s = np.exp2(rng.uniform(-1.5, 1.5, size=K)).astype(np.float32)
    delta = rng.normal(0, 0.5, size=K).astype(np.float32)
    return delta, s


def bf16_tensor_bits(t: torch.Tensor) -> np.ndarray:
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("abits", [2, 4, 5, 8])
@pytest.mark.parametrize("T,K,let,offset", [(1, 128, True, 0.0), (16, 4096, True, 0.0), (70, 640, False, 0.0),
                                            (5, 11008, True, 2.0), (33, 2304, False, -30.0), (300, 256, True, 0.0)])
def test_quantiser_is_bit_exact(mbq, abits, T, K, let, offset):
    print(f"[case] act_quant abits={abits} T={T} K={K} let={let} offset={offset}", flush=True)
    xb = activations(T, K, [abits, T, K], offset)
    xb[0, : min(K, 128)] = 0                                     # a stretch of zeros; with T = 1, K = 128: an all-zero row
    delta, s = let_params(K, [K, 7])
    if let:
        Xt = A.let_transform(xb, delta, s)
        got = mbq.mbq_act_quant(dev_bf16(xb).reshape(T, K), abits, dev(delta), dev(s))
    else:
        Xt = A.bf16_bits_to_f32(xb)
        got = mbq.mbq_act_quant(dev_bf16(xb).reshape(T, K), abits)
    torch.cuda.synchronize()
    xint, scale, zp, q = A.act_quant(Xt, abits)
    assert np.array_equal(got[1].cpu().numpy(), scale)
    assert np.array_equal(got[0].float().cpu().numpy().astype(np.int32), xint)
    if let:
        want_xr = A.router_input_bits(xint, scale, delta, s)
    else:
        want_xr = A.f32_to_bf16_bits_rne((xint.astype(np.float32) * scale[:, None]).astype(np.float32))
    assert np.array_equal(bf16_tensor_bits(got[2]), want_xr)
    # without the router input asked for, the rest is the same
    again = mbq.mbq_act_quant(dev_bf16(xb).reshape(T, K), abits, dev(delta) if let else None, dev(s) if let else None,
                              want_router_input=False)
    assert again[2] is None and torch.equal(again[0], got[0]) and torch.equal(again[1], got[1])


@pytest.mark.parametrize("abits,T,K,Ns", [(4, 16, 4096, (272, 130)), (4, 7, 11008, (64,)), (8, 16, 1280, (96, 40, 64)),
                                          (4, 40, 2048, (130,)), (4, 64, 4096, (272,)), (6, 300, 768, (260, 100)),
                                          (4, 1, 256, (16,))])
def test_stage_of_the_variant(mbq, abits, T, K, Ns):
    """mbq_act_quant -> mbq_route_group on the rebuilt activations -> mbq_linear_group on the integers ->
    mbq_scale_rows with the folded bias, against Y = scale_i ((q - zp) W~^(p_i)^T) + B~ of the oracle."""
    print(f"[case] W-A stage abits={abits} T={T} K={K} Ns={Ns}", flush=True)
    rng = np.random.default_rng([abits, T, K, len(Ns)])
    xb = activations(T, K, [T, K, 17])
    delta, s = let_params(K, [K, 19])
    Ws = [make_weight(N, K, [83, N, K, i], 4.0) for i, N in enumerate(Ns)]
    Bs = [rng.standard_normal(N).astype(np.float32) for N in Ns]
    folded = [A.let_fold(W, B, delta, s) for W, B in zip(Ws, Bs)]
    Wt = [f[0].astype(np.float32) for f in folded]               # what gets encoded: W~ in fp32
    Bt = [f[1].astype(np.float32) for f in folded]
    Wrs = [(rng.standard_normal((4, K)) / np.sqrt(K)).astype(np.float32) for _ in Ns]
    brs = [rng.normal(0, 0.3, size=4).astype(np.float32) for _ in Ns]
    # GPU
    X = dev_bf16(xb).reshape(T, K)
    Xint, row_scale, Xr = mbq.mbq_act_quant(X, abits, dev(delta), dev(s))
    blobs = [mbq.mbq_encode(dev(W)) for W in Wt]
    routing = mbq.mbq_route_group(Xr, [dev(w) for w in Wrs], [dev(b) for b in brs])
    Ys = mbq.mbq_linear_group(Xint, blobs, list(Ns), K, routing)
    for Y, B in zip(Ys, Bt):
        mbq.mbq_scale_rows(Y, row_scale, dev(B))
    torch.cuda.synchronize()
    # the stage as one call: the same numbers, bit for bit (above 64 tokens the tiled GEMM may add K parts in any order)
    routing1, Ys1, act1 = mbq.mbq_routed_linear_group_act(X, abits, dev(delta), dev(s), [dev(w) for w in Wrs],
                                                          [dev(b) for b in brs], blobs, list(Ns),
                                                          bias=[dev(B) for B in Bt])
    torch.cuda.synchronize()
    assert torch.equal(act1[0], Xint) and torch.equal(act1[1], row_scale) and torch.equal(act1[2], Xr)
    for i in range(len(Ns)):
        for a_, b_ in zip(routing1[i], routing[i]):
            assert torch.equal(a_, b_), i
        if T <= 64:
            assert torch.equal(Ys1[i], Ys[i]), i
        else:
            assert_output_close(Ys1[i].cpu().numpy(), Ys[i].double().cpu().numpy(), f"one call vs separate calls {i}")
    # oracle
    xint, scale, zp, q = A.act_quant(A.let_transform(xb, delta, s), abits)
    xr_bits = A.router_input_bits(xint, scale, delta, s)
    assert np.array_equal(bf16_tensor_bits(Xr), xr_bits)
    for i, N in enumerate(Ns):
        prec = routing[i][0].cpu().numpy()
        _, prec_ref, gap = O.route(xr_bits, Wrs[i], brs[i])
        compare_routing(prec, prec_ref, gap, f"router {i} on the rebuilt activations")
        check_bucket(prec, routing[i][1].cpu().numpy(), routing[i][2].cpu().numpy())
        codes, s0, z0 = O.encode(Wt[i])
        Wp = [O.dequant(codes, s0, z0, p) for p in range(4)]
        want = A.w_a_linear(xint, scale, lambda t: Wp[int(prec[t])], Bt[i])
        assert_output_close(Ys[i].cpu().numpy(), want, f"W-A stage abits={abits} matrix {i}")


def test_scale_rows_alone_and_empty_inputs(mbq):
    rng = np.random.default_rng(3)
    Y = rng.standard_normal((37, 130)).astype(np.float32)
    sc = np.exp2(rng.uniform(-4, 4, size=37)).astype(np.float32)
    b = rng.standard_normal(130).astype(np.float32)
    got = mbq.mbq_scale_rows(dev(Y.copy()), dev(sc), dev(b)).cpu().numpy()
    assert np.array_equal(got, ((Y * sc[:, None]).astype(np.float32) + b[None, :]).astype(np.float32))
    got = mbq.mbq_scale_rows(dev(Y.copy()), dev(sc)).cpu().numpy()
    assert np.array_equal(got, (Y * sc[:, None]).astype(np.float32))
    empty = torch.empty((0, 256), dtype=torch.bfloat16, device="cuda")
    xi, rs, xr = mbq.mbq_act_quant(empty, 4)
    assert xi.shape == (0, 256) and rs.shape == (0,)
    with pytest.raises(mbq.MbqError):
        mbq.mbq_act_quant(torch.zeros((2, 256), dtype=torch.bfloat16, device="cuda"), 9)
    with pytest.raises(mbq.MbqError):
        mbq.mbq_act_quant(torch.zeros((2, 192), dtype=torch.bfloat16, device="cuda"), 4)
    # the stage call without tokens, without a transform and without biases
    W = dev(make_weight(32, 256, [1], 4.0))
    Wr, br = dev(np.zeros((4, 256), dtype=np.float32)), dev(np.zeros(4, dtype=np.float32))
    routing, Ys, act = mbq.mbq_routed_linear_group_act(empty, 4, None, None, [Wr], [br], [mbq.mbq_encode(W)], [32])
    torch.cuda.synchronize()
    assert Ys[0].shape == (0, 32) and routing[0][2].cpu().tolist() == [0, 0, 0, 0, 0]
    xb = activations(9, 256, 5)
    routing, Ys, act = mbq.mbq_routed_linear_group_act(dev_bf16(xb).reshape(9, 256), 4, None, None, [Wr], [br],
                                                       [mbq.mbq_encode(W)], [32])
    xint, scale, zp, q = A.act_quant(A.bf16_bits_to_f32(xb), 4)
    codes, s0, z0 = O.encode(make_weight(32, 256, [1], 4.0))
    want = A.w_a_linear(xint, scale, lambda t: O.dequant(codes, s0, z0, 0))     # zero routers: first maximum, p = 0
    assert_output_close(Ys[0].cpu().numpy(), want, "stage call, no transform, no bias")


@pytest.mark.parametrize("T", [16, 40])
def test_stage_of_the_variant_replays_from_a_hip_graph(mbq, T):
    """The one-call stage captured once and replayed with new activations in the same buffers (eager work and
    synchronisation between the replays): every replay equals the eager call bit for bit."""
    K, Ns, abits = 4096, (272, 130), 4
    print(f"[case] W-A stage under graph replay T={T}", flush=True)
    rng = np.random.default_rng(53)
    delta, s = let_params(K, 53)
    d_delta, d_s = dev(delta), dev(s)
    Wrs = [dev((rng.standard_normal((4, K)) / np.sqrt(K)).astype(np.float32)) for _ in Ns]
    brs = [dev(rng.normal(0, 0.3, size=4).astype(np.float32)) for _ in Ns]
    bias = [dev(rng.standard_normal(N).astype(np.float32)) for N in Ns]
    blobs = [mbq.mbq_encode(dev(make_weight(N, K, [53, N], 4.0))) for N in Ns]
    X = dev_bf16(activations(T, K, [53, 0])).reshape(T, K)
    ws_r = mbq.route_workspace(T, K, "cuda")
    ws_l = mbq.linear_workspace(T, max(Ns), K, "cuda")
    routing = [(torch.empty(T, dtype=torch.int32, device="cuda"), torch.empty(T, dtype=torch.int32, device="cuda"),
                torch.empty(5, dtype=torch.int32, device="cuda")) for _ in Ns]
    Ys = [torch.empty((T, N), dtype=torch.float32, device="cuda") for N in Ns]
    act = (torch.empty_like(X), torch.empty((T,), dtype=torch.float32, device="cuda"), torch.empty_like(X))

    def call():
        mbq.mbq_routed_linear_group_act(X, abits, d_delta, d_s, Wrs, brs, blobs, list(Ns), bias=bias, routing=routing,
                                        Y=Ys, act=act, ws_route=ws_r, ws_linear=ws_l)

    call()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call()
    for rep in range(3):
        X.copy_(dev_bf16(activations(T, K, [53, rep + 1])).reshape(T, K))
        call()
        torch.cuda.synchronize()
        want = [[t.clone() for t in r] for r in routing], [y.clone() for y in Ys], [t.clone() for t in act]
        for y in Ys:
            y.fill_(float("nan"))
        for r in routing:
            for t in r:
                t.fill_(-7)
        act[1].fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        for i in range(len(Ns)):
            for a, b in zip(want[0][i], routing[i]):
                assert torch.equal(a, b), (rep, i)
            assert torch.equal(want[1][i], Ys[i]), (rep, i)
        for a, b in zip(want[2], act):
            assert torch.equal(a, b), rep


def test_calls_from_two_threads_do_not_disturb_each_other(mbq):
    """The header allows calls from several threads as long as they share no workspace.  One thread runs stage calls
    under the slice configuration {3,1,2,2}, the other the activation-quantised stage, each on a stream of its own
    (default priority) with its own buffers; every result equals what the same call gave alone.  (What a call runs
    under - configuration, linear operand, test hooks - is per thread inside the library.)"""
    import threading

    T, K, Ns = 16, 4096, (272, 130)
    rng = np.random.default_rng(71)
    Wr4 = [dev((rng.standard_normal((4, K)) / np.sqrt(K)).astype(np.float32)) for _ in Ns]
    br4 = [dev(rng.normal(0, 0.3, size=4).astype(np.float32)) for _ in Ns]
    blobs = [mbq.mbq_encode(dev(make_weight(N, K, [71, N], 4.0))) for N in Ns]
    delta, s = let_params(K, 71)
    d_delta, d_s = dev(delta), dev(s)
    cfg = mbq.Config((3, 1, 2, 2))
    Xs = [dev_bf16(activations(T, K, [71, i])).reshape(T, K) for i in range(6)]

    def run_cfg(X):
        routing, Ys = mbq.mbq_routed_linear_group_cfg(X, Wr4, br4, cfg, blobs, list(Ns))
        return [t for r in routing for t in r] + list(Ys)

    def run_act(X):
        routing, Ys, act = mbq.mbq_routed_linear_group_act(X, 4, d_delta, d_s, Wr4, br4, blobs, list(Ns))
        return [t for r in routing for t in r] + list(Ys) + list(act)

    want = {"cfg": [run_cfg(X) for X in Xs], "act": [run_act(X) for X in Xs]}
    torch.cuda.synchronize()
    failures = []

    def worker(name, fn):
        try:
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                for rep in range(20):
                    i = rep % len(Xs)
                    got = fn(Xs[i])
                    stream.synchronize()
                    for a, b in zip(got, want[name][i]):
                        if not torch.equal(a, b):
                            failures.append((name, rep))
                            return
        except Exception as e:                      # noqa: BLE001 - reported to the main thread
            failures.append((name, repr(e)))

    threads = [threading.Thread(target=worker, args=("cfg", run_cfg)), threading.Thread(target=worker, args=("act", run_act))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not failures, failures
