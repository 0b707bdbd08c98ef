"""Thin Python binding over libmbq.so (C ABI in include/mbq.h).

Argument marshalling only: every step of the path (encode, route, bucket, linear)
runs in the HIP kernels of the library.  torch is used for device memory and the
current stream, nothing else.  There is no CPU fallback: if the shared library is
missing, every call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmbq.so")

ALGO_AUTO, ALGO_SIMPLE, ALGO_DECODE, ALGO_PREFILL = 0, 1, 2, 3
N_PRECISIONS = 4
GROUP = 128

EXPORTS = (
    "mbq_version", "mbq_last_error", "mbq_blob_bytes", "mbq_route_workspace_bytes",
    "mbq_linear_workspace_bytes", "mbq_encode", "mbq_encode_with_params", "mbq_unpack", "mbq_dequant", "mbq_route",
    "mbq_route_group", "mbq_linear", "mbq_linear_group", "mbq_routed_linear_group", "mbq_set_knob",
    "mbq_route_mlp", "mbq_route_mlp_workspace_bytes", "mbq_threshold_quantile",
    "mbq_linear_static", "mbq_static_scratch_bytes",
    # other slice configurations
    "mbq_config_check", "mbq_config_bits", "mbq_config_precision_value", "mbq_config_counts_bits", "mbq_linear_cfg", "mbq_encode_cfg", "mbq_unpack_cfg", "mbq_blob_bytes_cfg",
    "mbq_dequant_cfg", "mbq_route_cfg", "mbq_route_group_cfg", "mbq_routed_linear_group_cfg",
    # activation-quantised variant
    "mbq_act_quant", "mbq_scale_rows", "mbq_routed_linear_group_act",
    # include/mbq_bench.h: measurement and diagnostic entry points
    "mbq_bench_copy", "mbq_bench_read", "mbq_bench_mfma_loop", "mbq_bench_linear_group_prepared",
    "mbq_bench_decode_timeline", "mbq_bench_decode_timeline_bytes", "mbq_bench_decode_timeline_workgroups",
)

_lib = None


class MbqError(RuntimeError):
    pass


class Config(ctypes.Structure):
    """mbq_config of include/mbq.h: slice widths (Sec. 4.1, App. C.1) and group size."""
    _fields_ = [("n_slices", ctypes.c_int), ("slice_bits", ctypes.c_int * 4), ("group", ctypes.c_int)]

    def __init__(self, slice_bits: Sequence[int] = (2, 2, 2, 2), group: int = GROUP):
        super().__init__()
        bits = [int(b) for b in slice_bits]
        self.n_slices = len(bits)
        for e in range(4):
            self.slice_bits[e] = bits[e] if e < min(len(bits), 4) else 0
        self.group = int(group)

    @property
    def bits(self):
        return [self.slice_bits[e] for e in range(min(self.n_slices, 4))]


def load() -> ctypes.CDLL:
    """Loads libmbq.so (built by ``python -m paper_2602_20191_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise MbqError(f"{LIB_PATH} not found: build it with `python -m paper_2602_20191_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    c_i64, c_sz, c_p, c_int = ctypes.c_int64, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int
    lib.mbq_version.restype = ctypes.c_char_p
    lib.mbq_last_error.restype = ctypes.c_char_p
    lib.mbq_blob_bytes.restype = c_sz
    lib.mbq_blob_bytes.argtypes = [c_i64, c_i64]
    lib.mbq_route_workspace_bytes.restype = c_sz
    lib.mbq_route_workspace_bytes.argtypes = [c_i64, c_i64]
    lib.mbq_linear_workspace_bytes.restype = c_sz
    lib.mbq_linear_workspace_bytes.argtypes = [c_i64, c_i64, c_i64]
    lib.mbq_encode.argtypes = [c_p, c_i64, c_i64, c_p, c_p]
    lib.mbq_encode_with_params.argtypes = [c_p, c_i64, c_i64, c_p, c_p, c_p, c_p]
    lib.mbq_unpack.argtypes = [c_p, c_i64, c_i64, c_p, c_p, c_p, c_p]
    lib.mbq_dequant.argtypes = [c_p, c_i64, c_i64, c_int, c_p, c_p]
    lib.mbq_route.argtypes = [c_p, c_i64, c_i64, c_p, c_p, c_int, c_p, c_p, c_p, c_p, c_p, c_sz, c_p]
    lib.mbq_route_group.argtypes = [c_p, c_i64, c_i64, c_int, c_p, c_p, c_int, c_p, c_p, c_p, c_p, c_sz, c_p]
    lib.mbq_route_mlp.argtypes = [c_p, c_i64, c_i64, c_p, c_p, c_int, c_p, c_p, c_int, ctypes.c_double, c_p, c_p, c_p,
                                  c_p, c_p, c_sz, c_p]
    lib.mbq_route_mlp_workspace_bytes.restype = c_sz
    lib.mbq_route_mlp_workspace_bytes.argtypes = [c_i64, c_i64, c_int]
    lib.mbq_threshold_quantile.argtypes = [c_p, c_i64, c_int, ctypes.c_double, c_p, c_p]
    lib.mbq_linear.argtypes = [c_p, c_i64, c_p, c_i64, c_i64, c_p, c_p, c_p, c_p, c_p, c_sz, c_int, c_p]
    lib.mbq_linear_static.argtypes = [c_p, c_i64, c_p, c_i64, c_i64, c_p, c_p, c_p, c_p, c_int, c_p]
    lib.mbq_linear_static.restype = c_int
    lib.mbq_static_scratch_bytes.restype = c_sz
    lib.mbq_static_scratch_bytes.argtypes = []
    lib.mbq_linear_group.argtypes = [c_p, c_i64, c_i64, c_int, c_p, c_p, c_p, c_p, c_p, c_p, c_p, c_sz, c_int, c_p]
    lib.mbq_routed_linear_group.argtypes = [c_p, c_i64, c_i64, c_int, c_p, c_p, c_int, c_p, c_p, c_p, c_p, c_p, c_p,
                                            c_p, c_sz, c_p, c_sz, c_int, c_p]
    lib.mbq_set_knob.argtypes = [c_int, c_int]
    c_cfg = ctypes.POINTER(Config)
    lib.mbq_config_check.argtypes = [c_cfg]
    lib.mbq_blob_bytes_cfg.argtypes = [c_cfg, c_i64, c_i64]
    lib.mbq_blob_bytes_cfg.restype = c_sz
    lib.mbq_config_bits.argtypes = [c_cfg, c_int]
    lib.mbq_config_precision_value.argtypes = [c_cfg, c_int]
    lib.mbq_config_counts_bits.argtypes = [c_cfg]
    lib.mbq_linear_cfg.argtypes = [c_p, c_i64, c_p, c_i64, c_i64, c_cfg, c_p, c_p, c_p, c_p, c_p, c_sz, c_int, c_p]
    lib.mbq_encode_cfg.argtypes = [c_p, c_i64, c_i64, c_cfg, c_p, c_p]
    lib.mbq_unpack_cfg.argtypes = [c_p, c_i64, c_i64, c_cfg, c_p, c_p, c_p, c_p]
    lib.mbq_dequant_cfg.argtypes = [c_p, c_i64, c_i64, c_cfg, c_int, c_p, c_p]
    lib.mbq_route_cfg.argtypes = [c_p, c_i64, c_i64, c_p, c_p, c_cfg, c_p, c_p, c_p, c_p, c_p, c_sz, c_p]
    lib.mbq_route_group_cfg.argtypes = [c_p, c_i64, c_i64, c_int, c_p, c_p, c_cfg, c_p, c_p, c_p, c_p, c_sz, c_p]
    lib.mbq_routed_linear_group_cfg.argtypes = [c_p, c_i64, c_i64, c_int, c_p, c_p, c_cfg, c_p, c_p, c_p, c_p, c_p,
                                                c_p, c_p, c_sz, c_p, c_sz, c_int, c_p]
    for name in ("mbq_config_check", "mbq_config_bits", "mbq_config_precision_value", "mbq_config_counts_bits", "mbq_linear_cfg", "mbq_encode_cfg",
                 "mbq_unpack_cfg", "mbq_dequant_cfg", "mbq_route_cfg", "mbq_route_group_cfg",
                 "mbq_routed_linear_group_cfg"):
        getattr(lib, name).restype = c_int
    lib.mbq_act_quant.argtypes = [c_p, c_i64, c_i64, c_int, c_p, c_p, c_p, c_p, c_p, c_p]
    lib.mbq_act_quant.restype = c_int
    lib.mbq_scale_rows.argtypes = [c_p, c_i64, c_i64, c_p, c_p, c_p]
    lib.mbq_scale_rows.restype = c_int
    lib.mbq_routed_linear_group_act.argtypes = [c_p, c_i64, c_i64, c_int, c_p, c_p, c_int, c_p, c_p, c_int, c_p, c_p,
                                                c_p, c_p, c_p, c_p, c_p, c_p, c_p, c_p, c_p, c_sz, c_p, c_sz, c_int,
                                                c_p]
    lib.mbq_routed_linear_group_act.restype = c_int
    lib.mbq_bench_copy.argtypes = [c_p, c_p, c_sz, c_int, c_p]
    lib.mbq_bench_read.argtypes = [c_p, c_sz, c_int, c_p, c_p]
    lib.mbq_bench_mfma_loop.argtypes = [c_int, c_int, c_p, ctypes.POINTER(ctypes.c_double), c_p]
    lib.mbq_bench_linear_group_prepared.argtypes = [c_i64, c_i64, c_int, c_p, c_p, c_p, c_p, c_p, c_sz, c_p]
    lib.mbq_bench_decode_timeline.argtypes = [c_i64, c_i64, c_int, c_p, c_p, c_p, c_p, c_p, c_sz, c_p, c_sz, c_p]
    lib.mbq_bench_decode_timeline_bytes.restype = c_sz
    lib.mbq_bench_decode_timeline_bytes.argtypes = []
    lib.mbq_bench_decode_timeline_workgroups.restype = c_int
    lib.mbq_bench_decode_timeline_workgroups.argtypes = []
    for name in ("mbq_encode", "mbq_encode_with_params", "mbq_unpack", "mbq_dequant", "mbq_route", "mbq_route_group", "mbq_linear",
                 "mbq_linear_group", "mbq_routed_linear_group", "mbq_set_knob", "mbq_route_mlp",
                 "mbq_threshold_quantile", "mbq_bench_copy", "mbq_bench_read", "mbq_bench_mfma_loop",
                 "mbq_bench_linear_group_prepared", "mbq_bench_decode_timeline"):
        getattr(lib, name).restype = c_int
    _lib = lib
    return lib


def _check(status: int, what: str) -> None:
    if status != 0:
        raise MbqError(f"{what} failed with status {status}: {load().mbq_last_error().decode()}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise MbqError("tensors handed to libmbq must be contiguous device tensors")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def version() -> str:
    return load().mbq_version().decode()


def set_knob(knob: int, value: int) -> None:
    _check(load().mbq_set_knob(knob, value), "mbq_set_knob")


def blob_bytes(N: int, K: int) -> int:
    n = load().mbq_blob_bytes(N, K)
    if n == 0:
        raise MbqError(f"invalid shape: {load().mbq_last_error().decode()}")
    return n


def mbq_encode(W: torch.Tensor, blob: Optional[torch.Tensor] = None) -> torch.Tensor:
    """W fp32 [N, K] on the device -> packed blob (uint8 tensor)."""
    assert W.dtype == torch.float32 and W.dim() == 2
    N, K = W.shape
    if blob is None:
        blob = torch.empty(blob_bytes(N, K), dtype=torch.uint8, device=W.device)
    _check(load().mbq_encode(_ptr(W), N, K, _ptr(blob), _stream()), "mbq_encode")
    return blob


def mbq_encode_with_params(W: torch.Tensor, scale: torch.Tensor, zero: torch.Tensor,
                           blob: Optional[torch.Tensor] = None) -> torch.Tensor:
    """As mbq_encode, with the base-slice scale and zero point (fp32 [N, K/128]) given instead of fitted."""
    assert W.dtype == torch.float32 and W.dim() == 2
    N, K = W.shape
    assert scale.dtype == zero.dtype == torch.float32 and tuple(scale.shape) == tuple(zero.shape) == (N, K // 128)
    assert scale.is_contiguous() and zero.is_contiguous() and W.is_contiguous()
    if blob is None:
        blob = torch.empty(blob_bytes(N, K), dtype=torch.uint8, device=W.device)
    _check(load().mbq_encode_with_params(_ptr(W), N, K, _ptr(scale), _ptr(zero), _ptr(blob), _stream()),
           "mbq_encode_with_params")
    return blob


def mbq_unpack(blob: torch.Tensor, N: int, K: int) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """blob -> (codes uint8 [4, N, K], s0 fp32 [N, K/128], z0 fp32 [N, K/128])."""
    codes = torch.empty((4, N, K), dtype=torch.uint8, device=blob.device)
    s0 = torch.empty((N, K // GROUP), dtype=torch.float32, device=blob.device)
    z0 = torch.empty((N, K // GROUP), dtype=torch.float32, device=blob.device)
    _check(load().mbq_unpack(_ptr(blob), N, K, _ptr(codes), _ptr(s0), _ptr(z0), _stream()), "mbq_unpack")
    return codes, s0, z0


def mbq_dequant(blob: torch.Tensor, N: int, K: int, p: int) -> torch.Tensor:
    out = torch.empty((N, K), dtype=torch.float32, device=blob.device)
    _check(load().mbq_dequant(_ptr(blob), N, K, p, _ptr(out), _stream()), "mbq_dequant")
    return out


def route_workspace(T: int, K: int, device) -> torch.Tensor:
    # the call clears the counters it keeps there itself: the contents do not matter
    return torch.empty(load().mbq_route_workspace_bytes(T, K), dtype=torch.uint8, device=device)


def linear_workspace(T: int, N: int, K: int, device) -> torch.Tensor:
    return torch.empty(load().mbq_linear_workspace_bytes(T, N, K), dtype=torch.uint8, device=device)


def mbq_route(X: torch.Tensor, Wr: torch.Tensor, br: torch.Tensor, want_logits: bool = False,
              out: Optional[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]] = None,
              ws: Optional[torch.Tensor] = None):
    """X bf16 [T, K], Wr fp32 [4, K], br fp32 [4] -> (prec, perm, offsets[, logits fp64])."""
    assert X.dtype == torch.bfloat16 and Wr.dtype == torch.float32 and br.dtype == torch.float32
    T, K = X.shape
    P = Wr.shape[0]
    dev = X.device
    if out is None:
        prec = torch.empty(T, dtype=torch.int32, device=dev)
        perm = torch.empty(T, dtype=torch.int32, device=dev)
        offsets = torch.empty(P + 1, dtype=torch.int32, device=dev)
    else:
        prec, perm, offsets = out
    logits = torch.empty((T, P), dtype=torch.float64, device=dev) if want_logits else None
    if ws is None:
        ws = route_workspace(T, K, dev)
    _check(load().mbq_route(_ptr(X), T, K, _ptr(Wr), _ptr(br), P, _ptr(prec), _ptr(perm), _ptr(offsets),
                            _ptr(logits), _ptr(ws), ws.numel(), _stream()), "mbq_route")
    return (prec, perm, offsets, logits) if want_logits else (prec, perm, offsets)


def route_mlp_workspace(T: int, K: int, H: int, device) -> torch.Tensor:
    """Workspace of mbq_route_mlp (ticket counter, cleared by the call, + hidden layer)."""
    n = load().mbq_route_mlp_workspace_bytes(T, K, H)
    return torch.empty(max(int(n), 256), dtype=torch.uint8, device=device)


def mbq_route_mlp(X: torch.Tensor, W1: torch.Tensor, b1: torch.Tensor, W2: torch.Tensor, b2: torch.Tensor,
                  delta: float, want_scores: bool = False,
                  out: Optional[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]] = None,
                  ws: Optional[torch.Tensor] = None):
    """The 2-layer router with a run-time threshold: X bf16 [T, K], W1 fp32 [H, K], b1 [H], W2 fp32 [4, H],
    b2 [4] -> (prec, perm, offsets[, scores fp64 [T, 4]])."""
    assert X.dtype == torch.bfloat16 and all(t.dtype == torch.float32 for t in (W1, b1, W2, b2))
    T, K = X.shape
    H, E = W1.shape[0], W2.shape[0]
    assert W1.shape == (H, K) and b1.shape == (H,) and W2.shape == (E, H) and b2.shape == (E,)
    dev = X.device
    if out is None:
        prec = torch.empty(T, dtype=torch.int32, device=dev)
        perm = torch.empty(T, dtype=torch.int32, device=dev)
        offsets = torch.empty(E + 1, dtype=torch.int32, device=dev)
    else:
        prec, perm, offsets = out
    scores = torch.empty((T, E), dtype=torch.float64, device=dev) if want_scores else None
    if ws is None:
        ws = route_mlp_workspace(T, K, H, dev)
    _check(load().mbq_route_mlp(_ptr(X), T, K, _ptr(W1), _ptr(b1), H, _ptr(W2), _ptr(b2), E, float(delta),
                                _ptr(prec), _ptr(perm), _ptr(offsets), _ptr(scores), _ptr(ws), ws.numel(),
                                _stream()), "mbq_route_mlp")
    return (prec, perm, offsets, scores) if want_scores else (prec, perm, offsets)


def mbq_threshold_quantile(scores: torch.Tensor, rho: float, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """scores fp64 [T, 4] (device) -> one-element fp64 device tensor: the threshold that leaves a fraction rho of
    the residual-slice scores active."""
    assert scores.dtype == torch.float64 and scores.dim() == 2 and scores.is_contiguous()
    T, E = scores.shape
    if out is None:
        out = torch.empty(1, dtype=torch.float64, device=scores.device)
    _check(load().mbq_threshold_quantile(_ptr(scores), T, E, float(rho), _ptr(out), _stream()),
           "mbq_threshold_quantile")
    return out


def _ptr_array(tensors: Sequence[torch.Tensor]):
    """Host array of device pointers (void* [n])."""
    return (ctypes.c_void_p * len(tensors))(*[_ptr(t) for t in tensors])


def mbq_route_group(X: torch.Tensor, Wr: Sequence[torch.Tensor], br: Sequence[torch.Tensor],
                    out: Optional[Sequence[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]]] = None,
                    ws: Optional[torch.Tensor] = None) -> List[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]]:
    """Several routers over the same X bf16 [T, K] -> [(prec, perm, offsets)] per router."""
    assert X.dtype == torch.bfloat16 and len(Wr) == len(br) and len(Wr) >= 1
    T, K = X.shape
    dev = X.device
    n = len(Wr)
    P = Wr[0].shape[0]
    for w, b in zip(Wr, br):
        assert w.dtype == torch.float32 and b.dtype == torch.float32 and tuple(w.shape) == (P, K)
    if out is None:
        out = [(torch.empty(T, dtype=torch.int32, device=dev), torch.empty(T, dtype=torch.int32, device=dev),
                torch.empty(P + 1, dtype=torch.int32, device=dev)) for _ in range(n)]
    if ws is None:
        ws = route_workspace(T, K, dev)
    _check(load().mbq_route_group(_ptr(X), T, K, n, _ptr_array(Wr), _ptr_array(br), P,
                                  _ptr_array([o[0] for o in out]), _ptr_array([o[1] for o in out]),
                                  _ptr_array([o[2] for o in out]), _ptr(ws), ws.numel(), _stream()),
           "mbq_route_group")
    return [tuple(o) for o in out]


def mbq_linear(X: torch.Tensor, blob: torch.Tensor, N: int, K: int, prec: torch.Tensor, perm: torch.Tensor,
               offsets: torch.Tensor, Y: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None,
               algo: int = ALGO_AUTO) -> torch.Tensor:
    """Routed output Y fp32 [T, N] in original token order."""
    assert X.dtype == torch.bfloat16 and X.dim() == 2 and X.shape[1] == K
    T = X.shape[0]
    if Y is None:
        Y = torch.empty((T, N), dtype=torch.float32, device=X.device)
    if ws is None:
        ws = linear_workspace(T, N, K, X.device)
    _check(load().mbq_linear(_ptr(X), T, _ptr(blob), N, K, _ptr(prec), _ptr(perm), _ptr(offsets), _ptr(Y),
                             _ptr(ws), ws.numel(), algo, _stream()), "mbq_linear")
    return Y


def mbq_linear_static(X: torch.Tensor, blob: torch.Tensor, N: int, K: int, prec: torch.Tensor, perm: torch.Tensor,
                      offsets: torch.Tensor, Y: torch.Tensor, algo: int = ALGO_AUTO) -> torch.Tensor:
    """mbq_linear on the library's built-in scratch buffer: no allocation anywhere (Y is the caller's)."""
    assert X.dtype == torch.bfloat16 and X.dim() == 2 and X.shape[1] == K
    _check(load().mbq_linear_static(_ptr(X), X.shape[0], _ptr(blob), N, K, _ptr(prec), _ptr(perm), _ptr(offsets),
                                    _ptr(Y), algo, _stream()), "mbq_linear_static")
    return Y


def mbq_linear_group(X: torch.Tensor, blobs: Sequence[torch.Tensor], Ns: Sequence[int], K: int,
                     routing: Sequence[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]],
                     Y: Optional[Sequence[torch.Tensor]] = None, ws: Optional[torch.Tensor] = None,
                     algo: int = ALGO_AUTO) -> List[torch.Tensor]:
    """Routed outputs of several matrices over the same X; routing[i] = (prec, perm, offsets) of matrix i."""
    assert X.dtype == torch.bfloat16 and X.dim() == 2 and X.shape[1] == K
    assert len(blobs) == len(Ns) == len(routing) >= 1
    T = X.shape[0]
    if Y is None:
        Y = [torch.empty((T, N), dtype=torch.float32, device=X.device) for N in Ns]
    if ws is None:
        ws = linear_workspace(T, max(Ns), K, X.device)
    n_arr = (ctypes.c_int64 * len(Ns))(*[int(N) for N in Ns])
    _check(load().mbq_linear_group(_ptr(X), T, K, len(Ns), _ptr_array(blobs), n_arr,
                                   _ptr_array([r[0] for r in routing]), _ptr_array([r[1] for r in routing]),
                                   _ptr_array([r[2] for r in routing]), _ptr_array(Y), _ptr(ws), ws.numel(), algo,
                                   _stream()), "mbq_linear_group")
    return list(Y)


def mbq_routed_linear_group(X: torch.Tensor, Wr: Sequence[torch.Tensor], br: Sequence[torch.Tensor],
                            blobs: Sequence[torch.Tensor], Ns: Sequence[int],
                            routing: Optional[Sequence[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]]] = None,
                            Y: Optional[Sequence[torch.Tensor]] = None, ws_route: Optional[torch.Tensor] = None,
                            ws_linear: Optional[torch.Tensor] = None, algo: int = ALGO_AUTO):
    """One stage: route X with every router, then the routed outputs.  -> (routing, Y) lists."""
    assert X.dtype == torch.bfloat16 and X.dim() == 2
    T, K = X.shape
    n = len(Ns)
    assert len(Wr) == len(br) == len(blobs) == n >= 1
    P = Wr[0].shape[0]
    dev = X.device
    if routing is None:
        routing = [(torch.empty(T, dtype=torch.int32, device=dev), torch.empty(T, dtype=torch.int32, device=dev),
                    torch.empty(P + 1, dtype=torch.int32, device=dev)) for _ in range(n)]
    if Y is None:
        Y = [torch.empty((T, N), dtype=torch.float32, device=dev) for N in Ns]
    if ws_route is None:
        ws_route = route_workspace(T, K, dev)
    if ws_linear is None:
        ws_linear = linear_workspace(T, max(Ns), K, dev)
    n_arr = (ctypes.c_int64 * n)(*[int(N) for N in Ns])
    _check(load().mbq_routed_linear_group(
        _ptr(X), T, K, n, _ptr_array(Wr), _ptr_array(br), P, _ptr_array(blobs), n_arr,
        _ptr_array([r[0] for r in routing]), _ptr_array([r[1] for r in routing]),
        _ptr_array([r[2] for r in routing]), _ptr_array(Y), _ptr(ws_route), ws_route.numel(), _ptr(ws_linear),
        ws_linear.numel(), algo, _stream()), "mbq_routed_linear_group")
    return [tuple(r) for r in routing], list(Y)


# ---- other slice configurations ----------------------------------------------------------------------

def config_check(cfg: Config) -> None:
    _check(load().mbq_config_check(ctypes.byref(cfg)), "mbq_config_check")


def config_bits(cfg: Config, p: int) -> int:
    return int(load().mbq_config_bits(ctypes.byref(cfg), p))


def config_precision_value(cfg: Config, p: int) -> int:
    """What a prec array holds for the configuration's precision p."""
    return int(load().mbq_config_precision_value(ctypes.byref(cfg), p))


def config_counts_bits(cfg: Config) -> bool:
    return int(load().mbq_config_counts_bits(ctypes.byref(cfg))) == 1


def mbq_linear_cfg(X: torch.Tensor, blob: torch.Tensor, N: int, K: int, cfg: Config, prec: torch.Tensor,
                   perm: Optional[torch.Tensor] = None, offsets: Optional[torch.Tensor] = None,
                   Y: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None,
                   algo: int = ALGO_AUTO) -> torch.Tensor:
    """mbq_linear on precision arrays written under a configuration."""
    T = X.shape[0]
    if Y is None:
        Y = torch.empty((T, N), dtype=torch.float32, device=X.device)
    if ws is None:
        ws = linear_workspace(T, N, K, X.device)
    _check(load().mbq_linear_cfg(_ptr(X), T, _ptr(blob), N, K, ctypes.byref(cfg), _ptr(prec), _ptr(perm),
                                 _ptr(offsets), _ptr(Y), _ptr(ws), ws.numel(), algo, _stream()), "mbq_linear_cfg")
    return Y


def blob_bytes_cfg(cfg: Config, N: int, K: int) -> int:
    n = int(load().mbq_blob_bytes_cfg(ctypes.byref(cfg), N, K))
    if n == 0:
        raise MbqError(f"mbq_blob_bytes_cfg: {load().mbq_last_error().decode()}")
    return n


def mbq_encode_cfg(W: torch.Tensor, cfg: Config, blob: Optional[torch.Tensor] = None) -> torch.Tensor:
    assert W.dtype == torch.float32 and W.dim() == 2
    N, K = W.shape
    if blob is None:
        blob = torch.empty(blob_bytes_cfg(cfg, N, K), dtype=torch.uint8, device=W.device)
    _check(load().mbq_encode_cfg(_ptr(W.contiguous()), N, K, ctypes.byref(cfg), _ptr(blob), _stream()),
           "mbq_encode_cfg")
    return blob


def mbq_unpack_cfg(blob: torch.Tensor, N: int, K: int, cfg: Config):
    """-> (codes uint8 [E, N, K], scale fp32 [N, K/group], zero fp32 [N, K/group]) in the configuration's terms."""
    codes = torch.empty((cfg.n_slices, N, K), dtype=torch.uint8, device=blob.device)
    scale = torch.empty((N, K // cfg.group), dtype=torch.float32, device=blob.device)
    zero = torch.empty_like(scale)
    _check(load().mbq_unpack_cfg(_ptr(blob), N, K, ctypes.byref(cfg), _ptr(codes), _ptr(scale), _ptr(zero), _stream()),
           "mbq_unpack_cfg")
    return codes, scale, zero


def mbq_dequant_cfg(blob: torch.Tensor, N: int, K: int, cfg: Config, p: int) -> torch.Tensor:
    What = torch.empty((N, K), dtype=torch.float32, device=blob.device)
    _check(load().mbq_dequant_cfg(_ptr(blob), N, K, ctypes.byref(cfg), p, _ptr(What), _stream()), "mbq_dequant_cfg")
    return What


def mbq_route_cfg(X: torch.Tensor, Wr: torch.Tensor, br: torch.Tensor, cfg: Config, want_logits: bool = False,
                  ws: Optional[torch.Tensor] = None):
    """X bf16 [T, K], Wr fp32 [E, K], br fp32 [E] -> (prec (digit precisions), perm, offsets[5][, logits [T, E]])."""
    assert X.dtype == torch.bfloat16 and Wr.dtype == torch.float32 and br.dtype == torch.float32
    T, K = X.shape
    assert Wr.shape == (cfg.n_slices, K) and br.shape == (cfg.n_slices,)
    dev = X.device
    prec = torch.empty(T, dtype=torch.int32, device=dev)
    perm = torch.empty(T, dtype=torch.int32, device=dev)
    offsets = torch.empty(N_PRECISIONS + 1, dtype=torch.int32, device=dev)
    logits = torch.empty((T, cfg.n_slices), dtype=torch.float64, device=dev) if want_logits else None
    if ws is None:
        ws = route_workspace(T, K, dev)
    _check(load().mbq_route_cfg(_ptr(X), T, K, _ptr(Wr), _ptr(br), ctypes.byref(cfg), _ptr(prec), _ptr(perm),
                                _ptr(offsets), _ptr(logits), _ptr(ws), ws.numel(), _stream()), "mbq_route_cfg")
    return (prec, perm, offsets, logits) if want_logits else (prec, perm, offsets)


def mbq_route_group_cfg(X: torch.Tensor, Wr: Sequence[torch.Tensor], br: Sequence[torch.Tensor], cfg: Config,
                        ws: Optional[torch.Tensor] = None):
    T, K = X.shape
    n = len(Wr)
    dev = X.device
    routing = [(torch.empty(T, dtype=torch.int32, device=dev), torch.empty(T, dtype=torch.int32, device=dev),
                torch.empty(N_PRECISIONS + 1, dtype=torch.int32, device=dev)) for _ in range(n)]
    if ws is None:
        ws = route_workspace(T, K, dev)
    _check(load().mbq_route_group_cfg(_ptr(X), T, K, n, _ptr_array(Wr), _ptr_array(br), ctypes.byref(cfg),
                                      _ptr_array([r[0] for r in routing]), _ptr_array([r[1] for r in routing]),
                                      _ptr_array([r[2] for r in routing]), _ptr(ws), ws.numel(), _stream()),
           "mbq_route_group_cfg")
    return routing


def mbq_routed_linear_group_cfg(X: torch.Tensor, Wr: Sequence[torch.Tensor], br: Sequence[torch.Tensor], cfg: Config,
                                blobs: Sequence[torch.Tensor], Ns: Sequence[int],
                                routing: Optional[Sequence[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]]] = None,
                                Y: Optional[Sequence[torch.Tensor]] = None, ws_route: Optional[torch.Tensor] = None,
                                ws_linear: Optional[torch.Tensor] = None, algo: int = ALGO_AUTO):
    """One stage under a slice configuration: route X with every E-output router, then the routed outputs."""
    assert X.dtype == torch.bfloat16 and X.dim() == 2
    T, K = X.shape
    n = len(Ns)
    dev = X.device
    if routing is None:
        routing = [(torch.empty(T, dtype=torch.int32, device=dev), torch.empty(T, dtype=torch.int32, device=dev),
                    torch.empty(N_PRECISIONS + 1, dtype=torch.int32, device=dev)) for _ in range(n)]
    if Y is None:
        Y = [torch.empty((T, N), dtype=torch.float32, device=dev) for N in Ns]
    if ws_route is None:
        ws_route = route_workspace(T, K, dev)
    if ws_linear is None:
        ws_linear = linear_workspace(T, max(Ns), K, dev)
    n_arr = (ctypes.c_int64 * n)(*[int(N) for N in Ns])
    _check(load().mbq_routed_linear_group_cfg(
        _ptr(X), T, K, n, _ptr_array(Wr), _ptr_array(br), ctypes.byref(cfg), _ptr_array(blobs), n_arr,
        _ptr_array([r[0] for r in routing]), _ptr_array([r[1] for r in routing]),
        _ptr_array([r[2] for r in routing]), _ptr_array(Y), _ptr(ws_route), ws_route.numel(), _ptr(ws_linear),
        ws_linear.numel(), algo, _stream()), "mbq_routed_linear_group_cfg")
    return [tuple(r) for r in routing], list(Y)


# ---- measurement and diagnostic entry points (include/mbq_bench.h) ----------------------------------

def bench_copy(src: torch.Tensor, dst: torch.Tensor, width: int = 1) -> None:
    """dst = src by the library's plain streaming copy kernel (uint8 tensors of equal size)."""
    assert src.numel() * src.element_size() == dst.numel() * dst.element_size()
    _check(load().mbq_bench_copy(_ptr(src), _ptr(dst), src.numel() * src.element_size(), width, _stream()),
           "mbq_bench_copy")


def bench_read(src: torch.Tensor, sink: torch.Tensor, width: int = 1, nbytes: Optional[int] = None) -> None:
    n = src.numel() * src.element_size() if nbytes is None else nbytes
    _check(load().mbq_bench_read(_ptr(src), n, width, _ptr(sink), _stream()), "mbq_bench_read")


def bench_mfma_loop(steps: int, with_barrier: bool, sink: torch.Tensor) -> float:
    """Enqueues the LDS-fed MFMA loop; returns the flops of the launch."""
    flops = ctypes.c_double(0.0)
    _check(load().mbq_bench_mfma_loop(steps, 1 if with_barrier else 0, _ptr(sink), ctypes.byref(flops), _stream()),
           "mbq_bench_mfma_loop")
    return flops.value


def bench_linear_group_prepared(T: int, K: int, blobs: Sequence[torch.Tensor], Ns: Sequence[int],
                                routing: Sequence[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]],
                                Y: Sequence[torch.Tensor], ws: torch.Tensor) -> None:
    """The T <= 16 linear kernel alone on a workspace prepared by an earlier call (timing only)."""
    n_arr = (ctypes.c_int64 * len(Ns))(*[int(N) for N in Ns])
    _check(load().mbq_bench_linear_group_prepared(T, K, len(Ns), _ptr_array(blobs), n_arr,
                                                  _ptr_array([r[0] for r in routing]), _ptr_array(Y), _ptr(ws),
                                                  ws.numel(), _stream()), "mbq_bench_linear_group_prepared")


def bench_decode_timeline(T: int, K: int, blobs: Sequence[torch.Tensor], Ns: Sequence[int],
                          routing: Sequence[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]],
                          Y: Sequence[torch.Tensor], ws: torch.Tensor) -> torch.Tensor:
    """The same launch from the timeline build; -> int64 tensor [workgroups, wavefronts, 32 slots] of 100 MHz
    clock stamps (layout in include/mbq_bench.h)."""
    lib = load()
    wgs = lib.mbq_bench_decode_timeline_workgroups()
    nbytes = lib.mbq_bench_decode_timeline_bytes()
    stamps = torch.zeros(nbytes // 8, dtype=torch.int64, device=ws.device)
    n_arr = (ctypes.c_int64 * len(Ns))(*[int(N) for N in Ns])
    _check(lib.mbq_bench_decode_timeline(T, K, len(Ns), _ptr_array(blobs), n_arr,
                                         _ptr_array([r[0] for r in routing]), _ptr_array(Y), _ptr(ws), ws.numel(),
                                         _ptr(stamps), nbytes, _stream()), "mbq_bench_decode_timeline")
    return stamps.view(wgs, -1, 32)


def mbq_act_quant(X: torch.Tensor, abits: int = 4, let_shift: Optional[torch.Tensor] = None,
                  let_scale: Optional[torch.Tensor] = None, want_router_input: bool = True, out=None):
    """X bf16 [T, K] -> (Xint bf16 [T, K] integers, row_scale fp32 [T], Xr bf16 [T, K] or None); App. E.4.
    out: (Xint, row_scale, Xr) buffers to write into instead of new ones."""
    assert X.dtype == torch.bfloat16 and X.dim() == 2 and X.is_contiguous()
    T, K = X.shape
    if out is not None:
        Xint, row_scale, Xr = out
    else:
        Xint = torch.empty_like(X)
        row_scale = torch.empty((T,), dtype=torch.float32, device=X.device)
        Xr = torch.empty_like(X) if want_router_input else None
    _check(load().mbq_act_quant(_ptr(X), T, K, abits, _ptr(let_shift), _ptr(let_scale), _ptr(Xint), _ptr(row_scale),
                                _ptr(Xr), _stream()), "mbq_act_quant")
    return Xint, row_scale, Xr


def mbq_scale_rows(Y: torch.Tensor, row_scale: torch.Tensor, bias: Optional[torch.Tensor] = None) -> torch.Tensor:
    """In place: Y[i, n] = Y[i, n] * row_scale[i] (+ bias[n])."""
    assert Y.dtype == torch.float32 and Y.dim() == 2 and Y.is_contiguous()
    T, N = Y.shape
    _check(load().mbq_scale_rows(_ptr(Y), T, N, _ptr(row_scale), _ptr(bias), _stream()), "mbq_scale_rows")
    return Y


def mbq_routed_linear_group_act(X: torch.Tensor, abits: int, let_shift: Optional[torch.Tensor],
                                let_scale: Optional[torch.Tensor], Wr: Sequence[torch.Tensor],
                                br: Sequence[torch.Tensor], blobs: Sequence[torch.Tensor], Ns: Sequence[int],
                                bias: Optional[Sequence[Optional[torch.Tensor]]] = None, routing=None, Y=None, act=None,
                                ws_route: Optional[torch.Tensor] = None, ws_linear: Optional[torch.Tensor] = None,
                                algo: int = ALGO_AUTO):
    """One stage of the activation-quantised variant (App. E.4) -> (routing, Y, (Xint, row_scale, Xr))."""
    assert X.dtype == torch.bfloat16 and X.dim() == 2 and X.is_contiguous()
    T, K = X.shape
    n = len(Ns)
    dev = X.device
    P = Wr[0].shape[0]
    if routing is None:
        routing = [(torch.empty(T, dtype=torch.int32, device=dev), torch.empty(T, dtype=torch.int32, device=dev),
                    torch.empty(P + 1, dtype=torch.int32, device=dev)) for _ in range(n)]
    if Y is None:
        Y = [torch.empty((T, N), dtype=torch.float32, device=dev) for N in Ns]
    if act is None:
        act = (torch.empty_like(X), torch.empty((T,), dtype=torch.float32, device=dev), torch.empty_like(X))
    if ws_route is None:
        ws_route = route_workspace(T, K, dev)
    if ws_linear is None:
        ws_linear = linear_workspace(T, max(Ns), K, dev)
    n_arr = (ctypes.c_int64 * n)(*[int(N) for N in Ns])
    bias_arr = None if bias is None else (ctypes.c_void_p * n)(*[_ptr(b) for b in bias])
    _check(load().mbq_routed_linear_group_act(
        _ptr(X), T, K, abits, _ptr(let_shift), _ptr(let_scale), n, _ptr_array(Wr), _ptr_array(br), P,
        _ptr_array(blobs), n_arr, bias_arr, _ptr_array([r[0] for r in routing]), _ptr_array([r[1] for r in routing]),
        _ptr_array([r[2] for r in routing]), _ptr_array(Y), _ptr(act[0]), _ptr(act[1]), _ptr(act[2]), _ptr(ws_route),
        ws_route.numel(), _ptr(ws_linear), ws_linear.numel(), algo, _stream()), "mbq_routed_linear_group_act")
    return [tuple(r) for r in routing], list(Y), act
