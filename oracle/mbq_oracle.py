"""Plain CPU oracle (numpy, fp64) for MoBiQuant's token-routed any-precision linear.

TEST INFRASTRUCTURE ONLY.  This module is the slow, obviously-correct statement of
what the hot path computes, written from the paper; it shares no code, tables or
helpers with the HIP library and must never be imported by the product path.
Every function is pinned by the CPU tests (error bound, nesting, closed forms,
brute force in exact rational arithmetic, library matmul / sort); nothing here is
"parity unpinned".

Notation (0-based, as in the library): slices e = 0..3 of 2 bits each, precision
index p in {0,1,2,3} <-> 2(p+1) bits <-> slices 0..p.  The paper's 1-based slices
W_1..W_E are our slices 0..3.  Weight ``W`` is ``N x K`` (output x input features),
quantisation groups are 128 consecutive input features of one output row.

Readings of the paper taken here (the paper is silent or inconsistent on them):
  * scale ratio between consecutive slices is 2^{b_e} = 4 (App. B "MoBiSlice
    construction", scale refinement), not 2^{b_e - 1} as Sec. 4.1 words it: only
    the former makes the merged-code identity and the half-step bound hold;
  * (s0, z0) of the base slice come from a plain asymmetric min/max fit with
    s0 = (max - min) / 4 so that four floor-aligned bins tile [min, max];
    z0 = -min / s0 is a continuous (non-integer) zero point; both stored fp32;
  * degenerate groups (max == min) get a range floor, see ``group_params``;
  * the router is a single linear map to 4 logits, argmax picks the precision,
    first maximum wins ties;
  * the paper's own router (``route_mlp``): a 2-layer MLP whose hidden width and
    activation the paper does not give - taken as ReLU between two affine maps; one
    score per slice, slice e active iff score - delta > 0 (Sec. 4.2, runtime
    threshold), the base slice always active (shared-expert slice), and - because
    the precision of a token is a prefix of slices - precision = number of leading
    active residual slices (an active slice after an inactive one is ignored).
"""
from __future__ import annotations

import numpy as np

GROUP = 128          # input features per quantisation group   (App. C.1)
N_SLICES = 4         # E                                       (Sec. 4.1, default)
SLICE_BITS = 2       # b_e                                     (Sec. 4.1, default)
LEVELS = 1 << SLICE_BITS
RESIDUAL_ZERO = float(1 << (SLICE_BITS - 1))   # z_e = 2^{b_e-1} for e >= 1 (App. B)

__all__ = [
    "GROUP", "N_SLICES", "SLICE_BITS",
    "bf16_bits_to_f64", "group_params", "encode", "encode_digits", "slice_matrix",
    "dequant", "merged_code", "dequant_merged", "pack_canonical", "unpack_canonical",
    "blob_bytes", "pack_blob", "route", "bucket", "linear", "avg_bits",
    "route_mlp", "threshold_quantile",
]


# ----------------------------------------------------------------------------- inputs
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> exact fp64 values."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


# ----------------------------------------------------------------------------- encode
def group_params(W: np.ndarray):
    """Base-slice scale and continuous zero point per (row, group), fp32.

    Min/max fit of the floor-aligned 2-bit quantiser of App. B: four bins of width
    s0 tile [lo, hi], so s0 = (hi - lo)/4 and z0 = -lo/s0 (then lo maps to code 0
    and hi sits on the top edge, which the clamp folds into code 3).  All three
    operations are single fp32 operations (subtract, divide by 4, IEEE divide).
    A constant group has no range; its range is floored at 2^-16 of its magnitude
    (and at 2^-100) so that z0 stays finite.
    """
    W = np.ascontiguousarray(W, dtype=np.float32)
    N, K = W.shape
    assert K % GROUP == 0
    Wg = W.reshape(N, K // GROUP, GROUP)
    lo = Wg.min(axis=2)
    hi = Wg.max(axis=2)
    rng = (hi - lo).astype(np.float32)
    mag = np.maximum(np.abs(lo), np.abs(hi)).astype(np.float32)
    floor_rng = np.maximum(mag * np.float32(2.0 ** -16), np.float32(2.0 ** -100)).astype(np.float32)
    rng = np.maximum(rng, floor_rng).astype(np.float32)
    s0 = (rng / np.float32(4.0)).astype(np.float32)
    z0 = ((-lo).astype(np.float32) / s0).astype(np.float32)
    return s0, z0


def encode(W: np.ndarray, s0: np.ndarray = None, z0: np.ndarray = None):
    """Recursive residual quantisation (Sec. 4.1 Eq. 2 with the quantiser of App. B).

    R_0 = W;  for e = 0..3:  s_e = s0 / 4^e,  z_e = z0 (e = 0) or 2 (e >= 1),
        c_e = clamp(floor(R_e / s_e + z_e), 0, 3)
        R_{e+1} = R_e - s_e * (c_e - z_e + 0.5)
    evaluated in fp64 exactly in this order (divide, add, floor, clamp; subtract,
    add, multiply, subtract) from the stored fp32 (s0, z0).

    Returns codes uint8 [4, N, K], s0 fp32 [N, G], z0 fp32 [N, G].
    """
    W = np.ascontiguousarray(W, dtype=np.float32)
    N, K = W.shape
    if s0 is None:
        s0, z0 = group_params(W)
    G = K // GROUP
    s0d = np.repeat(s0.astype(np.float64), GROUP, axis=1)
    z0d = np.repeat(z0.astype(np.float64), GROUP, axis=1)
    R = W.astype(np.float64)
    codes = np.empty((N_SLICES, N, K), dtype=np.uint8)
    for e in range(N_SLICES):
        s_e = s0d / float(LEVELS ** e)
        z_e = z0d if e == 0 else RESIDUAL_ZERO
        q = np.floor(R / s_e + z_e)
        c = np.clip(q, 0.0, float(LEVELS - 1))
        codes[e] = c.astype(np.uint8)
        R = R - s_e * ((c - z_e) + 0.5)
    assert s0.shape == (N, G)
    return codes, s0, z0


def encode_digits(W: np.ndarray, s0: np.ndarray, z0: np.ndarray) -> np.ndarray:
    """Closed form of ``encode`` (App. B, merged-code identity): with
    u = W/s0 + z0 the codes are the base-4 digits of clamp(floor(64 u), 0, 255).
    Used only as a cross-check of the recursion; it may differ from it within
    rounding of a bin edge."""
    W = np.ascontiguousarray(W, dtype=np.float32).astype(np.float64)
    N, K = W.shape
    s0d = np.repeat(s0.astype(np.float64), GROUP, axis=1)
    z0d = np.repeat(z0.astype(np.float64), GROUP, axis=1)
    top = float(LEVELS ** N_SLICES)
    full = np.clip(np.floor((W / s0d + z0d) * (top / LEVELS)), 0.0, top - 1.0).astype(np.int64)
    codes = np.empty((N_SLICES, N, K), dtype=np.uint8)
    for e in range(N_SLICES):
        codes[e] = (full >> (SLICE_BITS * (N_SLICES - 1 - e))) & (LEVELS - 1)
    return codes


# ---------------------------------------------------------------------------- dequant
def slice_matrix(codes: np.ndarray, s0: np.ndarray, z0: np.ndarray, e: int) -> np.ndarray:
    """W_e = s_e (c_e - z_e + 0.5), fp64 [N, K]  (App. B dequantiser, slice e)."""
    s_e = np.repeat(s0.astype(np.float64), GROUP, axis=1) / float(LEVELS ** e)
    z_e = np.repeat(z0.astype(np.float64), GROUP, axis=1) if e == 0 else RESIDUAL_ZERO
    return s_e * ((codes[e].astype(np.float64) - z_e) + 0.5)


def dequant(codes: np.ndarray, s0: np.ndarray, z0: np.ndarray, p: int) -> np.ndarray:
    """W^(p) = sum_{e <= p} W_e   (Sec. 4.1 Eq. 3)."""
    out = slice_matrix(codes, s0, z0, 0)
    for e in range(1, p + 1):
        out = out + slice_matrix(codes, s0, z0, e)
    return out


def merged_code(codes: np.ndarray, p: int) -> np.ndarray:
    """I_p = sum_{e <= p} c_e 4^{p-e}: the (2p+2)-bit code whose digits are slices 0..p."""
    I = np.zeros(codes.shape[1:], dtype=np.int64)
    for e in range(p + 1):
        I = I * LEVELS + codes[e].astype(np.int64)
    return I


def dequant_merged(codes: np.ndarray, s0: np.ndarray, z0: np.ndarray, p: int) -> np.ndarray:
    """Closed form of ``dequant`` (App. B, Eq. for the merged code generalised to p+1
    slices): W^(p) = s_p (I_p - 4^p z0 + 0.5), s_p = s0 / 4^p."""
    s_p = np.repeat(s0.astype(np.float64), GROUP, axis=1) / float(LEVELS ** p)
    z_p = np.repeat(z0.astype(np.float64), GROUP, axis=1) * float(LEVELS ** p)
    return s_p * ((merged_code(codes, p).astype(np.float64) - z_p) + 0.5)


# ---------------------------------------------------------------------------- packing
def pack_canonical(codes: np.ndarray) -> np.ndarray:
    """Canonical bit-major packing: per slice, row-major over (n, k), 16 codes per
    little-endian uint32, code k at bits 2*(k mod 16).  uint32 [4, N, K/16]."""
    E, N, K = codes.shape
    assert K % 16 == 0
    c = codes.reshape(E, N, K // 16, 16).astype(np.uint32)
    shifts = (np.arange(16, dtype=np.uint32) * np.uint32(SLICE_BITS))
    return np.bitwise_or.reduce(c << shifts, axis=3).astype(np.uint32)


def unpack_canonical(words: np.ndarray) -> np.ndarray:
    E, N, Kw = words.shape
    shifts = (np.arange(16, dtype=np.uint32) * np.uint32(SLICE_BITS))
    c = (words[..., None] >> shifts) & np.uint32(LEVELS - 1)
    return c.reshape(E, N, Kw * 16).astype(np.uint8)


# The library's device blob (format documented in include/mbq.h, "Packed weight
# blob").  Re-stated here from that description so that the encoder's output can be
# compared byte for byte.
_TILE_N = 16
_TILE_K = 256


def blob_bytes(N: int, K: int) -> int:
    nt = -(-N // _TILE_N)
    kb = -(-K // _TILE_K)
    return N_SLICES * nt * kb * 1024 + nt * (2 * kb) * _TILE_N * 8


def pack_blob(codes: np.ndarray, s0: np.ndarray, z0: np.ndarray) -> np.ndarray:
    """Byte image of the packed weight blob for (codes, s0, z0)."""
    E, N, K = codes.shape
    assert E == N_SLICES and K % GROUP == 0
    nt = -(-N // _TILE_N)
    kb = -(-K // _TILE_K)
    Np, Kp = nt * _TILE_N, kb * _TILE_K
    cp = np.zeros((E, Np, Kp), dtype=np.uint32)
    cp[:, :N, :K] = codes
    # k = 256*kb + 64*d + 32*step + 8*kq + s ; n = 16*nt + nn ; lane = 16*kq + nn
    c = cp.reshape(E, nt, _TILE_N, kb, 4, 2, 4, 8)          # e, nt, nn, kb, d, step, kq, s
    c = c.transpose(0, 1, 3, 6, 2, 4, 5, 7)                   # e, nt, kb, kq, nn, d, step, s
    step = np.arange(2).reshape(2, 1)
    s = np.arange(8).reshape(1, 8)
    field = 16 * (s & 1) + 4 * (s >> 1) + 2 * step            # bit of the code in the unrotated word
    words = np.empty((E, nt, kb, 4, _TILE_N, 4), dtype=np.uint32)
    for e in range(E):
        rot = (2 - 2 * e) % 32                                 # slice e is stored rotated left by 2-2e
        sh = ((field + rot) % 32).astype(np.uint32)
        words[e] = np.bitwise_or.reduce(
            np.bitwise_or.reduce(c[e] << sh, axis=-1), axis=-1)
    code_bytes = words.reshape(-1).view(np.uint8)
    meta = np.zeros((nt, 2 * kb, _TILE_N, 2), dtype=np.float32)
    G = K // GROUP
    sp = np.zeros((Np, 2 * kb), dtype=np.float32)
    zp = np.zeros((Np, 2 * kb), dtype=np.float32)
    sp[:N, :G] = s0
    zp[:N, :G] = z0
    meta[..., 0] = sp.reshape(nt, _TILE_N, 2 * kb).transpose(0, 2, 1)
    meta[..., 1] = zp.reshape(nt, _TILE_N, 2 * kb).transpose(0, 2, 1)
    return np.concatenate([code_bytes, meta.reshape(-1).view(np.uint8)])


# ------------------------------------------------------------------------------ route
def route(x_bits: np.ndarray, Wr: np.ndarray, br: np.ndarray):
    """Router scores and precision choice (Sec. 4.2 Eq. 4, linear-router reading):
    S = X Wr^T + br in fp64, p_i = argmax_q S[i, q] (first maximum), gap_i = top1-top2.
    Returns (S fp64 [T, P], prec int32 [T], gap fp64 [T])."""
    X = bf16_bits_to_f64(x_bits)
    S = X @ Wr.astype(np.float64).T + br.astype(np.float64)[None, :]
    prec = np.argmax(S, axis=1).astype(np.int32)
    if S.shape[0]:
        srt = np.sort(S, axis=1)
        gap = srt[:, -1] - srt[:, -2]
    else:
        gap = np.zeros(0)
    return S, prec, gap


def route_mlp(x_bits: np.ndarray, W1: np.ndarray, b1: np.ndarray, W2: np.ndarray, b2: np.ndarray,
              delta: float):
    """The paper's router (Sec. 4.2 Eq. 4 and the runtime threshold of Sec. 4.2, last paragraph):
    S = relu(X W1^T + b1) W2^T + b2 in fp64, one score per slice (S is T x E);
    G[i, e] = 1[(S[i, e] - delta) > 0]; slice 0 is always active (shared-expert slice) and the
    precision of token i is the number of leading active residual slices e = 1, 2, ...
    Returns (S fp64 [T, E], prec int32 [T], margin fp64 [T]) where margin is the smallest
    |S - delta| among the comparisons that decided the token's precision."""
    X = bf16_bits_to_f64(x_bits)
    Hd = X @ W1.astype(np.float64).T + b1.astype(np.float64)[None, :]
    Hd = np.maximum(Hd, 0.0)
    S = Hd @ W2.astype(np.float64).T + b2.astype(np.float64)[None, :]
    T, E = S.shape
    prec = np.zeros(T, dtype=np.int32)
    margin = np.full(T, np.inf)
    for i in range(T):
        p = 0
        for e in range(1, E):
            d = S[i, e] - delta
            margin[i] = min(margin[i], abs(d))
            if d > 0:
                p = e
            else:
                break
        prec[i] = p
    return S, prec, margin


def threshold_quantile(S: np.ndarray, rho: float) -> float:
    """Layer-wise threshold calibration (App. C.2): the threshold that leaves a fraction rho of
    the residual-slice scores of a calibration batch active.  With M = T (E - 1) residual scores
    and k = floor(rho M + 1/2) (clipped to 0..M), the threshold is the (k+1)-th largest of them,
    so that exactly the k largest satisfy score - delta > 0 (ties aside); -inf if k = M."""
    R = np.sort(np.asarray(S, dtype=np.float64)[:, 1:].reshape(-1))[::-1]
    M = R.size
    k = int(np.floor(rho * M + 0.5))
    k = max(0, min(M, k))
    return float(R[k]) if k < M else float("-inf")


def bucket(prec: np.ndarray, n_prec: int = N_SLICES):
    """Token permutation after routing (Sec. 4.3, challenge 3): tokens grouped by
    precision, ascending precision, ascending token id inside a group.
    Returns (perm int32 [T], offsets int32 [P+1]); group q is perm[offsets[q]:offsets[q+1]]."""
    T = len(prec)
    perm = np.empty(T, dtype=np.int32)
    offsets = np.zeros(n_prec + 1, dtype=np.int32)
    pos = 0
    for q in range(n_prec):
        offsets[q] = pos
        for i in range(T):
            if prec[i] == q:
                perm[pos] = i
                pos += 1
    offsets[n_prec] = pos
    assert pos == T
    return perm, offsets


# ----------------------------------------------------------------------------- linear
def linear(x_bits: np.ndarray, codes: np.ndarray, s0: np.ndarray, z0: np.ndarray,
           prec: np.ndarray) -> np.ndarray:
    """Routed output (Sec. 4.2 Eq. 6 with the prefix mask G[i, e] = 1[e <= p_i]):
    Y_i = sum_e W_e^T (G[i, e] * X_i), fp64 [T, N]."""
    X = bf16_bits_to_f64(x_bits)
    T = X.shape[0]
    N = codes.shape[1]
    Y = np.zeros((T, N), dtype=np.float64)
    for e in range(N_SLICES):
        gate = (np.asarray(prec) >= e).astype(np.float64)[:, None]
        if not gate.any():
            continue
        Y += (gate * X) @ slice_matrix(codes, s0, z0, e).T
    return Y


def avg_bits(prec: np.ndarray) -> float:
    """AvgBits (Sec. 4.2 Eq. 8): mean over tokens of the bits of their active slices."""
    prec = np.asarray(prec)
    if prec.size == 0:
        return 0.0
    return float(np.mean((prec + 1) * SLICE_BITS))
