"""Seeded generators for the five synthetic workloads.

Recipe (all draws from ``numpy.random.default_rng`` with an explicit seed sequence
``[config seed, linear index, stream id, ...]`` so that every array can be rebuilt
independently of the others):

* weights  : ``W[n, k] = t_df * 0.02 * exp(0.3 * g_n)`` with ``t_df`` Student-t and
  ``g_n`` a standard normal per output row (heavy-tailed entries, log-normal row
  scale), stored fp32, shape ``N x K`` (out features x in features).
* tokens   : ``X ~ N(0, 1)``; optionally ``floor(frac * K)`` seeded *outlier
  channels* multiplied by 20, optionally a fraction of *outlier tokens*
  ``x = z + sqrt(99 K) v`` along one fixed unit direction ``v`` (row norm x10);
  rounded to bf16 (round-to-nearest-even) and returned as ``uint16`` bit patterns.
* router   : ``Wr ~ N(0, 1/K)`` (4 x K fp32).  For a uniform mix the bias is zero
  (the four rows are exchangeable).  For a target mix the bias is fitted on a
  seeded calibration draw from the same token distribution by iterating
  ``b_q += log(target_q / achieved_q)``.  With outlier tokens the random part of
  every router row is made orthogonal to ``v`` and the last row gets ``+2 v /
  sqrt(K)`` so that outlier tokens land in the highest precision.

Nothing here quantises, packs, routes or multiplies by the layer's weights.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

N_PRECISIONS = 4


@dataclass(frozen=True)
class LinearSpec:
    name: str
    N: int  # output features (rows of W)
    K: int  # input features (columns of W)


@dataclass(frozen=True)
class WorkloadConfig:
    index: int
    title: str
    seed: int
    linears: Tuple[LinearSpec, ...]
    token_counts: Tuple[int, ...]
    weight_df: float = 4.0
    mix: Optional[Tuple[float, float, float, float]] = None  # None -> uniform, zero bias
    outlier_channel_frac: float = 0.0
    outlier_token_frac: float = 0.0
    notes: str = ""


def _llama_block(hidden: int, kv: int, ffn: int) -> Tuple[LinearSpec, ...]:
    return (
        LinearSpec("q", hidden, hidden),
        LinearSpec("k", kv, hidden),
        LinearSpec("v", kv, hidden),
        LinearSpec("o", hidden, hidden),
        LinearSpec("gate", ffn, hidden),
        LinearSpec("up", ffn, hidden),
        LinearSpec("down", hidden, ffn),
    )


def _mlp(hidden: int, ffn: int) -> Tuple[LinearSpec, ...]:
    return (
        LinearSpec("gate", ffn, hidden),
        LinearSpec("up", ffn, hidden),
        LinearSpec("down", hidden, ffn),
    )


CONFIGS: Dict[int, WorkloadConfig] = {
    0: WorkloadConfig(
        index=0,
        title="single 2048x2048 routed linear, 32 tokens",
        seed=0,
        linears=(LinearSpec("lin", 2048, 2048),),
        token_counts=(32,),
        mix=(0.40, 0.30, 0.20, 0.10),
        outlier_channel_frac=0.01,
    ),
    1: WorkloadConfig(
        index=1,
        title="Llama-2-7B-shaped decode block, batch 1/4/16",
        seed=1,
        linears=_llama_block(4096, 4096, 11008),
        token_counts=(1, 4, 16),
        mix=None,
        outlier_channel_frac=0.01,
    ),
    2: WorkloadConfig(
        index=2,
        title="Llama-2-7B-shaped prefill MLP, 2048 tokens",
        seed=2,
        linears=_mlp(4096, 11008),
        token_counts=(2048,),
        mix=(0.50, 0.30, 0.15, 0.05),
        outlier_token_frac=0.02,
    ),
    3: WorkloadConfig(
        index=3,
        title="Llama-3-8B-shaped decoder block (GQA), decode batch 64",
        seed=3,
        linears=_llama_block(4096, 1024, 14336),
        token_counts=(64,),
        mix=None,
    ),
    4: WorkloadConfig(
        index=4,
        title="Llama-70B-shaped MLP, 4096 prefill tokens + 256 decode tokens",
        seed=4,
        linears=_mlp(8192, 28672),
        token_counts=(4096, 256),
        weight_df=3.0,
        mix=(0.70, 0.20, 0.08, 0.02),
    ),
}


# --------------------------------------------------------------------------- bf16
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def _bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ------------------------------------------------------------------------ weights
def make_weight(N: int, K: int, seed: Sequence[int], df: float = 4.0,
                rows: Optional[np.ndarray] = None) -> np.ndarray:
    """fp32 ``N x K`` heavy-tailed weight.  Row ``n`` depends only on (seed, n), so a
    subset of rows (``rows``) can be rebuilt without generating the whole matrix."""
    seed = list(seed)
    row_scale = np.exp(0.3 * np.random.default_rng(seed + [10]).standard_normal(N))
    if rows is None:
        rows = np.arange(N)
    out = np.empty((len(rows), K), dtype=np.float32)
    # one generator per block of 64 rows: cheap to rebuild any row subset
    blk = 64
    rows = np.asarray(rows)
    for b in np.unique(rows // blk):
        r0 = int(b) * blk
        r1 = min(N, r0 + blk)
        t = np.random.default_rng(seed + [11, int(b)]).standard_t(df, size=(r1 - r0, K))
        t *= 0.02 * row_scale[r0:r1, None]
        sel = np.nonzero(rows // blk == b)[0]
        out[sel] = t[rows[sel] - r0].astype(np.float32)
    return out


# ------------------------------------------------------------------------- tokens
def _outlier_channels(K: int, frac: float, seed: Sequence[int]) -> np.ndarray:
    n = int(np.floor(frac * K))
    if n == 0:
        return np.zeros(0, dtype=np.int64)
    return np.sort(np.random.default_rng(list(seed) + [20]).choice(K, size=n, replace=False))


def _direction(K: int, seed: Sequence[int]) -> np.ndarray:
    v = np.random.default_rng(list(seed) + [21]).standard_normal(K)
    return v / np.linalg.norm(v)


def _draw_tokens(rng: np.random.Generator, T: int, K: int, channels: np.ndarray,
                 outlier_rows: np.ndarray, v: Optional[np.ndarray]) -> np.ndarray:
    x = rng.standard_normal((T, K)).astype(np.float32)
    if channels.size:
        x[:, channels] *= np.float32(20.0)
    if outlier_rows.size:
        x[outlier_rows] += (np.sqrt(99.0 * K) * v).astype(np.float32)[None, :]
    return x


def make_tokens(T: int, K: int, seed: Sequence[int], outlier_channel_frac: float = 0.0,
                outlier_token_frac: float = 0.0) -> Tuple[np.ndarray, np.ndarray]:
    """Returns (bf16 bit patterns ``T x K`` uint16, indices of the outlier tokens)."""
    seed = list(seed)
    channels = _outlier_channels(K, outlier_channel_frac, seed)
    n_out = int(round(outlier_token_frac * T))
    rng = np.random.default_rng(seed + [22, T])
    outlier_rows = (np.sort(rng.choice(T, size=n_out, replace=False))
                    if n_out else np.zeros(0, dtype=np.int64))
    v = _direction(K, seed) if n_out or outlier_token_frac > 0 else None
    x = _draw_tokens(rng, T, K, channels, outlier_rows, v)
    return f32_to_bf16_bits(x), outlier_rows


# ------------------------------------------------------------------------- router
def make_router(K: int, seed: Sequence[int], mix: Optional[Sequence[float]] = None,
                outlier_channel_frac: float = 0.0, outlier_token_frac: float = 0.0
                ) -> Tuple[np.ndarray, np.ndarray]:
    """Router parameters ``Wr`` (4 x K fp32) and ``br`` (4 fp32) for a target mix."""
    seed = list(seed)
    rng = np.random.default_rng(seed + [30])
    wr = rng.standard_normal((N_PRECISIONS, K)) / np.sqrt(K)
    if outlier_token_frac > 0:
        v = _direction(K, seed)
        wr -= np.outer(wr @ v, v)
        wr[N_PRECISIONS - 1] += 2.0 * v / np.sqrt(K)
    wr = wr.astype(np.float32)
    br = np.zeros(N_PRECISIONS, dtype=np.float64)
    if mix is not None:
        target = np.asarray(mix, dtype=np.float64)
        target = target / target.sum()
        n_cal = int(min(16384, max(4096, (1 << 26) // K)))
        channels = _outlier_channels(K, outlier_channel_frac, seed)
        cal_rng = np.random.default_rng(seed + [31])
        scores = np.empty((n_cal, N_PRECISIONS), dtype=np.float64)
        step = 4096
        wr64 = wr.astype(np.float64)
        for t0 in range(0, n_cal, step):
            t1 = min(n_cal, t0 + step)
            xc = _draw_tokens(cal_rng, t1 - t0, K, channels, np.zeros(0, dtype=np.int64), None)
            xc = _bf16_bits_to_f32(f32_to_bf16_bits(xc)).astype(np.float64)
            scores[t0:t1] = xc @ wr64.T
        br = np.log(target)
        for _ in range(400):
            got = np.bincount(np.argmax(scores + br, axis=1), minlength=N_PRECISIONS) / n_cal
            if np.max(np.abs(got - target)) < 3e-3:
                break
            br = br + 0.5 * np.log(target / np.maximum(got, 1e-6))
        br = br - br.mean()
    return wr, br.astype(np.float32)


def make_mlp_router(K: int, hidden: int, seed: Sequence[int], n_slices: int = N_PRECISIONS
                    ) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """Parameters of a 2-layer router: ``W1`` (hidden x K), ``b1`` (hidden), ``W2`` (n_slices x hidden),
    ``b2`` (n_slices), all fp32.  Rows of W1 ~ N(0, 1/K) so hidden pre-activations are O(1) on N(0,1) tokens;
    W2 ~ N(0, 4/hidden); b2 falls with the slice index so that later slices are active less often."""
    rng = np.random.default_rng(list(seed) + [40])
    w1 = (rng.standard_normal((hidden, K)) / np.sqrt(K)).astype(np.float32)
    b1 = (0.1 * rng.standard_normal(hidden)).astype(np.float32)
    w2 = (2.0 * rng.standard_normal((n_slices, hidden)) / np.sqrt(hidden)).astype(np.float32)
    b2 = (0.5 - 0.5 * np.arange(n_slices)).astype(np.float32)
    return w1, b1, w2, b2


# --------------------------------------------------------------------------- case
def make_case(cfg: WorkloadConfig, linear_index: int, T: int,
              weight_rows: Optional[np.ndarray] = None, with_weight: bool = True) -> dict:
    """All inputs of one routed linear call: ``W`` (fp32 N x K, or the requested rows),
    ``X`` (bf16 bits T x K), ``Wr``/``br`` (router), plus bookkeeping."""
    spec = cfg.linears[linear_index]
    seed = [cfg.seed, linear_index]
    case = {"spec": spec, "T": T, "seed": seed}
    if with_weight:
        case["W"] = make_weight(spec.N, spec.K, seed, cfg.weight_df, rows=weight_rows)
    x, outlier_rows = make_tokens(T, spec.K, seed, cfg.outlier_channel_frac, cfg.outlier_token_frac)
    case["X"] = x
    case["outlier_tokens"] = outlier_rows
    wr, br = make_router(spec.K, seed, cfg.mix, cfg.outlier_channel_frac, cfg.outlier_token_frac)
    case["Wr"] = wr
    case["br"] = br
    return case
