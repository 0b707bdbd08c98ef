"""Shared helpers of the GPU parity tests (uploading inputs, the parity bar)."""
from __future__ import annotations

import numpy as np
import torch

import oracle as O

# The bar for floating-point outputs (fp32 accumulate vs the fp64 oracle):
REL_FRO_TOL = 1e-3          # ||Y - Y_ref||_F / ||Y_ref||_F
MAX_ABS_TOL = 5e-3          # max |Y - Y_ref| / rms(Y_ref)
NEAR_TIE_GAP = 1e-5         # tokens whose top-2 router logits are closer than this are reported apart


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def output_errors(Y: np.ndarray, Yref: np.ndarray):
    Y = np.asarray(Y, dtype=np.float64)
    diff = Y - Yref
    fro = float(np.linalg.norm(diff) / max(np.linalg.norm(Yref), 1e-300))
    rms = float(np.sqrt(np.mean(Yref ** 2))) if Yref.size else 1.0
    mx = float(np.max(np.abs(diff)) / max(rms, 1e-300)) if Yref.size else 0.0
    return fro, mx


def assert_output_close(Y, Yref, what=""):
    fro, mx = output_errors(Y, Yref)
    print(f"[parity] {what}: rel-Frobenius {fro:.3e}  max-abs/rms {mx:.3e}", flush=True)
    assert fro <= REL_FRO_TOL, (what, fro)
    assert mx <= MAX_ABS_TOL, (what, mx)
    return fro, mx


def compare_routing(prec_gpu: np.ndarray, prec_ref: np.ndarray, gap: np.ndarray, what=""):
    """Bit-exact except on the near-tie list, which is reported separately."""
    near = gap < NEAR_TIE_GAP
    bad = (prec_gpu != prec_ref) & ~near
    print(f"[parity] {what}: {len(prec_ref)} tokens, {int(near.sum())} near-tie, "
          f"{int((prec_gpu != prec_ref).sum())} differing (all must be near-ties)", flush=True)
    assert not bad.any(), (what, np.nonzero(bad)[0][:10])


def check_bucket(prec: np.ndarray, perm: np.ndarray, offsets: np.ndarray):
    want_perm, want_off = O.bucket(prec)
    assert np.array_equal(offsets, want_off), (offsets, want_off)
    assert np.array_equal(perm, want_perm)
