"""Helpers shared by the GPU parity tests: the error metric and host<->device plumbing."""
from __future__ import annotations

import numpy as np
import torch

# Bars from the benchmark spec: max relative error, fp32 inputs / bf16 inputs with fp32 accumulation.
TOL = {"f32": 1e-4, "bf16": 2e-2}
# S and z after a verify / decode / tree-verify / generation step that was handed its state in fp32: the state
# is fp32 on both sides of the call, and every kernel adds phi(k) v^T with at least sixteen significant bits of
# phi(k) (fp32 products, or phi(k) as the sum of two bf16 terms on the matrix cores): each product is off by at
# most 2^-17 of itself, a few 1e-6 of the head's rms after up to 64 tokens.
STATE_TOL = 2e-5


def rel_err(got, want) -> float:
    """max_e |got - want| / max(|want_e|, rms(want over its (b, h) slice)).

    A plain elementwise relative error is unbounded where an output crosses zero, so
    every element's denominator is floored by the root-mean-square of its own head.
    """
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if want.size == 0:
        return 0.0
    assert np.all(np.isfinite(got)), "non-finite values in the GPU result"
    B, H = want.shape[:2]
    w2 = want.reshape(B, H, -1)
    rms = np.sqrt(np.mean(w2 * w2, axis=-1)).reshape((B, H) + (1,) * (want.ndim - 2))
    den = np.maximum(np.abs(want), np.maximum(rms, 1e-30))
    return float(np.max(np.abs(got - want) / den))


def err_stats(got, want):
    """(rel_err as above, plain max abs error, 99.9th percentile of the un-floored relative error)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return 0.0, 0.0, 0.0
    diff = np.abs(got - want)
    unfloored = diff / np.maximum(np.abs(want), 1e-30)
    return rel_err(got, want), float(diff.max()), float(np.percentile(unfloored, 99.9))


def check_unfloored(got, want, tol, what, percentile=99.0):
    """The plain elementwise relative error |got - want| / |want| has no finite maximum where an output crosses
    zero, so it is held to the bar at a percentile instead: at most 1 % of the elements may exceed it."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return 0.0
    p = float(np.percentile(np.abs(got - want) / np.maximum(np.abs(want), 1e-30), percentile))
    assert p <= tol, f"{what}: {percentile}th percentile of the un-floored relative error {p:.3e} > {tol:.1e}"
    return p


def check(got, want, tol, what):
    e = rel_err(got, want)
    assert e <= tol, f"{what}: rel err {e:.3e} > {tol:.1e} (max abs {np.max(np.abs(np.asarray(got, dtype=np.float64) - want)):.3e})"
    return e


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)
