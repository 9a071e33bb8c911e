"""CPU oracle for the augmented causal linear attention path (fp64, plain C).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by the ``cpu_baseline`` leg of ``bench.py``.  The product package never
imports it, and it never imports the product package.

The arithmetic lives in ``linattn_oracle.c`` (see its header for the passages
of the paper each function follows).  This module only builds that file with
gcc and marshals numpy float64 arrays through ctypes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "linattn_oracle.c")
_LIB = os.path.join(_HERE, "liblinattn_oracle.so")
_lib = None

_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int)


def build(force: bool = False, src: str = _SRC, out: str = _LIB) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over heads, no fast-math)."""
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-ffp-contract=off", "-Wall", "-Wextra", src, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)
    return out


def _load(path: str | None = None):
    global _lib
    if path is not None:
        return _declare(ctypes.CDLL(path))
    if _lib is None:
        _lib = _declare(ctypes.CDLL(build()))
    return _lib


def _declare(lib):
    i, f = ctypes.c_int, ctypes.c_double
    lib.oracle_set_feature_map.restype = None
    lib.oracle_set_feature_map.argtypes = [i]
    lib.oracle_phi.restype = f
    lib.oracle_phi.argtypes = [f]
    lib.oracle_causal_conv.restype = None
    lib.oracle_causal_conv.argtypes = [i, i, i, i, i, _dp, _dp, _dp, _dp]
    for name in ("oracle_prefill_quadratic", "oracle_prefill_recurrent"):
        fn = getattr(lib, name)
        fn.restype = i
        fn.argtypes = [i, i, i, i, i, f] + [_dp] * 11
    lib.oracle_prefill_grouped.restype = i
    lib.oracle_prefill_grouped.argtypes = [i, i, i, i, i, i, f, f] + [_dp] * 11
    lib.oracle_prefill_grouped_backward.restype = i
    lib.oracle_prefill_grouped_backward.argtypes = [i, i, i, i, i, i, f, f] + [_dp] * 17
    lib.oracle_verify_grouped.restype = i
    lib.oracle_verify_grouped.argtypes = [i, i, i, i, i, i, f, f] + [_dp] * 9 + [_ip, _ip, _dp]
    lib.oracle_verify.restype = i
    lib.oracle_verify.argtypes = [i, i, i, i, i, f] + [_dp] * 7 + [_ip, _dp]
    lib.oracle_verify_tree.restype = i
    lib.oracle_verify_tree.argtypes = [i, i, i, i, i, f] + [_dp] * 3 + [_ip] + [_dp] * 4 + [_ip, _dp]
    lib.oracle_decode.restype = i
    lib.oracle_decode.argtypes = [i, i, i, i, f] + [_dp] * 8
    lib.oracle_num_threads.restype = i
    lib.oracle_set_num_threads.argtypes = [i]
    return lib


def _c(a, shape=None):
    """float64, C-contiguous copy-if-needed; None passes through."""
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(_dp)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


FEATURE_MAPS = {"elu1": 0, "relu": 1}


class feature_map:
    """``with oracle.feature_map("relu"): ...`` -- every oracle call inside uses phi(x) = max(x, 0)
    instead of elu(x) + 1 (a setting of the loaded library, restored on exit)."""

    def __init__(self, kind: str, lib=None):
        self.code = FEATURE_MAPS[kind]
        self.lib = lib or _load()

    def __enter__(self):
        self.lib.oracle_set_feature_map(self.code)
        return self

    def __exit__(self, *exc):
        self.lib.oracle_set_feature_map(0)
        return False


def phi(x, lib=None):
    lib = lib or _load()
    return np.vectorize(lambda t: lib.oracle_phi(float(t)), otypes=[np.float64])(np.asarray(x, dtype=np.float64))


def causal_conv(v, w, hist=None, lib=None):
    """U[b,h,t,c] = sum_j w[h,c,j] * vext[b,h,t-j,c]; v [B,H,L,d], w [H,d,Kc]."""
    lib = lib or _load()
    v = _c(v)
    B, H, L, d = v.shape
    w = _c(w)
    Kc = w.shape[2]
    w = _c(w, (H, d, Kc))
    hist = _c(hist, (B, H, Kc - 1, d)) if hist is not None else None
    u = np.empty_like(v)
    lib.oracle_causal_conv(B, H, L, d, Kc, _p(v), _p(w), _p(hist), _p(u))
    return u


def _prefill(fname, q, k, v, w, S0, z0, hist0, eps, lib):
    lib = lib or _load()
    q = _c(q)
    B, H, L, d = q.shape
    k = _c(k, q.shape)
    v = _c(v, q.shape)
    w = _c(w)
    Kc = w.shape[2]
    w = _c(w, (H, d, Kc))
    S0 = _c(S0, (B, H, d, d)) if S0 is not None else None
    z0 = _c(z0, (B, H, d)) if z0 is not None else None
    hist0 = _c(hist0, (B, H, Kc - 1, d)) if hist0 is not None else None
    out = np.empty_like(q)
    S1 = np.empty((B, H, d, d))
    z1 = np.empty((B, H, d))
    h1 = np.empty((B, H, Kc - 1, d))
    rc = getattr(lib, fname)(B, H, L, d, Kc, float(eps), _p(q), _p(k), _p(v), _p(w),
                             _p(S0), _p(z0), _p(hist0), _p(out), _p(S1), _p(z1), _p(h1))
    if rc != 0:
        raise ValueError(f"{fname} rejected its arguments (code {rc})")
    return out, S1, z1, h1


def _value_blocks(d, v):
    """Value rows wider than key rows (Sec. 3, Eq. 1: Q, K of width d_k, V of width d_v).  Column c of the output
    -- of the attention part and of the depthwise conv alike -- is a function of Q, K and column c of V only, and
    so are column c of S and of the history; z does not involve V at all.  A V of width d_v = m d_k is therefore
    m problems of width d_k that share Q and K: the slices of the last axis of v, w, S, hist, one per problem."""
    dv = np.shape(v)[-1]
    if dv == d:
        return None
    if dv % d != 0:
        raise ValueError(f"value width {dv} is not a multiple of the key width {d}")
    return [slice(i, i + d) for i in range(0, dv, d)]


def _cut(a, sl, axis=-1):
    if a is None:
        return None
    idx = [slice(None)] * np.ndim(a)
    idx[axis] = sl
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64)[tuple(idx)])


def _prefill_any_width(fname, q, k, v, w, S0, z0, hist0, eps, lib):
    blocks = _value_blocks(np.shape(q)[-1], v)
    if blocks is None:
        return _prefill(fname, q, k, v, w, S0, z0, hist0, eps, lib)
    parts = [_prefill(fname, q, k, _cut(v, sl), _cut(w, sl, axis=1), _cut(S0, sl), z0, _cut(hist0, sl), eps, lib)
             for sl in blocks]
    return (np.concatenate([p[0] for p in parts], axis=-1), np.concatenate([p[1] for p in parts], axis=-1), parts[0][2],
            np.concatenate([p[3] for p in parts], axis=-1))


def prefill_quadratic(q, k, v, w, S0=None, z0=None, hist0=None, eps=0.0, lib=None):
    """Brute-force masked quadratic form.  Returns (out, S, z, hist).  v may be wider than q, k (see _value_blocks)."""
    return _prefill_any_width("oracle_prefill_quadratic", q, k, v, w, S0, z0, hist0, eps, lib)


def prefill_recurrent(q, k, v, w, S0=None, z0=None, hist0=None, eps=0.0, lib=None):
    """Token-by-token recurrence.  Returns (out, S, z, hist).  v may be wider than q, k (see _value_blocks)."""
    return _prefill_any_width("oracle_prefill_recurrent", q, k, v, w, S0, z0, hist0, eps, lib)


def prefill_grouped(q, k, v, w, group, alpha=1.0, S0=None, z0=None, hist0=None, eps=0.0, lib=None):
    """The three-branch form of Sec. 4.1: grouped linear attention over the groups before a token's own
    (weight alpha) + causal softmax attention inside its group + masked conv.  group: tokens per group.
    Returns (out, S, z, hist); the state is the same running sum as in the other forms."""
    lib = lib or _load()
    q = _c(q)
    B, H, L, d = q.shape
    k = _c(k, q.shape)
    v = _c(v, q.shape)
    w = _c(w)
    Kc = w.shape[2]
    w = _c(w, (H, d, Kc))
    S0 = _c(S0, (B, H, d, d)) if S0 is not None else None
    z0 = _c(z0, (B, H, d)) if z0 is not None else None
    hist0 = _c(hist0, (B, H, Kc - 1, d)) if hist0 is not None else None
    out = np.empty_like(q)
    S1 = np.empty((B, H, d, d))
    z1 = np.empty((B, H, d))
    h1 = np.empty((B, H, Kc - 1, d))
    rc = lib.oracle_prefill_grouped(B, H, L, d, Kc, int(group), float(eps), float(alpha), _p(q), _p(k), _p(v), _p(w),
                                    _p(S0), _p(z0), _p(hist0), _p(out), _p(S1), _p(z1), _p(h1))
    if rc != 0:
        raise ValueError(f"oracle_prefill_grouped rejected its arguments (code {rc})")
    return out, S1, z1, h1


def prefill_grouped_backward(q, k, v, w, dout, group, alpha=1.0, S0=None, z0=None, hist0=None, dS1=None, dz1=None,
                             eps=0.0, lib=None):
    """Gradient of the three-branch form (the training direction of Sec. 5.3): for the loss
    sum(dout * out) + sum(dS1 * S1) + sum(dz1 * z1) of ``prefill_grouped`` with the same arguments, the derivatives with
    respect to q, k, v, the conv weights (summed over the batch), the incoming state and the incoming history.
    Returns a dict with dq, dk, dv, dw, dS0, dz0, dhist0."""
    lib = lib or _load()
    q = _c(q)
    B, H, L, d = q.shape
    k = _c(k, q.shape)
    v = _c(v, q.shape)
    dout = _c(dout, q.shape)
    w = _c(w)
    Kc = w.shape[2]
    w = _c(w, (H, d, Kc))
    S0 = _c(S0, (B, H, d, d)) if S0 is not None else None
    z0 = _c(z0, (B, H, d)) if z0 is not None else None
    hist0 = _c(hist0, (B, H, Kc - 1, d)) if hist0 is not None else None
    dS1 = _c(dS1, (B, H, d, d)) if dS1 is not None else None
    dz1 = _c(dz1, (B, H, d)) if dz1 is not None else None
    r = {"dq": np.empty_like(q), "dk": np.empty_like(q), "dv": np.empty_like(q), "dw": np.empty((H, d, Kc)),
         "dS0": np.empty((B, H, d, d)), "dz0": np.empty((B, H, d)), "dhist0": np.empty((B, H, Kc - 1, d))}
    rc = lib.oracle_prefill_grouped_backward(B, H, L, d, Kc, int(group), float(eps), float(alpha), _p(q), _p(k), _p(v),
                                             _p(w), _p(S0), _p(z0), _p(hist0), _p(dout), _p(dS1), _p(dz1), _p(r["dq"]),
                                             _p(r["dk"]), _p(r["dv"]), _p(r["dw"]), _p(r["dS0"]), _p(r["dz0"]),
                                             _p(r["dhist0"]))
    if rc != 0:
        raise ValueError(f"oracle_prefill_grouped_backward rejected its arguments (code {rc})")
    return r


def verify(q, k, v, w, S, z, hist, n_commit=None, eps=0.0, lib=None):
    """kk sequential steps from one state; returns (out, S', z', hist').

    q, k, v: [B,H,kk,d].  n_commit: None (keep all) or int array [B] in 0..kk.
    The incoming state arrays are not modified.
    """
    lib = lib or _load()
    blocks = _value_blocks(np.shape(q)[-1], v)
    if blocks is not None:                     # v wider than q, k: one problem per block of value channels
        parts = [verify(q, k, _cut(v, sl), _cut(w, sl, axis=1), _cut(S, sl), z, _cut(hist, sl), n_commit, eps, lib)
                 for sl in blocks]
        return (np.concatenate([p[0] for p in parts], axis=-1), np.concatenate([p[1] for p in parts], axis=-1),
                parts[0][2], np.concatenate([p[3] for p in parts], axis=-1))
    q = _c(q)
    B, H, kk, d = q.shape
    k = _c(k, q.shape)
    v = _c(v, q.shape)
    w = _c(w)
    Kc = w.shape[2]
    w = _c(w, (H, d, Kc))
    S = np.array(_c(S, (B, H, d, d)), copy=True)
    z = np.array(_c(z, (B, H, d)), copy=True)
    hist = np.array(_c(hist, (B, H, Kc - 1, d)), copy=True)
    nc = None
    if n_commit is not None:
        nc = np.ascontiguousarray(n_commit, dtype=np.int32)
        if nc.shape != (B,):
            raise ValueError("n_commit must have shape [B]")
    out = np.empty_like(q)
    rc = lib.oracle_verify(B, H, kk, d, Kc, float(eps), _p(q), _p(k), _p(v), _p(w),
                           _p(S), _p(z), _p(hist),
                           None if nc is None else nc.ctypes.data_as(_ip), _p(out))
    if rc != 0:
        raise ValueError(f"oracle_verify rejected its arguments (code {rc})")
    return out, S, z, hist


def verify_grouped(q, k, v, w, group, S, z, hist, kwin, vwin, fill, n_commit=None, alpha=1.0, eps=0.0, lib=None):
    """kk token steps of the three-branch form from one state.  S, z: sums over the completed groups;
    kwin, vwin [B,H,group,d]: raw key / value rows of the current group, rows 0..fill[b]-1 in use; fill int [B].
    Returns (out, S', z', hist', kwin', vwin', fill') after the first n_commit[b] steps (None: all); the
    incoming arrays are not modified."""
    lib = lib or _load()
    q = _c(q)
    B, H, kk, d = q.shape
    k = _c(k, q.shape)
    v = _c(v, q.shape)
    w = _c(w)
    Kc = w.shape[2]
    w = _c(w, (H, d, Kc))
    C = int(group)
    S = np.array(_c(S, (B, H, d, d)), copy=True)
    z = np.array(_c(z, (B, H, d)), copy=True)
    hist = np.array(_c(hist, (B, H, Kc - 1, d)), copy=True)
    kwin = np.array(_c(kwin, (B, H, C, d)), copy=True)
    vwin = np.array(_c(vwin, (B, H, C, d)), copy=True)
    fill = np.array(np.ascontiguousarray(fill, dtype=np.int32), copy=True)
    if fill.shape != (B,):
        raise ValueError("fill must have shape [B]")
    nc = None
    if n_commit is not None:
        nc = np.ascontiguousarray(n_commit, dtype=np.int32)
        if nc.shape != (B,):
            raise ValueError("n_commit must have shape [B]")
    out = np.empty_like(q)
    rc = lib.oracle_verify_grouped(B, H, kk, d, Kc, C, float(eps), float(alpha), _p(q), _p(k), _p(v), _p(w),
                                   _p(S), _p(z), _p(hist), _p(kwin), _p(vwin), fill.ctypes.data_as(_ip),
                                   None if nc is None else nc.ctypes.data_as(_ip), _p(out))
    if rc != 0:
        raise ValueError(f"oracle_verify_grouped rejected its arguments (code {rc})")
    return out, S, z, hist, kwin, vwin, fill


def verify_tree(q, k, v, parent, w, S, z, hist, accept=None, eps=0.0, lib=None):
    """Tree-structured verification (Sec. 4.2): n candidates, parent[i] < i (or -1 for a candidate that
    follows the verified sequence directly), every candidate scored from the verified state and its own
    root path only.  accept: None (nothing is committed) or int array [B], the candidate whose root path is
    committed (-1: none).  Returns (out, S', z', hist'); the incoming state arrays are not modified.
    """
    lib = lib or _load()
    q = _c(q)
    B, H, n, d = q.shape
    k = _c(k, q.shape)
    v = _c(v, q.shape)
    w = _c(w)
    Kc = w.shape[2]
    w = _c(w, (H, d, Kc))
    par = np.ascontiguousarray(parent, dtype=np.int32)
    if par.shape != (n,):
        raise ValueError("parent must have shape [n]")
    S = np.array(_c(S, (B, H, d, d)), copy=True)
    z = np.array(_c(z, (B, H, d)), copy=True)
    hist = np.array(_c(hist, (B, H, Kc - 1, d)), copy=True)
    acc = None
    if accept is not None:
        acc = np.ascontiguousarray(accept, dtype=np.int32)
        if acc.shape != (B,):
            raise ValueError("accept must have shape [B]")
    out = np.empty_like(q)
    rc = lib.oracle_verify_tree(B, H, n, d, Kc, float(eps), _p(q), _p(k), _p(v), par.ctypes.data_as(_ip), _p(w),
                                _p(S), _p(z), _p(hist), None if acc is None else acc.ctypes.data_as(_ip), _p(out))
    if rc != 0:
        raise ValueError(f"oracle_verify_tree rejected its arguments (code {rc})")
    return out, S, z, hist


def decode(q, k, v, w, S, z, hist, eps=0.0, lib=None):
    """One generated token per head: q, k, v [B,H,1,d]; the state always advances."""
    lib = lib or _load()
    blocks = _value_blocks(np.shape(q)[-1], v)
    if blocks is not None:                     # v wider than q, k: one problem per block of value channels
        parts = [decode(q, k, _cut(v, sl), _cut(w, sl, axis=1), _cut(S, sl), z, _cut(hist, sl), eps, lib) for sl in blocks]
        return (np.concatenate([p[0] for p in parts], axis=-1), np.concatenate([p[1] for p in parts], axis=-1),
                parts[0][2], np.concatenate([p[3] for p in parts], axis=-1))
    q = _c(q)
    B, H, one, d = q.shape
    if one != 1:
        raise ValueError("decode takes exactly one token per head")
    k = _c(k, q.shape)
    v = _c(v, q.shape)
    w = _c(w)
    Kc = w.shape[2]
    w = _c(w, (H, d, Kc))
    S = np.array(_c(S, (B, H, d, d)), copy=True)
    z = np.array(_c(z, (B, H, d)), copy=True)
    hist = np.array(_c(hist, (B, H, Kc - 1, d)), copy=True)
    out = np.empty_like(q)
    rc = lib.oracle_decode(B, H, d, Kc, float(eps), _p(q), _p(k), _p(v), _p(w),
                           _p(S), _p(z), _p(hist), _p(out))
    if rc != 0:
        raise ValueError(f"oracle_decode rejected its arguments (code {rc})")
    return out, S, z, hist
