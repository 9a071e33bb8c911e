"""Pins for the CPU oracle: facts fixed by the paper or by mathematics.

Each ``pin_*`` function takes an oracle library handle (``lib``; None = the
real one) and raises AssertionError if the oracle violates the fact.  They are
run against the real oracle in ``test_oracle_pins.py`` and against deliberately
broken copies of it in ``test_oracle_mutants.py`` (every planted mistake must
trip at least one pin).

None of them re-derives the oracle from its own formula: they use closed
forms, special cases that reduce to library routines (cumsum, outer, grouped
conv1d), exact rational arithmetic on a tiny case, invariances and the
conv-window example the paper gives in Sec. 4.2.
"""
from __future__ import annotations

import math
import os
from fractions import Fraction

import numpy as np
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


def _rand(seed, B=2, H=3, L=17, d=5, Kc=3, with_state=False):
    r = _rng(seed)
    q, k, v = (r.standard_normal((B, H, L, d)) for _ in range(3))
    w = r.standard_normal((H, d, Kc))
    if not with_state:
        return q, k, v, w
    S0 = r.standard_normal((B, H, d, d))
    z0 = np.abs(r.standard_normal((B, H, d))) + 0.5
    h0 = r.standard_normal((B, H, Kc - 1, d))
    return q, k, v, w, S0, z0, h0


def _close(a, b, tol=1e-12, what=""):
    a, b = np.asarray(a), np.asarray(b)
    assert a.shape == b.shape, f"{what}: shape {a.shape} vs {b.shape}"
    err = np.max(np.abs(a - b)) if a.size else 0.0
    scale = max(1.0, float(np.max(np.abs(b))) if b.size else 1.0)
    assert err <= tol * scale, f"{what}: max abs err {err:.3e} (scale {scale:.3e})"


FORMS = ("prefill_quadratic", "prefill_recurrent")


# --- the feature map ---------------------------------------------------------
def pin_phi_values(lib=None):
    """elu(x)+1: 1 at 0, x+1 above, exp(x) below (library exp), positive, increasing."""
    xs = np.array([-30.0, -3.5, -1.0, -1e-9, 0.0, 1e-9, 0.25, 1.0, 7.5])
    got = oracle.phi(xs, lib=lib)
    want = np.array([math.exp(x) if x <= 0 else x + 1.0 for x in xs])
    _close(got, want, 1e-15, "phi")
    assert got[4] == 1.0
    assert np.all(got > 0) and np.all(np.diff(got) > 0)


# --- inclusive causal sum and the normaliser -----------------------------------
def pin_first_token_is_its_own_value(lib=None):
    """With one visible token the attention weight is 1: Y_1 = v_1 (Sec. 4.1, sum from i=1 to t)."""
    q, k, v, w = _rand(11)
    w0 = np.zeros_like(w)
    for f in FORMS:
        out = getattr(oracle, f)(q, k, v, w0, lib=lib)[0]
        _close(out[:, :, 0], v[:, :, 0], 1e-13, f + " first token")


def pin_zero_keys_give_running_mean(lib=None):
    """K == 0 -> phi(K) == 1 -> every visible token weighs the same: cumsum(V)/count."""
    q, k, v, w = _rand(12, L=23)
    k = np.zeros_like(k)
    want = np.cumsum(v, axis=2) / np.arange(1, v.shape[2] + 1)[None, None, :, None]
    for f in FORMS:
        out = getattr(oracle, f)(q, k, v, np.zeros_like(w), lib=lib)[0]
        _close(out, want, 1e-12, f + " running mean")


def pin_zero_queries_weigh_by_key_mass(lib=None):
    """Q == 0 -> phi(q) is all ones -> weight of token i is sum_c phi(k_i)[c]."""
    q, k, v, w = _rand(13, L=19, d=4)
    q = np.zeros_like(q)
    r = np.where(k > 0, k + 1.0, np.exp(k)).sum(-1, keepdims=True)
    want = np.cumsum(r * v, axis=2) / np.cumsum(r, axis=2)
    for f in FORMS:
        out = getattr(oracle, f)(q, k, v, np.zeros_like(w), lib=lib)[0]
        _close(out, want, 1e-12, f + " key-mass weights")


def pin_head_dim_one_ignores_queries(lib=None):
    """d == 1: phi(q_t) cancels between numerator and normaliser."""
    q, k, v, w = _rand(14, L=15, d=1)
    r = np.where(k > 0, k + 1.0, np.exp(k))
    want = np.cumsum(r * v, axis=2) / np.cumsum(r, axis=2)
    for f in FORMS:
        out = getattr(oracle, f)(q, k, v, np.zeros_like(w), lib=lib)[0]
        _close(out, want, 1e-12, f + " d=1")
        out2 = getattr(oracle, f)(3.0 * q - 1.0, k, v, np.zeros_like(w), lib=lib)[0]
        _close(out2, want, 1e-12, f + " d=1, other q")


def pin_constant_values_pass_through(lib=None):
    """All value rows equal c -> Y_t = c for every t (weights are positive and sum to one)."""
    q, k, v, w = _rand(15)
    c = _rng(150).standard_normal(v.shape[-1])
    v = np.broadcast_to(c, v.shape).copy()
    for f in FORMS:
        out = getattr(oracle, f)(q, k, v, np.zeros_like(w), lib=lib)[0]
        _close(out, v, 1e-12, f + " constant V")


def pin_query_selects_feature(lib=None):
    """A query that is (nearly) one-hot in feature i reads column i of the state.

    q = -40 everywhere except +a at feature i: phi(q) = (a+1) e_i + O(e^-40), so
    Y_t = sum_s phi(k_s)[i] v_s / sum_s phi(k_s)[i] -- a weighted running mean whose
    weights depend on WHICH feature the query picked.
    """
    B, H, L, d = 1, 2, 12, 4
    r = _rng(16)
    k, v = r.standard_normal((B, H, L, d)), r.standard_normal((B, H, L, d))
    fk = np.where(k > 0, k + 1.0, np.exp(k))
    w = np.zeros((H, d, 3))
    for i in range(d):
        q = np.full((B, H, L, d), -40.0)
        q[..., i] = 1.5
        want = np.cumsum(fk[..., i:i + 1] * v, axis=2) / np.cumsum(fk[..., i:i + 1], axis=2)
        for f in FORMS:
            out = getattr(oracle, f)(q, k, v, w, lib=lib)[0]
            _close(out, want, 1e-10, f"{f} one-hot query {i}")


def pin_linearity_in_values(lib=None):
    q, k, v, w = _rand(17)
    v2 = _rng(170).standard_normal(v.shape)
    a, b = 0.75, -2.5
    for f in FORMS:
        fn = getattr(oracle, f)
        lhs = fn(q, k, a * v + b * v2, w, lib=lib)[0]
        rhs = a * fn(q, k, v, w, lib=lib)[0] + b * fn(q, k, v2, w, lib=lib)[0]
        _close(lhs, rhs, 1e-11, f + " linearity")


def pin_eps_enters_the_denominator(lib=None):
    """d=1, one token: out = phi(q)phi(k) v / (phi(q)phi(k) + eps)."""
    q = np.array([[[[0.5]]]])
    k = np.array([[[[1.0]]]])
    v = np.array([[[[3.0]]]])
    w = np.zeros((1, 1, 1))
    a = 1.5 * 2.0
    for f in FORMS:
        out = getattr(oracle, f)(q, k, v, w, eps=0.25, lib=lib)[0]
        _close(out, [[[[a * 3.0 / (a + 0.25)]]]], 1e-15, f + " eps")


# --- exact arithmetic on a tiny case ----------------------------------------------
def _phi_frac(x):
    """Inputs are chosen so that phi is rational: integers >= 0, or log(1/2), log(1/4)."""
    if x >= 0:
        return Fraction(x) + 1
    return {math.log(0.5): Fraction(1, 2), math.log(0.25): Fraction(1, 4)}[x]


def pin_exact_rational_brute_force(lib=None):
    """L=5, d=3, Kc=3, incoming state and history: exact fractions vs the oracle."""
    L, d, Kc = 5, 3, 3
    lh, lq = math.log(0.5), math.log(0.25)
    q = np.array([[0, 1, lh], [2, lq, 0], [lh, lh, 3], [1, 0, 0], [lq, 2, 1]], dtype=float)
    k = np.array([[1, lh, 0], [0, 0, 2], [lq, 1, lh], [3, lh, lq], [0, 1, 1]], dtype=float)
    v = np.array([[1, -2, 0.5], [0.25, 3, -1], [-4, 0, 2], [1.5, 1, 1], [0, -0.75, 8]])
    w = np.array([[0.5, -1, 2], [1, 0.25, -0.5], [-2, 4, 0.125]])          # [d, Kc]
    S0 = np.array([[1, 0, -1], [2, 0.5, 0], [0, 1, 3]], dtype=float)
    z0 = np.array([2, 1, 0.5])
    h0 = np.array([[1, 2, 3], [-1, 0.5, 4]], dtype=float)                   # oldest first

    F = Fraction
    fq = [[_phi_frac(x) for x in row] for row in q]
    fk = [[_phi_frac(x) for x in row] for row in k]
    vf = [[F(x) for x in row] for row in v]
    ext = [[F(x) for x in row] for row in h0] + vf                         # index s+2
    want = np.zeros((L, d))
    for t in range(L):
        den = sum(fq[t][i] * F(z0[i]) for i in range(d))
        num = [sum(fq[t][i] * F(S0[i][c]) for i in range(d)) for c in range(d)]
        for s in range(t + 1):
            a = sum(fq[t][i] * fk[s][i] for i in range(d))
            den += a
            num = [num[c] + a * vf[s][c] for c in range(d)]
        for c in range(d):
            u = sum(F(w[c][j]) * ext[t - j + 2][c] for j in range(Kc))
            want[t, c] = float(num[c] / den + u)
    S1 = [[F(S0[i][c]) + sum(fk[t][i] * vf[t][c] for t in range(L)) for c in range(d)] for i in range(d)]
    z1 = [F(z0[i]) + sum(fk[t][i] for t in range(L)) for i in range(d)]
    for f in FORMS:
        out, S, z, h = getattr(oracle, f)(q[None, None], k[None, None], v[None, None], w[None],
                                          S0[None, None], z0[None, None], h0[None, None], lib=lib)
        _close(out[0, 0], want, 1e-14, f + " exact out")
        _close(S[0, 0], np.array([[float(x) for x in row] for row in S1]), 1e-14, f + " exact S")
        _close(z[0, 0], np.array([float(x) for x in z1]), 1e-14, f + " exact z")
        _close(h[0, 0], v[-2:], 0.0, f + " hist")


# --- state layout ----------------------------------------------------------------
def pin_single_token_state_is_outer_product(lib=None):
    """After one token S = phi(k) v^T (row = key feature, column = value channel), z = phi(k)."""
    r = _rng(18)
    k, v, q = r.standard_normal((1, 1, 1, 4)), r.standard_normal((1, 1, 1, 4)), r.standard_normal((1, 1, 1, 4))
    fk = np.where(k > 0, k + 1.0, np.exp(k))[0, 0, 0]
    w = np.zeros((1, 4, 2))
    for f in FORMS:
        _, S, z, h = getattr(oracle, f)(q, k, v, w, lib=lib)
        _close(S[0, 0], np.outer(fk, v[0, 0, 0]), 1e-15, f + " S outer")
        _close(z[0, 0], fk, 1e-15, f + " z")
        _close(h[0, 0, 0], v[0, 0, 0], 0.0, f + " hist")


def pin_feature_and_channel_permutations(lib=None):
    """Permuting the q/k feature axis changes nothing; permuting value channels (and the
    conv weights with them) permutes the output channels."""
    q, k, v, w = _rand(19, d=6)
    pf = _rng(190).permutation(6)
    pc = _rng(191).permutation(6)
    for f in FORMS:
        fn = getattr(oracle, f)
        base = fn(q, k, v, w, lib=lib)[0]
        _close(fn(q[..., pf], k[..., pf], v, w, lib=lib)[0], base, 1e-12, f + " feature perm")
        _close(fn(q, k, v[..., pc], w[:, pc], lib=lib)[0], base[..., pc], 1e-12, f + " channel perm")


def pin_heads_are_independent(lib=None):
    """Swapping two heads (inputs and their conv weights) swaps their outputs."""
    q, k, v, w = _rand(20, B=2, H=3)
    perm = [2, 0, 1]
    for f in FORMS:
        fn = getattr(oracle, f)
        base = fn(q, k, v, w, lib=lib)[0]
        got = fn(q[:, perm], k[:, perm], v[:, perm], w[perm], lib=lib)[0]
        _close(got, base[:, perm], 0.0, f + " head perm")


# --- the causal depthwise convolution -----------------------------------------------
def pin_conv_matches_library_grouped_conv(lib=None):
    """Left-padded (by the history) grouped conv1d; cross-correlation needs the taps reversed."""
    B, H, L, d, Kc = 2, 3, 21, 4, 5
    r = _rng(21)
    v = r.standard_normal((B, H, L, d))
    w = r.standard_normal((H, d, Kc))
    for hist in (None, r.standard_normal((B, H, Kc - 1, d))):
        left = np.zeros((B, H, Kc - 1, d)) if hist is None else hist
        x = np.concatenate([left, v], axis=2)                                  # [B,H,L+Kc-1,d]
        x = torch.from_numpy(x).permute(0, 1, 3, 2).reshape(B, H * d, L + Kc - 1)
        wt = torch.from_numpy(w[:, :, ::-1].copy()).reshape(H * d, 1, Kc)
        want = torch.nn.functional.conv1d(x, wt, groups=H * d).reshape(B, H, d, L).permute(0, 1, 3, 2).numpy()
        _close(oracle.causal_conv(v, w, hist, lib=lib), want, 1e-13, "conv vs conv1d")
        q, k = r.standard_normal(v.shape), r.standard_normal(v.shape)
        for f in FORMS:
            fn = getattr(oracle, f)
            with_conv = fn(q, k, v, w, hist0=hist, lib=lib)[0]
            without = fn(q, k, v, np.zeros_like(w), hist0=hist, lib=lib)[0]
            _close(with_conv - without, want, 1e-12, f + " conv added to attention output")


def _window_table(path):
    table = {}
    with open(path) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if not line:
                continue
            key, val = line.split(":")
            table[int(key)] = sorted(int(x) for x in val.split())
    return table


def pin_conv_window_example_from_the_paper(lib=None):
    """Sec. 4.2: a kernel-3 conv at step t1 must cover {t0, t1}.  An impulse at token s with
    tap weights 1, 10, 100 tells which tap of which output sees s."""
    want = _window_table(os.path.join(GOLDEN, "conv_window_k3.txt"))
    L, Kc = 5, 3
    w = np.array([[[1.0, 10.0, 100.0]]])
    seen = {t: [] for t in range(L)}
    for s in range(L):
        v = np.zeros((1, 1, L, 1))
        v[0, 0, s, 0] = 1.0
        u = oracle.causal_conv(v, w, None, lib=lib)[0, 0, :, 0]
        for t in range(L):
            if u[t] != 0.0:
                seen[t].append(s)
                assert u[t] == 10.0 ** (t - s), f"tap order: token {s} seen by {t} with weight {u[t]}"
    assert {t: sorted(x) for t, x in seen.items()} == want
    # the same windows in a draft block that follows a verified history (t0 = history)
    S = np.zeros((1, 1, 1, 1)); z = np.ones((1, 1, 1)); hist = np.array([[[[5.0], [7.0]]]])
    zero = np.zeros((1, 1, 2, 1))
    drafts = np.array([[[[2.0], [3.0]]]])
    out = oracle.verify(zero, np.full_like(zero, -745.0), drafts, w, S, z, hist, lib=lib)[0][0, 0, :, 0]
    # keys ~ -inf -> phi(k) = 0 -> the attention part is 0/1; only the conv remains
    _close(out, [2.0 + 10 * 7.0 + 100 * 5.0, 3.0 + 10 * 2.0 + 100 * 7.0], 1e-12, "draft windows")


# --- no information leakage ---------------------------------------------------------------
def pin_no_leak_from_later_tokens(lib=None):
    """Changing any of q, k, v after position t leaves outputs up to t bit-identical (Sec. 4.1)."""
    q, k, v, w, S0, z0, h0 = _rand(22, L=14, with_state=True)
    r = _rng(220)
    for f in FORMS:
        fn = getattr(oracle, f)
        base = fn(q, k, v, w, S0, z0, h0, lib=lib)[0]
        for t in (0, 5, 12):
            q2, k2, v2 = q.copy(), k.copy(), v.copy()
            for a in (q2, k2, v2):
                a[:, :, t + 1:] += 10.0 * r.standard_normal(a[:, :, t + 1:].shape)
            got = fn(q2, k2, v2, w, S0, z0, h0, lib=lib)[0]
            assert np.array_equal(got[:, :, :t + 1], base[:, :, :t + 1]), f"{f}: leak into <= {t}"
            assert not np.array_equal(got[:, :, t + 1:], base[:, :, t + 1:])


def pin_every_earlier_token_matters(lib=None):
    """The converse: output t does change when any token s <= t changes (nothing is dropped)."""
    q, k, v, w = _rand(23, B=1, H=1, L=9)
    w = np.zeros_like(w)
    for f in FORMS:
        fn = getattr(oracle, f)
        base = fn(q, k, v, w, lib=lib)[0]
        for s in range(9):
            v2 = v.copy()
            v2[:, :, s] += 1.0
            got = fn(q, k, v2, w, lib=lib)[0]
            changed = np.any(got != base, axis=-1)[0, 0]
            assert list(changed) == [t >= s for t in range(9)], f"{f}: token {s} -> {changed}"


# --- re-association, chunking, resuming -------------------------------------------------------
def pin_recurrent_equals_quadratic(lib=None):
    """Sec. 3: phi(Q)(phi(K)^T V) is a re-association of (phi(Q)phi(K)^T)V."""
    for seed, kw in ((30, {}), (31, dict(B=1, H=2, L=32, d=8, Kc=1)), (32, dict(L=9, d=2, Kc=5)),
                     (33, dict(B=1, H=1, L=1, d=3))):
        args = _rand(seed, with_state=True, **kw)
        a = oracle.prefill_quadratic(*args, eps=1e-3, lib=lib)
        b = oracle.prefill_recurrent(*args, eps=1e-3, lib=lib)
        for x, y, n in zip(a, b, ("out", "S", "z", "hist")):
            _close(x, y, 1e-12, f"quadratic vs recurrent {n} (seed {seed})")
        a = oracle.prefill_quadratic(*args[:4], lib=lib)
        b = oracle.prefill_recurrent(*args[:4], lib=lib)
        for x, y, n in zip(a, b, ("out", "S", "z", "hist")):
            _close(x, y, 1e-12, f"quadratic vs recurrent from zero state {n} (seed {seed})")


def pin_split_invariance(lib=None):
    """prefill(L) == prefill(L1) then prefill(L - L1) from the handed-over state (Sec. 5.3:
    a shared prefix is computed once)."""
    q, k, v, w, S0, z0, h0 = _rand(34, L=20, with_state=True)
    for f in FORMS:
        fn = getattr(oracle, f)
        full = fn(q, k, v, w, S0, z0, h0, lib=lib)
        for L1 in (1, 2, 7, 19):
            a = fn(q[:, :, :L1], k[:, :, :L1], v[:, :, :L1], w, S0, z0, h0, lib=lib)
            b = fn(q[:, :, L1:], k[:, :, L1:], v[:, :, L1:], w, a[1], a[2], a[3], lib=lib)
            _close(np.concatenate([a[0], b[0]], axis=2), full[0], 1e-12, f"{f} split {L1} out")
            for x, y, n in zip(b[1:], full[1:], ("S", "z", "hist")):
                _close(x, y, 1e-12, f"{f} split {L1} {n}")


def pin_empty_sequence_is_identity(lib=None):
    q, k, v, w, S0, z0, h0 = _rand(35, L=0, with_state=True)
    for f in FORMS:
        out, S, z, h = getattr(oracle, f)(q, k, v, w, S0, z0, h0, lib=lib)
        assert out.shape[2] == 0
        assert np.array_equal(S, S0) and np.array_equal(z, z0) and np.array_equal(h, h0)


# --- verification of draft tokens -----------------------------------------------------------------
def pin_verify_equals_sequential_decode(lib=None):
    """Sec. 4.2: scoring k drafts at once must give what k single steps give."""
    B, H, d, Kc, kk = 2, 2, 4, 3, 5
    q, k, v, w, S0, z0, h0 = _rand(40, B=B, H=H, L=kk, d=d, Kc=Kc, with_state=True)
    out, S, z, h = oracle.verify(q, k, v, w, S0, z0, h0, lib=lib)
    Ss, zs, hs = S0, z0, h0
    for j in range(kk):
        o, Ss, zs, hs = oracle.decode(q[:, :, j:j + 1], k[:, :, j:j + 1], v[:, :, j:j + 1], w, Ss, zs, hs, lib=lib)
        assert np.array_equal(o[:, :, 0], out[:, :, j]), f"draft {j}"
    assert np.array_equal(S, Ss) and np.array_equal(z, zs) and np.array_equal(h, hs)
    # and both equal the last rows of one long prefill over prefix ++ drafts
    P = 6
    pq, pk, pv, _ = _rand(41, B=B, H=H, L=P, d=d, Kc=Kc)
    _, S1, z1, h1 = oracle.prefill_recurrent(pq, pk, pv, w, lib=lib)
    vo = oracle.verify(q, k, v, w, S1, z1, h1, lib=lib)
    cat = [np.concatenate([a, b], axis=2) for a, b in ((pq, q), (pk, k), (pv, v))]
    full = oracle.prefill_quadratic(*cat, w, lib=lib)
    _close(vo[0], full[0][:, :, P:], 1e-12, "prefill -> verify vs long prefill")
    for x, y, n in zip(vo[1:], full[1:], ("S", "z", "hist")):
        _close(x, y, 1e-12, "prefill -> verify " + n)


def pin_verify_commit_counts(lib=None):
    """Rejected drafts leave no trace: n_commit = n gives the state of n single steps,
    n_commit = 0 hands the state back bit-unchanged; outputs do not depend on n_commit."""
    B, H, d, Kc, kk = 3, 2, 4, 4, 4
    q, k, v, w, S0, z0, h0 = _rand(42, B=B, H=H, L=kk, d=d, Kc=Kc, with_state=True)
    all_out = oracle.verify(q, k, v, w, S0, z0, h0, lib=lib)[0]
    nc = np.array([0, 2, 4], dtype=np.int32)
    out, S, z, h = oracle.verify(q, k, v, w, S0, z0, h0, n_commit=nc, lib=lib)
    assert np.array_equal(out, all_out)
    assert np.array_equal(S[0], S0[0]) and np.array_equal(z[0], z0[0]) and np.array_equal(h[0], h0[0])
    for b, n in enumerate(nc):
        Ss, zs, hs = S0[b:b + 1], z0[b:b + 1], h0[b:b + 1]
        for j in range(n):
            _, Ss, zs, hs = oracle.decode(q[b:b + 1, :, j:j + 1], k[b:b + 1, :, j:j + 1], v[b:b + 1, :, j:j + 1],
                                          w, Ss, zs, hs, lib=lib)
        assert np.array_equal(S[b:b + 1], Ss) and np.array_equal(z[b:b + 1], zs) and np.array_equal(h[b:b + 1], hs), \
            f"batch {b} n_commit {n}"


def pin_verify_no_leak_between_drafts(lib=None):
    B, H, d, Kc, kk = 1, 2, 4, 3, 6
    q, k, v, w, S0, z0, h0 = _rand(43, B=B, H=H, L=kk, d=d, Kc=Kc, with_state=True)
    base = oracle.verify(q, k, v, w, S0, z0, h0, lib=lib)[0]
    for j in range(kk - 1):
        q2, k2, v2 = q.copy(), k.copy(), v.copy()
        for a in (q2, k2, v2):
            a[:, :, j + 1:] = -3.0 * a[:, :, j + 1:] + 1.0
        got = oracle.verify(q2, k2, v2, w, S0, z0, h0, lib=lib)[0]
        assert np.array_equal(got[:, :, :j + 1], base[:, :, :j + 1]), f"draft {j} saw a later draft"
        assert not np.array_equal(got[:, :, j + 1:], base[:, :, j + 1:])


# --- the other feature map: phi(x) = max(x, 0) (the "ReLU" linear attention of Sec. 3) ------------------
def pin_relu_feature_map_values(lib=None):
    xs = np.array([-30.0, -1.0, -1e-9, 0.0, 1e-9, 0.25, 7.5])
    with oracle.feature_map("relu", lib):
        got = oracle.phi(xs, lib=lib)
    assert np.array_equal(got, np.maximum(xs, 0.0))
    assert oracle.phi(np.array([0.0]), lib=lib)[0] == 1.0      # and the default is back afterwards


def pin_relu_on_inputs_above_one_is_the_default_map_shifted(lib=None):
    """For x > 1: max(x, 0) = x = elu(x - 1) + 1, so on such inputs the two maps must give the same
    results when the default map is fed q - 1 and k - 1 (every form, incoming state included)."""
    r = _rng(61)
    B, H, L, d, Kc = 2, 2, 9, 4, 3
    q, k = (1.0 + np.abs(r.standard_normal((B, H, L, d))) + 0.125 for _ in range(2))
    v = r.standard_normal((B, H, L, d))
    w = r.standard_normal((H, d, Kc))
    S0 = r.standard_normal((B, H, d, d)); z0 = np.abs(r.standard_normal((B, H, d))) + 0.5
    h0 = r.standard_normal((B, H, Kc - 1, d))
    for form in FORMS:
        want = getattr(oracle, form)(q - 1.0, k - 1.0, v, w, S0, z0, h0, eps=0.5, lib=lib)
        with oracle.feature_map("relu", lib):
            got = getattr(oracle, form)(q, k, v, w, S0, z0, h0, eps=0.5, lib=lib)
        for g, x, what in zip(got, want, ("out", "S", "z", "hist")):
            _close(g, x, 1e-12, f"relu {form} {what}")
    n_commit = np.array([4, 0], dtype=np.int32)
    want = oracle.verify(q - 1.0, k - 1.0, v, w, S0, z0, h0, n_commit, eps=0.5, lib=lib)
    parent = np.array([-1, 0, 0, 2, 1, 4, -1, 6, 3], dtype=np.int32)
    want_t = oracle.verify_tree(q - 1.0, k - 1.0, v, parent, w, S0, z0, h0, n_commit - 1, eps=0.5, lib=lib)
    with oracle.feature_map("relu", lib):
        got = oracle.verify(q, k, v, w, S0, z0, h0, n_commit, eps=0.5, lib=lib)
        got_t = oracle.verify_tree(q, k, v, parent, w, S0, z0, h0, n_commit - 1, eps=0.5, lib=lib)
    for g, x in zip(got + got_t, want + want_t):
        _close(g, x, 1e-12, "relu verify")


def pin_relu_drops_negative_entries(lib=None):
    """Negative entries of q and k do not exist for this map; with every key negative only eps and the
    convolution are left."""
    q, k, v, w = _rand(62, L=11)
    with oracle.feature_map("relu", lib):
        a = oracle.prefill_recurrent(q, k, v, w, eps=0.25, lib=lib)
        b = oracle.prefill_recurrent(np.maximum(q, 0.0), np.maximum(k, 0.0), v, w, eps=0.25, lib=lib)
        dead = oracle.prefill_quadratic(q, -np.abs(k) - 0.5, v, w, eps=0.25, lib=lib)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    _close(dead[0], oracle.causal_conv(v, w, None, lib=lib), 1e-12, "all keys dead: out = conv")
    assert np.all(dead[1] == 0.0) and np.all(dead[2] == 0.0)
    default = oracle.prefill_recurrent(q, k, v, w, eps=0.25, lib=lib)
    assert not np.allclose(a[0], default[0])


# --- tree-structured verification (Sec. 4.2, "Proposed Solution") -------------------------------
def _tree_case(seed, n=11, B=2, H=2, d=4, Kc=4):
    r = _rng(seed)
    parent = np.array([-1] + [int(r.integers(-1, i)) for i in range(1, n)], dtype=np.int32)
    q, k, v = (r.standard_normal((B, H, n, d)) for _ in range(3))
    w = r.standard_normal((H, d, Kc))
    S = r.standard_normal((B, H, d, d))
    z = np.abs(r.standard_normal((B, H, d))) + 0.5
    hist = r.standard_normal((B, H, Kc - 1, d))
    return parent, q, k, v, w, S, z, hist


def _root_path(parent, i):
    path = []
    while i >= 0:
        path.append(i)
        i = int(parent[i])
    return path[::-1]          # oldest first


def pin_tree_example_from_the_paper(lib=None):
    """Two candidates for the same step stored side by side: the second one's window is {t0, t1b}."""
    rows = {}
    for line in open(os.path.join(GOLDEN, "tree_verify_example.txt")):
        line = line.split("#")[0].strip()
        if line:
            node, rest = line.split(":")
            tok = rest.split()
            rows[int(node)] = (int(tok[1]), float(tok[-1]))
    parent = np.array([rows[i][0] for i in sorted(rows)], dtype=np.int32)
    v = np.array([2.0, 3.0, 11.0]).reshape(1, 1, 3, 1)
    zero = np.zeros_like(v)
    w = np.array([[[1.0, 10.0, 100.0]]])
    hist = np.array([5.0, 7.0]).reshape(1, 1, 2, 1)
    out = oracle.verify_tree(zero, zero, v, parent, w, np.zeros((1, 1, 1, 1)), np.zeros((1, 1, 1)), hist, lib=lib)[0]
    _close(out[0, 0, :, 0], [rows[i][1] for i in sorted(rows)], 1e-12, "paper's tree example")


def pin_tree_that_is_a_chain_is_plain_verify(lib=None):
    """parent[i] = i - 1 is the chain of drafts; accepting candidate n - 1 is n_commit = n."""
    parent, q, k, v, w, S, z, hist = _tree_case(31)
    n = q.shape[2]
    chain = np.arange(n, dtype=np.int32) - 1
    n_commit = np.array([4, 0], dtype=np.int32)
    got = oracle.verify_tree(q, k, v, chain, w, S, z, hist, n_commit - 1, eps=0.25, lib=lib)
    want = oracle.verify(q, k, v, w, S, z, hist, n_commit, eps=0.25, lib=lib)
    for g, x, what in zip(got, want, ("out", "S", "z", "hist")):
        _close(g, x, 1e-12, "chain tree " + what)


def pin_tree_candidate_equals_chain_over_its_root_path(lib=None):
    """Every candidate's output, and the state after accepting it, are those of plain verification of the
    tokens on its root path in time order (the same prefix is computed once, Sec. 5.3)."""
    parent, q, k, v, w, S, z, hist = _tree_case(32)
    n = q.shape[2]
    out = oracle.verify_tree(q, k, v, parent, w, S, z, hist, lib=lib)[0]
    for i in range(n):
        path = _root_path(parent, i)
        want = oracle.verify(q[:, :, path], k[:, :, path], v[:, :, path], w, S, z, hist, lib=lib)
        _close(out[:, :, i], want[0][:, :, -1], 1e-12, f"candidate {i}")
        got = oracle.verify_tree(q, k, v, parent, w, S, z, hist, np.array([i, -1], dtype=np.int32), lib=lib)
        for b in (0, 1):
            ref = want if b == 0 else (None, S, z, hist)
            _close(got[1][b], ref[1][b], 1e-12, f"S after accepting {i}, row {b}")
            _close(got[2][b], ref[2][b], 1e-12, f"z after accepting {i}, row {b}")
            _close(got[3][b], ref[3][b], 1e-12, f"hist after accepting {i}, row {b}")


def pin_tree_candidates_off_the_path_are_invisible(lib=None):
    """Changing any candidate that is not on the root path of candidate i leaves out[i] bit-identical."""
    parent, q, k, v, w, S, z, hist = _tree_case(33)
    n = q.shape[2]
    base = oracle.verify_tree(q, k, v, parent, w, S, z, hist, lib=lib)[0]
    for i in range(n):
        on = set(_root_path(parent, i))
        off = [a for a in range(n) if a not in on]
        if not off:
            continue
        q2, k2, v2 = q.copy(), k.copy(), v.copy()
        for a in (q2, k2, v2):
            a[:, :, off] = -3.0 * a[:, :, off] + 1.0
        other = oracle.verify_tree(q2, k2, v2, parent, w, S, z, hist, lib=lib)[0]
        assert np.array_equal(other[:, :, i], base[:, :, i]), f"candidate {i} saw a candidate off its path"
        for a in on:                                   # ... and every candidate on the path does matter
            v3 = v.copy()
            v3[:, :, a] += 1.0
            moved = oracle.verify_tree(q, k, v3, parent, w, S, z, hist, lib=lib)[0]
            assert not np.array_equal(moved[:, :, i], base[:, :, i]), f"candidate {i} ignores {a} on its path"


def pin_tree_without_acceptance_leaves_the_state(lib=None):
    parent, q, k, v, w, S, z, hist = _tree_case(34)
    for accept in (None, np.array([-1, -1], dtype=np.int32)):
        got = oracle.verify_tree(q, k, v, parent, w, S, z, hist, accept, lib=lib)
        assert np.array_equal(got[1], S) and np.array_equal(got[2], z) and np.array_equal(got[3], hist)


# --- the grouped (three-branch) form of Sec. 4.1 -------------------------------
def pin_grouped_single_group_is_library_softmax_attention(lib=None):
    """One group covering the sequence, no state: nothing precedes the group, so what is left is causal
    softmax attention with logits q.k/sqrt(d) (Eq. 1) -- a library routine -- plus the conv."""
    q, k, v, w = _rand(401, B=2, H=2, L=13, d=5, Kc=3)
    for group in (13, 64):
        got = oracle.prefill_grouped(q, k, v, w, group, alpha=0.7, lib=lib)[0]
        tq, tk, tv = (torch.from_numpy(a) for a in (q, k, v))
        want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True).numpy()
        _close(got, want + oracle.causal_conv(v, w), 1e-12, "one group vs library softmax attention")


def pin_grouped_one_token_groups_are_the_token_level_form_shifted(lib=None):
    """Groups of one token: the local branch is the token's own value (a softmax over one logit) and the
    grouped branch is linear attention over the strictly earlier tokens.  The latter is the token-level
    oracle run on keys and values moved one step later, the vacated first slot cancelled through the
    incoming normaliser (phi(0) = 1 per feature, value 0)."""
    q, k, v, w = _rand(402, B=1, H=2, L=9, d=4, Kc=3)
    eps = 0.3
    ks, vs = np.zeros_like(k), np.zeros_like(v)
    ks[:, :, 1:], vs[:, :, 1:] = k[:, :, :-1], v[:, :, :-1]
    B, H, L, d = q.shape
    w0 = np.zeros_like(w)
    earlier = oracle.prefill_recurrent(q, ks, vs, w0, S0=np.zeros((B, H, d, d)), z0=-np.ones((B, H, d)),
                                       hist0=np.zeros((B, H, 2, d)), eps=eps)[0]
    got = oracle.prefill_grouped(q, k, v, w, 1, alpha=1.0, eps=eps, lib=lib)[0]
    _close(got, earlier + v + oracle.causal_conv(v, w), 1e-12, "one-token groups")


def pin_grouped_closed_form_example(lib=None):
    """d = 1, Q = K = 0: every logit is 0 (uniform local weights) and phi = 1 (uniform linear weights), so
    the local branch is the mean of the group's values so far and the grouped branch the mean over all
    earlier groups.  Groups of 2, alpha = 2, taps (current, one back) = (1, 10), history 1:
        v      =  2   4   6  10   20
        local  =  2   3   6   8   20
        grouped=  -   -   3   3   5.5      (x alpha)
        conv   = 12  24  46  70  120
    """
    v = np.array([2.0, 4.0, 6.0, 10.0, 20.0]).reshape(1, 1, 5, 1)
    zero = np.zeros_like(v)
    w = np.array([1.0, 10.0]).reshape(1, 1, 2)
    got = oracle.prefill_grouped(zero, zero, v, w, 2, alpha=2.0, hist0=np.ones((1, 1, 1, 1)), lib=lib)
    _close(got[0].ravel(), [14.0, 27.0, 58.0, 84.0, 151.0], 1e-13, "closed-form example")
    _close(got[1].ravel(), [42.0], 1e-13, "S = sum of values (phi = 1)")
    _close(got[2].ravel(), [5.0], 1e-13, "z = number of tokens")


def pin_grouped_logit_scale(lib=None):
    """d = 4, two tokens, q_1.k_1 = 2 ln 3 and q_1.k_0 = 0: with logits divided by sqrt(d) = 2 the local
    weights of token 1 are (1/4, 3/4)."""
    q = np.zeros((1, 1, 2, 4)); k = np.zeros((1, 1, 2, 4))
    q[0, 0, 1, 0] = 2.0
    k[0, 0, 1, 0] = math.log(3.0)
    v = _rng(403).standard_normal((1, 1, 2, 4))
    got = oracle.prefill_grouped(q, k, v, np.zeros((1, 4, 1)), 2, alpha=0.0, lib=lib)[0]
    _close(got[0, 0, 0], v[0, 0, 0], 1e-14, "first token")
    _close(got[0, 0, 1], 0.25 * v[0, 0, 0] + 0.75 * v[0, 0, 1], 1e-14, "second token")


def pin_grouped_local_weights_ignore_a_common_logit_shift(lib=None):
    """Adding one vector to every key moves all logits of a query by the same amount: the local branch
    (alpha = 0 isolates it) does not change, however large the shift."""
    q, k, v, w = _rand(404, B=1, H=2, L=11, d=4, Kc=2)
    base = oracle.prefill_grouped(q, k, v, w, 4, alpha=0.0, lib=lib)[0]
    for shift in (0.5, 400.0):
        moved = oracle.prefill_grouped(q, k + shift * np.array([1.0, -2.0, 0.5, 3.0]), v, w, 4, alpha=0.0, lib=lib)[0]
        assert np.all(np.isfinite(moved)), "overflow in the local weights"
        _close(moved, base, 1e-9, f"shift {shift}")


def pin_grouped_alpha_weighs_the_grouped_branch_only(lib=None):
    """out is affine in alpha; the alpha-part is absent in the first group (nothing before it) and, in
    any group, does not depend on keys and values of that group."""
    q, k, v, w = _rand(405, B=1, H=2, L=12, d=3, Kc=3)
    o0, o1, o25 = (oracle.prefill_grouped(q, k, v, w, 4, alpha=a, lib=lib)[0] for a in (0.0, 1.0, 2.5))
    g = o1 - o0
    _close(o25 - o0, 2.5 * g, 1e-12, "affine in alpha")
    assert np.array_equal(o1[:, :, :4], o0[:, :, :4]), "first group has a grouped part"
    assert np.max(np.abs(g[:, :, 4:])) > 1e-3, "no grouped part after the first group"
    k2, v2 = k.copy(), v.copy()
    k2[:, :, 8:10] += 1.0
    v2[:, :, 8:10] -= 2.0
    p0, p1 = (oracle.prefill_grouped(q, k2, v2, w, 4, alpha=a, lib=lib)[0] for a in (0.0, 1.0))
    _close((p1 - p0)[:, :, 8:], g[:, :, 8:], 1e-12, "grouped part sees its own group")
    assert np.max(np.abs(p0[:, :, 9:] - o0[:, :, 9:])) > 1e-3, "local part does not see its own group"


def pin_grouped_split_at_a_group_boundary(lib=None):
    """Everything before a group boundary reaches later tokens through (S, z, hist) alone."""
    q, k, v, w, S0, z0, h0 = _rand(406, B=2, H=2, L=14, d=4, Kc=3, with_state=True)
    whole = oracle.prefill_grouped(q, k, v, w, 3, alpha=1.3, S0=S0, z0=z0, hist0=h0, eps=1e-3, lib=lib)
    cut = 6
    a = oracle.prefill_grouped(q[:, :, :cut], k[:, :, :cut], v[:, :, :cut], w, 3, alpha=1.3, S0=S0, z0=z0, hist0=h0, eps=1e-3, lib=lib)
    b = oracle.prefill_grouped(q[:, :, cut:], k[:, :, cut:], v[:, :, cut:], w, 3, alpha=1.3, S0=a[1], z0=a[2], hist0=a[3], eps=1e-3, lib=lib)
    _close(np.concatenate([a[0], b[0]], axis=2), whole[0], 1e-12, "outputs")
    for i, name in ((1, "S"), (2, "z"), (3, "hist")):
        _close(b[i], whole[i], 1e-12, name)


def pin_grouped_no_leak_and_long_memory(lib=None):
    """A later token never changes an earlier output (bit for bit); a token of the first group still
    reaches the last one (through the grouped branch)."""
    q, k, v, w = _rand(407, B=1, H=1, L=10, d=3, Kc=2)
    base = oracle.prefill_grouped(q, k, v, w, 4, alpha=1.0, lib=lib)[0]
    for j in (1, 4, 7, 9):
        q2, k2, v2 = q.copy(), k.copy(), v.copy()
        q2[:, :, j] += 1.0; k2[:, :, j] -= 1.0; v2[:, :, j] += 3.0
        o = oracle.prefill_grouped(q2, k2, v2, w, 4, alpha=1.0, lib=lib)[0]
        assert np.array_equal(o[:, :, :j], base[:, :, :j]), f"token {j} leaked backwards"
    v2 = v.copy(); v2[:, :, 0] += 5.0
    o = oracle.prefill_grouped(q, k, v2, w, 4, alpha=1.0, lib=lib)[0]
    assert np.max(np.abs(o[:, :, 9] - base[:, :, 9])) > 1e-3, "the first token is forgotten"


def pin_grouped_state_is_the_same_running_sum(lib=None):
    """The state handed back does not depend on the grouping: it is the token-level form's."""
    q, k, v, w, S0, z0, h0 = _rand(408, B=1, H=2, L=11, d=4, Kc=4, with_state=True)
    want = oracle.prefill_recurrent(q, k, v, w, S0=S0, z0=z0, hist0=h0)
    for group in (1, 4, 64):
        got = oracle.prefill_grouped(q, k, v, w, group, S0=S0, z0=z0, hist0=h0, lib=lib)
        for i, name in ((1, "S"), (2, "z"), (3, "hist")):
            _close(got[i], want[i], 1e-12, f"{name}, groups of {group}")


def pin_grouped_feature_map_touches_the_linear_branch_only(lib=None):
    """The feature map belongs to the linear branch: with alpha = 0 the output is the same under either
    map, while the state follows the map."""
    q, k, v, w = _rand(409, B=1, H=1, L=9, d=3, Kc=2)
    base = oracle.prefill_grouped(q, k, v, w, 4, alpha=0.0, lib=lib)
    with oracle.feature_map("relu", lib=lib):
        other = oracle.prefill_grouped(q, k, v, w, 4, alpha=0.0, lib=lib)
    _close(other[0], base[0], 1e-13, "local + conv under the other map")
    _close(other[1], np.einsum("bhti,bhtc->bhic", np.maximum(k, 0.0), v), 1e-12, "state under max(x, 0)")


# --- generation with the three-branch form ---------------------------------------
def _empty_grouped_state(B, H, d, Kc, C):
    return (np.zeros((B, H, d, d)), np.zeros((B, H, d)), np.zeros((B, H, Kc - 1, d)),
            np.zeros((B, H, C, d)), np.zeros((B, H, C, d)), np.zeros(B, dtype=np.int32))


def _window_sums(kwin, vwin, fill, lib=None):
    """sum of phi(k) v^T and of phi(k) over the window rows in use, per (b, h)"""
    B, H, C, d = kwin.shape
    S = np.zeros((B, H, d, d)); z = np.zeros((B, H, d))
    for b in range(B):
        fk = oracle.phi(kwin[b, :, :fill[b]], lib=lib) if fill[b] else np.zeros((H, 0, d))
        S[b] = np.einsum("hti,htc->hic", fk, vwin[b, :, :fill[b]])
        z[b] = fk.sum(axis=1)
    return S, z


def pin_grouped_steps_reproduce_the_grouped_prefill(lib=None):
    """Fed token by token, or in blocks of drafts that are all kept, a sequence gives the outputs of the
    whole-sequence form; what is carried is the state of the completed groups plus the open group's rows."""
    C = 4
    q, k, v, w, S0, z0, h0 = _rand(501, B=2, H=2, L=14, d=3, Kc=3, with_state=True)
    want = oracle.prefill_grouped(q, k, v, w, C, alpha=0.6, S0=S0, z0=z0, hist0=h0, eps=1e-3, lib=lib)
    for block in (1, 3, 5):
        st = (S0, z0, h0) + _empty_grouped_state(2, 2, 3, 3, C)[3:]
        outs = []
        for t0 in range(0, 14, block):
            sl = slice(t0, min(t0 + block, 14))
            r = oracle.verify_grouped(q[:, :, sl], k[:, :, sl], v[:, :, sl], w, C, *st, alpha=0.6, eps=1e-3, lib=lib)
            outs.append(r[0]); st = r[1:]
        _close(np.concatenate(outs, axis=2), want[0], 1e-12, f"outputs, blocks of {block}")
        assert st[5].tolist() == [14 % C] * 2, "rows in the open group"
        Sw, zw = _window_sums(st[3], st[4], st[5], lib=lib)
        _close(st[0] + Sw, want[1], 1e-12, "completed groups + open group = running sum (S)")
        _close(st[1] + zw, want[2], 1e-12, "completed groups + open group = running sum (z)")
        _close(st[2], want[3], 1e-12, "conv history")
        _close(st[3][:, :, :2], k[:, :, 12:14], 0, "open group's key rows")
        _close(st[4][:, :, :2], v[:, :, 12:14], 0, "open group's value rows")


def pin_grouped_verify_commit_counts(lib=None):
    """All outputs are produced whatever is kept; the state is the one after exactly n_commit[b] steps
    (crossing a group boundary or not); nothing kept = nothing changed, bit for bit."""
    C, kk = 4, 6
    r = _rng(502)
    B, H, d, Kc = 3, 2, 3, 3
    q, k, v = (r.standard_normal((B, H, kk, d)) for _ in range(3))
    w = r.standard_normal((H, d, Kc))
    st = (r.standard_normal((B, H, d, d)), np.abs(r.standard_normal((B, H, d))) + 0.5, r.standard_normal((B, H, Kc - 1, d)),
          r.standard_normal((B, H, C, d)), r.standard_normal((B, H, C, d)), np.array([1, 3, 0], dtype=np.int32))
    every = oracle.verify_grouped(q, k, v, w, C, *st, alpha=1.2, eps=1e-3, lib=lib)
    n_commit = np.array([0, 2, 5], dtype=np.int32)          # row 1 crosses the boundary (3 + 2 > 4), row 2 too (0 + 5)
    some = oracle.verify_grouped(q, k, v, w, C, *st, n_commit=n_commit, alpha=1.2, eps=1e-3, lib=lib)
    assert np.array_equal(some[0], every[0]), "outputs depend on what is kept"
    for b, n in enumerate(n_commit):
        sb = tuple(a[b:b + 1] for a in st)
        if n == 0:
            for got, was in zip(some[1:], st):
                assert np.array_equal(got[b], was[b]), "nothing kept, yet the state moved"
            continue
        ref = oracle.verify_grouped(q[b:b + 1, :, :n], k[b:b + 1, :, :n], v[b:b + 1, :, :n], w, C, *sb, alpha=1.2, eps=1e-3, lib=lib)
        for i in range(1, 7):
            _close(some[i][b], ref[i][0], 1e-13, f"row {b}, state item {i}")
    assert some[6].tolist() == [1, (3 + 2) % C, (0 + 5) % C]


def pin_grouped_verify_ignores_rows_beyond_fill_and_later_drafts(lib=None):
    """Window rows at or beyond fill are not part of the state; a later draft never changes an earlier output."""
    C, kk = 5, 4
    r = _rng(503)
    B, H, d, Kc = 2, 2, 3, 2
    q, k, v = (r.standard_normal((B, H, kk, d)) for _ in range(3))
    w = r.standard_normal((H, d, Kc))
    fill = np.array([2, 4], dtype=np.int32)
    st = [r.standard_normal((B, H, d, d)), np.abs(r.standard_normal((B, H, d))) + 0.5, r.standard_normal((B, H, Kc - 1, d)),
          r.standard_normal((B, H, C, d)), r.standard_normal((B, H, C, d)), fill]
    base = oracle.verify_grouped(q, k, v, w, C, *st, lib=lib)
    junk = [a.copy() for a in st]
    for b in range(B):
        junk[3][b, :, fill[b]:] = 77.0
        junk[4][b, :, fill[b]:] = -55.0
    other = oracle.verify_grouped(q, k, v, w, C, *junk, lib=lib)
    assert np.array_equal(other[0], base[0]), "rows beyond fill were read"
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    q2[:, :, 2:] += 1.0; k2[:, :, 2:] -= 1.0; v2[:, :, 2:] += 2.0
    later = oracle.verify_grouped(q2, k2, v2, w, C, *st, lib=lib)
    assert np.array_equal(later[0][:, :, :2], base[0][:, :, :2]), "a later draft leaked backwards"
    assert np.max(np.abs(later[0][:, :, 3] - base[0][:, :, 3])) > 1e-3


# ---- the sizes of the paper's FLASH experiment (Sec. 4.1: masked DWConv of kernel size 63; Sec. 5 "Settings": groups of 256) --
def pin_conv_of_63_taps_matches_library_grouped_conv(lib=None):
    """Kernel size 63: sequences shorter and longer than the window, with and without a 62-row history; in both
    prefill forms and in the three-branch form the conv is what is added on top of the attention output."""
    B, H, d, Kc = 1, 2, 3, 63
    r = _rng(901)
    w = r.standard_normal((H, d, Kc))
    for L in (5, 62, 63, 150):
        v = r.standard_normal((B, H, L, d))
        for hist in (None, r.standard_normal((B, H, Kc - 1, d))):
            left = np.zeros((B, H, Kc - 1, d)) if hist is None else hist
            x = np.concatenate([left, v], axis=2)
            x = torch.from_numpy(x).permute(0, 1, 3, 2).reshape(B, H * d, L + Kc - 1)
            wt = torch.from_numpy(w[:, :, ::-1].copy()).reshape(H * d, 1, Kc)
            want = torch.nn.functional.conv1d(x, wt, groups=H * d).reshape(B, H, d, L).permute(0, 1, 3, 2).numpy()
            _close(oracle.causal_conv(v, w, hist, lib=lib), want, 1e-12, f"63 taps vs conv1d, L={L}")
            q, k = r.standard_normal(v.shape), r.standard_normal(v.shape)
            for f in FORMS:
                fn = getattr(oracle, f)
                res = fn(q, k, v, w, hist0=hist, lib=lib)
                without = fn(q, k, v, np.zeros_like(w), hist0=hist, lib=lib)
                _close(res[0] - without[0], want, 1e-11, f"{f}: 63-tap conv added to the attention output, L={L}")
                _close(res[3], np.concatenate([left, v], axis=2)[:, :, -(Kc - 1):], 0.0, f"{f}: history after L={L}")
            g = oracle.prefill_grouped(q, k, v, w, 256, hist0=hist, lib=lib)
            g0 = oracle.prefill_grouped(q, k, v, np.zeros_like(w), 256, hist0=hist, lib=lib)
            _close(g[0] - g0[0], want, 1e-11, f"three-branch form: 63-tap conv added, L={L}")


def pin_grouped_256_token_groups(lib=None):
    """Groups of 256 tokens.  A sequence of at most 256 tokens is one group: library causal softmax attention plus
    the conv.  A longer one: its first 256 outputs are that again; the tokens after the boundary see the first
    group only through (S, z, hist), so they equal a fresh call started from the token-level state of the first
    256 tokens; and the state handed back is the token-level running sum."""
    q, k, v, w = _rand(902, B=1, H=2, L=300, d=4, Kc=5)
    tq, tk, tv = (torch.from_numpy(a[:, :, :256]) for a in (q, k, v))
    first = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True).numpy()
    conv = oracle.causal_conv(v, w)
    whole = oracle.prefill_grouped(q, k, v, w, 256, alpha=0.6, eps=1e-3, lib=lib)
    _close(whole[0][:, :, :256], first + conv[:, :, :256], 1e-11, "first group of 256 vs library softmax attention")
    st = oracle.prefill_recurrent(q[:, :, :256], k[:, :, :256], v[:, :, :256], w, lib=lib)
    tail = oracle.prefill_grouped(q[:, :, 256:], k[:, :, 256:], v[:, :, 256:], w, 256, alpha=0.6, S0=st[1], z0=st[2],
                                  hist0=st[3], eps=1e-3, lib=lib)
    _close(whole[0][:, :, 256:], tail[0], 1e-11, "tokens after the boundary")
    full = oracle.prefill_recurrent(q, k, v, w, lib=lib)
    for i, name in ((1, "S"), (2, "z"), (3, "hist")):
        _close(whole[i], full[i], 1e-11, name)
    # the group size is part of the result: 64-token groups give something else from token 64 on
    other = oracle.prefill_grouped(q, k, v, w, 64, alpha=0.6, eps=1e-3, lib=lib)[0]
    _close(other[:, :, :64], whole[0][:, :, :64], 1e-11, "before the first 64-token boundary")
    assert np.max(np.abs(other[:, :, 64:] - whole[0][:, :, 64:])) > 1e-3


# ---- value rows wider than key rows (Sec. 3, Eq. 1: Q, K in R^{n x d_k}, V in R^{n x d_v}) ----------------------------
def _wide_case(seed, B=2, H=2, L=9, d=3, m=2, Kc=3):
    r = _rng(seed)
    q, k = r.standard_normal((B, H, L, d)), r.standard_normal((B, H, L, d))
    v = r.standard_normal((B, H, L, m * d))
    w = r.standard_normal((H, m * d, Kc))
    S0 = r.standard_normal((B, H, d, m * d))
    z0 = np.abs(r.standard_normal((B, H, d))) + 1.0
    h0 = r.standard_normal((B, H, Kc - 1, m * d))
    return q, k, v, w, S0, z0, h0


def pin_wide_values_exact_rational_brute_force(lib=None):
    """d_k = 2, d_v = 4, one head, four tokens, an incoming state and history: every output, S, z and the history
    from the definition in exact rational arithmetic (inputs are small integers or logs of 1/2 and 1/4, whose
    feature-map values are rationals), in both prefill forms and token by token."""
    ln2, ln4 = math.log(0.5), math.log(0.25)
    q = np.array([[0.0, 1.0], [ln2, 2.0], [1.0, ln4], [0.0, 0.0]])
    k = np.array([[1.0, 0.0], [ln4, 1.0], [0.0, ln2], [2.0, 1.0]])
    v = np.array([[1.0, -2.0, 3.0, 0.0], [0.0, 1.0, -1.0, 2.0], [2.0, 2.0, 0.0, -3.0], [-1.0, 0.0, 1.0, 1.0]])
    w = np.array([[1.0, -1.0], [2.0, 0.5], [0.0, 3.0], [-2.0, 1.0]])          # [d_v][Kc = 2]
    S0 = np.array([[1.0, 0.0, -1.0, 2.0], [0.5, 1.0, 0.0, -0.5]])               # [d_k][d_v]
    z0 = np.array([2.0, 1.0])
    h0 = np.array([[3.0, -1.0, 0.5, 2.0]])                                       # [Kc - 1][d_v]
    F = Fraction
    phi = lambda x: F(x) + 1 if x > 0 else _phi_frac(x) if x < 0 else F(1)
    fq = [[phi(x) for x in row] for row in q]
    fk = [[phi(x) for x in row] for row in k]
    S = [[F(x) for x in row] for row in S0]
    z = [F(x) for x in z0]
    want = []
    for t in range(4):
        for i in range(2):
            z[i] += fk[t][i]
            for c in range(4):
                S[i][c] += fk[t][i] * F(v[t][c])
        den = sum(fq[t][i] * z[i] for i in range(2))
        row = []
        for c in range(4):
            prev = F(v[t - 1][c]) if t > 0 else F(h0[0][c])
            row.append(sum(fq[t][i] * S[i][c] for i in range(2)) / den + F(w[c][0]) * F(v[t][c]) + F(w[c][1]) * prev)
        want.append(row)
    want = np.array([[float(x) for x in row] for row in want])
    args = (q[None, None], k[None, None], v[None, None], w[None], S0[None, None], z0[None, None], h0[None, None])
    for f in FORMS:
        got = getattr(oracle, f)(*args, lib=lib)
        _close(got[0][0, 0], want, 1e-13, f + " wide values: outputs")
        _close(got[1][0, 0], np.array([[float(x) for x in row] for row in S]), 1e-13, f + " wide values: S")
        _close(got[2][0, 0], np.array([float(x) for x in z]), 1e-13, f + " wide values: z")
        _close(got[3][0, 0], v[3:4], 0.0, f + " wide values: history")
    got = oracle.verify(*args, lib=lib)
    _close(got[0][0, 0], want, 1e-13, "verify, wide values: outputs")


def pin_wide_values_zero_keys_give_running_mean(lib=None):
    """K == 0 makes every weight equal: the attention part is the running mean of the d_v-wide value rows."""
    q, k, v, w, _, _, _ = _wide_case(911, L=12, d=3, m=3)
    k = np.zeros_like(k)
    want = np.cumsum(v, axis=2) / np.arange(1, v.shape[2] + 1)[None, None, :, None]
    for f in FORMS:
        _close(getattr(oracle, f)(q, k, v, np.zeros_like(w), lib=lib)[0], want, 1e-12, f + " running mean, wide values")


def pin_wide_values_verify_is_sequential_decode_and_prefill(lib=None):
    """With d_v = 2 d_k as with d_v = d_k: k drafts at once = k decode steps = the same tokens through the prefill;
    commit counts move the state over the kept drafts only."""
    q, k, v, w, S0, z0, h0 = _wide_case(912, L=5, d=4, m=2, Kc=4)
    ver = oracle.verify(q, k, v, w, S0, z0, h0, lib=lib)
    pre = oracle.prefill_recurrent(q, k, v, w, S0, z0, h0, lib=lib)
    for x, y, n in zip(ver, pre, ("out", "S", "z", "hist")):
        _close(x, y, 1e-12, "verify vs prefill, wide values: " + n)
    S, z, h = S0, z0, h0
    for j in range(5):
        o, S, z, h = oracle.decode(q[:, :, j:j + 1], k[:, :, j:j + 1], v[:, :, j:j + 1], w, S, z, h, lib=lib)
        _close(o, ver[0][:, :, j:j + 1], 1e-12, f"decode step {j}, wide values")
    part = oracle.verify(q, k, v, w, S0, z0, h0, np.array([2, 0], dtype=np.int32), lib=lib)
    two = oracle.prefill_recurrent(q[:1, :, :2], k[:1, :, :2], v[:1, :, :2], w, S0[:1], z0[:1], h0[:1], lib=lib)
    _close(part[1][:1], two[1], 1e-12, "two kept drafts: S")
    _close(part[3][:1], two[3], 0.0, "two kept drafts: history")
    _close(part[1][1:], S0[1:], 0.0, "nothing kept: S untouched")


# --- gradient of the three-branch form (training direction) --------------------------------------------------
def _fd_gradients(loss, arrays, h=1e-6):
    """Central differences of a scalar function of several arrays, element by element (the arrays are changed in place
    and restored)."""
    grads = []
    for a in arrays:
        g = np.zeros_like(a)
        it = np.nditer(a, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = a[idx]
            a[idx] = old + h
            up = loss()
            a[idx] = old - h
            dn = loss()
            a[idx] = old
            g[idx] = (up - dn) / (2 * h)
        grads.append(g)
    return grads


def _backward_case(seed, B=2, H=2, L=11, d=3, Kc=3):
    r = _rng(seed)
    q, k, v = (r.standard_normal((B, H, L, d)) for _ in range(3))
    w = r.standard_normal((H, d, Kc))
    S0 = 0.3 * r.standard_normal((B, H, d, d)) + 0.5
    z0 = r.random((B, H, d)) + 0.5
    h0 = r.standard_normal((B, H, Kc - 1, d))
    dout = r.standard_normal((B, H, L, d))
    dS1 = r.standard_normal((B, H, d, d))
    dz1 = r.standard_normal((B, H, d))
    return q, k, v, w, S0, z0, h0, dout, dS1, dz1


_GRAD_NAMES = ("dq", "dk", "dv", "dw", "dS0", "dz0", "dhist0")


def pin_grouped_backward_matches_finite_differences_of_the_forward(lib=None):
    """The gradient is by definition the derivative of the (pinned) forward function: central differences of
    sum(dout*out) + sum(dS1*S1) + sum(dz1*z1) in fp64, every element of every input, short last group included."""
    for seed, group, alpha, eps in ((501, 4, 0.7, 0.1), (502, 3, 1.0, 0.0), (503, 16, 1.9, 0.0)):
        q, k, v, w, S0, z0, h0, dout, dS1, dz1 = _backward_case(seed)
        args = [q, k, v, w, S0, z0, h0]

        def loss():
            o, S1, z1, _ = oracle.prefill_grouped(q, k, v, w, group, alpha, S0, z0, h0, eps, lib=lib)
            return float((o * dout).sum() + (S1 * dS1).sum() + (z1 * dz1).sum())

        got = oracle.prefill_grouped_backward(q, k, v, w, dout, group, alpha, S0, z0, h0, dS1, dz1, eps, lib=lib)
        for name, fd in zip(_GRAD_NAMES, _fd_gradients(loss, args)):
            _close(got[name], fd, 2e-7, f"{name} (group {group})")


def pin_grouped_backward_from_an_empty_state(lib=None):
    """No incoming state, eps = 0: the first group has no grouped branch at all (its denominator is exactly zero), and the
    gradient must say the same; this is the training case."""
    q, k, v, w, _, _, _, dout, _, _ = _backward_case(504, L=10)
    for group in (4, 5):
        def loss():
            return float((oracle.prefill_grouped(q, k, v, w, group, 1.3, lib=lib)[0] * dout).sum())

        got = oracle.prefill_grouped_backward(q, k, v, w, dout, group, 1.3, lib=lib)
        for name, fd in zip(_GRAD_NAMES[:4], _fd_gradients(loss, [q, k, v, w])):
            _close(got[name], fd, 2e-7, f"{name} (group {group}, empty state)")
        assert np.all(np.isfinite(got["dq"]))


def pin_grouped_backward_single_group_is_the_library_attention_gradient(lib=None):
    """One group, no state, zero conv weights: the function is the library's causal softmax attention, and its gradient
    is what the library's own differentiation gives."""
    r = _rng(505)
    B, H, L, d = 2, 2, 9, 4
    q, k, v, dout = (r.standard_normal((B, H, L, d)) for _ in range(4))
    w = np.zeros((H, d, 2))
    got = oracle.prefill_grouped_backward(q, k, v, w, dout, 16, alpha=0.4, lib=lib)
    tq, tk, tv = (torch.from_numpy(a).requires_grad_(True) for a in (q, k, v))
    out = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    out.backward(torch.from_numpy(dout))
    for name, t in (("dq", tq), ("dk", tk), ("dv", tv)):
        _close(got[name], t.grad.numpy(), 1e-12, f"{name} vs library attention gradient")


def pin_grouped_backward_conv_part_is_the_library_conv_gradient(lib=None):
    """The conv branch adds to the output, so it adds to dv, and it alone feeds dw and dhist0: the difference to a run
    with zero weights, and dw / dhist0 themselves, against the library's differentiation of its grouped conv1d."""
    q, k, v, w, S0, z0, h0, dout, _, _ = _backward_case(506, L=12, d=4, Kc=5)
    B, H, L, d = q.shape
    Kc = w.shape[2]
    got = oracle.prefill_grouped_backward(q, k, v, w, dout, 4, 1.0, S0, z0, h0, lib=lib)
    base = oracle.prefill_grouped_backward(q, k, v, np.zeros_like(w), dout, 4, 1.0, S0, z0, h0, lib=lib)
    ext = torch.from_numpy(np.concatenate([h0, v], axis=2)).requires_grad_(True)      # [B, H, Kc-1+L, d]
    tw = torch.from_numpy(w).requires_grad_(True)
    x = ext.permute(0, 1, 3, 2).reshape(B, H * d, Kc - 1 + L)                          # channels = (h, c)
    ker = torch.flip(tw, dims=[2]).reshape(H * d, 1, Kc)                               # tap j meets v[t-j]
    u = torch.nn.functional.conv1d(x, ker, groups=H * d).reshape(B, H, d, L).permute(0, 1, 3, 2)
    u.backward(torch.from_numpy(dout))
    g_ext = ext.grad.numpy()
    _close(got["dv"] - base["dv"], g_ext[:, :, Kc - 1:], 1e-12, "conv part of dv")
    _close(got["dhist0"], g_ext[:, :, :Kc - 1], 1e-12, "dhist0")
    _close(got["dw"], tw.grad.numpy(), 1e-12, "dw")
    for name in ("dq", "dk", "dS0", "dz0"):
        assert np.array_equal(got[name], base[name]), f"{name} must not depend on the conv weights"


def pin_grouped_backward_is_linear_in_dout(lib=None):
    q, k, v, w, S0, z0, h0, d1, dS1, dz1 = _backward_case(507)
    d2 = _rng(508).standard_normal(d1.shape)
    a = oracle.prefill_grouped_backward(q, k, v, w, d1, 4, 0.8, S0, z0, h0, eps=0.05, lib=lib)
    b = oracle.prefill_grouped_backward(q, k, v, w, d2, 4, 0.8, S0, z0, h0, eps=0.05, lib=lib)
    c = oracle.prefill_grouped_backward(q, k, v, w, 2.0 * d1 - 0.5 * d2, 4, 0.8, S0, z0, h0, eps=0.05, lib=lib)
    for name in _GRAD_NAMES:
        _close(c[name], 2.0 * a[name] - 0.5 * b[name], 1e-12, name)


def pin_grouped_backward_is_causal(lib=None):
    """A loss that looks at token t alone cannot move because of a later token: dk, dv are exactly zero after t, dq is
    exactly zero everywhere but at t; and it does depend on the first token (through the sums) and on its own group."""
    q, k, v, w, S0, z0, h0, dout, _, _ = _backward_case(509, L=13)
    t = 9                                                # the second token of the group 8..11
    only = np.zeros_like(dout)
    only[:, :, t] = dout[:, :, t]
    g = oracle.prefill_grouped_backward(q, k, v, w, only, 4, 1.0, S0, z0, h0, lib=lib)
    assert np.all(g["dk"][:, :, t + 1:] == 0.0) and np.all(g["dv"][:, :, t + 1:] == 0.0)
    assert np.all(g["dq"][:, :, :t] == 0.0) and np.all(g["dq"][:, :, t + 1:] == 0.0)
    assert np.all(np.abs(g["dq"][:, :, t]).max(axis=-1) > 0)
    assert np.all(np.abs(g["dk"][:, :, 0]).max(axis=-1) > 0) and np.all(np.abs(g["dv"][:, :, 0]).max(axis=-1) > 0)
    assert np.all(np.abs(g["dk"][:, :, t]).max(axis=-1) > 0)        # its own key: the local branch
    # token 8 of t's own group reaches it through the local branch only, tokens 4..7 of the group before through the sums
    # only: both kinds must be there
    assert np.all(np.abs(g["dv"][:, :, 8]).max(axis=-1) > 0) and np.all(np.abs(g["dk"][:, :, 8]).max(axis=-1) > 0)
    assert np.all(np.abs(g["dv"][:, :, 5]).max(axis=-1) > 0) and np.all(np.abs(g["dk"][:, :, 5]).max(axis=-1) > 0)


def pin_grouped_backward_chains_across_a_split(lib=None):
    """A sequence cut at a group boundary is two calls chained through (S, z, hist); the gradient chains the other way
    round through (dS0, dz0, dhist0) of the second call."""
    q, k, v, w, S0, z0, h0, dout, dS1, dz1 = _backward_case(510, L=14, d=4, Kc=3)
    Kc = w.shape[2]
    G, cut = 3, 6
    whole = oracle.prefill_grouped_backward(q, k, v, w, dout, G, 1.3, S0, z0, h0, dS1, dz1, eps=1e-3, lib=lib)
    fa = oracle.prefill_grouped(q[:, :, :cut], k[:, :, :cut], v[:, :, :cut], w, G, 1.3, S0, z0, h0, eps=1e-3, lib=lib)
    gb = oracle.prefill_grouped_backward(q[:, :, cut:], k[:, :, cut:], v[:, :, cut:], w, dout[:, :, cut:], G, 1.3,
                                         fa[1], fa[2], fa[3], dS1, dz1, eps=1e-3, lib=lib)
    ga = oracle.prefill_grouped_backward(q[:, :, :cut], k[:, :, :cut], v[:, :, :cut], w, dout[:, :, :cut], G, 1.3,
                                         S0, z0, h0, gb["dS0"], gb["dz0"], eps=1e-3, lib=lib)
    dv_a = ga["dv"].copy()
    dv_a[:, :, cut - (Kc - 1):] += gb["dhist0"]          # the second call's history is the first call's last rows
    _close(np.concatenate([ga["dq"], gb["dq"]], axis=2), whole["dq"], 1e-12, "dq")
    _close(np.concatenate([ga["dk"], gb["dk"]], axis=2), whole["dk"], 1e-12, "dk")
    _close(np.concatenate([dv_a, gb["dv"]], axis=2), whole["dv"], 1e-12, "dv")
    _close(ga["dw"] + gb["dw"], whole["dw"], 1e-12, "dw")
    for name in ("dS0", "dz0", "dhist0"):
        _close(ga[name], whole[name], 1e-12, name)


def pin_grouped_backward_closed_form_for_zero_queries_and_keys(lib=None):
    """Q = K = 0: every feature is 1 and every logit 0, so out_t = alpha * mean(v before t's group) + mean(v of the group up
    to t) + conv, and dv follows by hand: token i receives alpha * dout_t / (tokens before t's group) from every t of a
    later group and dout_t / (t - g0 + 1) from every t >= i of its own group (plus the conv part, zero here)."""
    r = _rng(511)
    B, H, L, d, G, alpha = 1, 2, 10, 3, 4, 0.6
    v, dout = r.standard_normal((B, H, L, d)), r.standard_normal((B, H, L, d))
    zero = np.zeros((B, H, L, d))
    got = oracle.prefill_grouped_backward(zero, zero, v, np.zeros((H, d, 2)), dout, G, alpha, lib=lib)
    want = np.zeros_like(v)
    for t in range(L):
        g0 = (t // G) * G
        for i in range(g0):
            want[:, :, i] += alpha * dout[:, :, t] / g0
        for i in range(g0, t + 1):
            want[:, :, i] += dout[:, :, t] / (t - g0 + 1)
    _close(got["dv"], want, 1e-12, "dv, closed form")


def pin_grouped_backward_relu_map_matches_finite_differences(lib=None):
    """The other feature map (derivative 1 above zero, 0 below); inputs kept away from the kink."""
    q, k, v, w, S0, z0, h0, dout, dS1, dz1 = _backward_case(512, L=9)
    q[np.abs(q) < 0.05] = 0.3
    k[np.abs(k) < 0.05] = -0.3
    with oracle.feature_map("relu", lib):
        def loss():
            o, S1, z1, _ = oracle.prefill_grouped(q, k, v, w, 4, 0.9, S0, z0, h0, 0.5, lib=lib)
            return float((o * dout).sum() + (S1 * dS1).sum() + (z1 * dz1).sum())

        got = oracle.prefill_grouped_backward(q, k, v, w, dout, 4, 0.9, S0, z0, h0, dS1, dz1, 0.5, lib=lib)
        fds = _fd_gradients(loss, [q, k, v, w, S0, z0, h0])
    for name, fd in zip(_GRAD_NAMES, fds):
        _close(got[name], fd, 2e-7, f"{name} (relu map)")
    # a negative key entry is invisible to the sums: its derivative comes from the local branch alone, which does not
    # know alpha, dS1 or dz1
    with oracle.feature_map("relu", lib):
        other = oracle.prefill_grouped_backward(q, k, v, w, dout, 4, 0.0, S0, z0, h0, None, None, 0.5, lib=lib)
    _close(got["dk"][k < 0], other["dk"][k < 0], 1e-12, "dk of negative key entries")


ALL_PINS = [obj for name, obj in sorted(globals().items()) if name.startswith("pin_") and callable(obj)]
