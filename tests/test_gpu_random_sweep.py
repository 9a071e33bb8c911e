"""Seeded random sweeps over the entry points: shapes, layouts, feature maps, states and commit patterns drawn at random
(fixed seeds, so every run sees the same cases), each compared with the oracle through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from parity import STATE_TOL, TOL, check, dev, host
from paper_2406_07368_amd import binding, workloads

pytestmark = pytest.mark.gpu

IO = {"f32": torch.float32, "bf16": torch.bfloat16}
LENGTHS = [1, 2, 63, 64, 65, 127, 128, 129, 191, 257, 300, 511, 777, 1025, 1500, 2050]


def random_state(rng, B, H, d, Kc, io):
    return ((rng.standard_normal((B, H, d, d)) * 3).astype(np.float32),
            (np.abs(rng.standard_normal((B, H, d))) * 5 + 1).astype(np.float32),
            workloads.round_to_io(rng.standard_normal((B, H, Kc - 1, d)), io))


def in_layout(a, dt, layout, pad=24):
    """dense [B,H,L,d]; a transposed view of a token-major tensor; or a view into a longer, padded tensor"""
    t = dev(a, dt)
    if layout == "blhd":
        return t.transpose(1, 2).contiguous().transpose(1, 2)
    if layout == "padded":
        B, H, L, d = t.shape
        big = torch.zeros((B, H, L + pad, d), dtype=dt, device="cuda")
        big[:, :, :L] = t
        return big[:, :, :L]
    return t


@pytest.mark.parametrize("seed", range(24))
def test_prefill_random_case(seed):
    """Both prefill forms on the same random case (the three-branch form with groups of 64)."""
    rng = np.random.default_rng(9000 + seed)
    io = "bf16" if rng.random() < 0.8 else "f32"
    d, chunk, Kc = int(rng.choice([64, 128])), int(rng.choice([64, 128])), int(rng.integers(1, 9))
    B, H = int(rng.integers(1, 4)), int(rng.integers(1, 5))
    L = int(rng.choice(LENGTHS))
    if io == "f32":
        L = min(L, 300)
    layout = str(rng.choice(["bhld", "blhd", "padded"]))
    phi = "relu" if rng.random() < 0.25 else "elu1"
    eps = 0.05 if phi == "relu" else float(rng.choice([0.0, 1e-3]))
    alpha = float(rng.choice([1.0, 0.5, 2.0]))
    q, k, v = (workloads.round_to_io(rng.standard_normal((B, H, L, d)), io) for _ in range(3))
    w = workloads.conv_weights(rng, H, d, Kc)
    state = random_state(rng, B, H, d, Kc, io) if rng.random() < 0.5 else None
    what = f"seed {seed}: {io} d{d} chunk{chunk} Kc{Kc} B{B} H{H} L{L} {layout} {phi} state={state is not None}"
    print(what, flush=True)
    dt = IO[io]
    args = (None, None, None) if state is None else state
    with oracle.feature_map(phi):
        want = oracle.prefill_recurrent(q, k, v, w, *args, eps=eps)
        want_g = oracle.prefill_grouped(q, k, v, w, 64, alpha, *args, eps=eps)
    gq, gk, gv, gw = in_layout(q, dt, layout), in_layout(k, dt, layout), in_layout(v, dt, layout), dev(w)

    def gpu_state():
        return None if state is None else (dev(state[0]), dev(state[1]), dev(state[2], dt))

    def compare(got, ref, tag):
        out, (S, z, h) = got
        torch.cuda.synchronize()
        check(host(out), ref[0], TOL[io], f"{what} {tag} out")
        check(host(S), ref[1], TOL[io], f"{what} {tag} S")
        check(host(z), ref[2], TOL[io], f"{what} {tag} z")
        assert np.array_equal(host(h), workloads.round_to_io(ref[3], io).astype(np.float64)), f"{what} {tag} hist"

    compare(binding.prefill(gq, gk, gv, gw, gpu_state(), chunk, eps, phi=phi), want, "token-level")
    compare(binding.prefill_grouped(gq, gk, gv, gw, alpha, gpu_state(), eps, phi=phi), want_g, "three-branch")


@pytest.mark.parametrize("seed", range(16))
def test_groups_of_256_random_case(seed):
    """The three-branch form in groups of 256 (bf16 rows): forward with and without an incoming state, any tap count up
    to 63 (up to 8 taps the attention kernel adds the conv itself, beyond that it adds to what the conv pass wrote),
    and its gradient, for which the conv pass always runs first and beside the other kernels."""
    rng = np.random.default_rng(9500 + seed)
    d = int(rng.choice([64, 128]))
    Kc = int(rng.choice([1, 2, 3, 5, 8, 9, 16, 17, 33, 63]))
    B, H = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    L = int(rng.choice([1, 31, 255, 256, 257, 300, 511, 513, 777, 1025, 1300]))
    layout = str(rng.choice(["bhld", "blhd", "padded"]))
    phi = "relu" if rng.random() < 0.25 else "elu1"
    eps = 0.05 if phi == "relu" else float(rng.choice([0.0, 1e-3]))
    alpha = float(rng.choice([1.0, 0.5, 2.0]))
    scale = float(rng.choice([1.0, 0.5, d ** -0.5]))
    q, k, v = (workloads.round_to_io(rng.standard_normal((B, H, L, d)) * scale, "bf16") for _ in range(3))
    w = workloads.conv_weights(rng, H, d, Kc)
    dout = workloads.upstream_gradient((B, H, L, d), "bf16", 9600 + seed)
    state = random_state(rng, B, H, d, Kc, "bf16") if rng.random() < 0.5 else None
    what = f"seed {seed}: d{d} Kc{Kc} B{B} H{H} L{L} {layout} {phi} alpha {alpha} scale {scale:.3f} state={state is not None}"
    print(what, flush=True)
    dt = torch.bfloat16
    args = (None, None, None) if state is None else state
    with oracle.feature_map(phi):
        want = oracle.prefill_grouped(q, k, v, w, 256, alpha, *args, eps=eps)
        want_b = oracle.prefill_grouped_backward(q, k, v, w, dout, 256, alpha=alpha, eps=eps)
    gq, gk, gv, gd = (in_layout(x, dt, layout) for x in (q, k, v, dout))
    gw = dev(w)
    gstate = None if state is None else (dev(state[0]), dev(state[1]), dev(state[2], dt))
    out, (S, z, h) = binding.prefill_grouped(gq, gk, gv, gw, alpha, gstate, eps, phi=phi, group=256)
    dq, dk, dv, dw = binding.prefill_grouped_backward(gq, gk, gv, gw, gd, alpha, eps, phi=phi, group=256)
    torch.cuda.synchronize()
    check(host(out), want[0], TOL["bf16"], f"{what} out")
    check(host(S), want[1], TOL["bf16"], f"{what} S")
    check(host(z), want[2], TOL["bf16"], f"{what} z")
    assert np.array_equal(host(h), workloads.round_to_io(want[3], "bf16").astype(np.float64)), f"{what} hist"
    for name, got in (("dq", dq), ("dk", dk), ("dv", dv)):
        check(host(got), want_b[name], TOL["bf16"], f"{what} {name}")
    rms = max(float(np.sqrt(np.mean(want_b["dw"] ** 2))), 1e-30)
    err = float(np.max(np.abs(host(dw) - want_b["dw"]))) / rms
    assert err <= TOL["f32"], f"{what} dw: max abs err / rms {err:.3e}"


@pytest.mark.parametrize("seed", range(16))
def test_verify_random_case(seed):
    """Chain verify with random commit counts; whole heads (matrix cores) and split heads (streaming kernel)."""
    rng = np.random.default_rng(9100 + seed)
    io = "bf16" if rng.random() < 0.75 else "f32"
    d, Kc, kk = int(rng.choice([64, 128])), int(rng.integers(1, 9)), int(rng.integers(1, 17))
    B, H = (int(rng.integers(24, 28)), 32) if rng.random() < 0.4 else (int(rng.integers(1, 5)), int(rng.integers(1, 6)))
    phi = "relu" if rng.random() < 0.25 else "elu1"
    eps = 0.05 if phi == "relu" else 1e-3
    what = f"seed {seed}: {io} d{d} Kc{Kc} k{kk} B{B} H{H} {phi}"
    print(what, flush=True)
    S, z, hist = random_state(rng, B, H, d, Kc, io)
    S = np.abs(S)                                                 # a state that positive features could have produced
    q, k, v = (workloads.round_to_io(rng.standard_normal((B, H, kk, d)), io) for _ in range(3))
    w = workloads.conv_weights(rng, H, d, Kc)
    n_commit = None if rng.random() < 0.3 else rng.integers(0, kk + 1, size=B).astype(np.int32)
    with oracle.feature_map(phi):
        want = oracle.verify(q, k, v, w, S, z, hist, n_commit, eps=eps)
    dt = IO[io]
    state = (dev(S), dev(z), dev(hist, dt))
    nc = None if n_commit is None else torch.from_numpy(n_commit).cuda()
    out = binding.verify(dev(q, dt), dev(k, dt), dev(v, dt), dev(w), state, nc, eps, phi=phi)
    torch.cuda.synchronize()
    check(host(out), want[0], TOL[io], what + " out")
    check(host(state[0]), want[1], STATE_TOL, what + " S")
    check(host(state[1]), want[2], STATE_TOL, what + " z")
    assert np.array_equal(host(state[2]), workloads.round_to_io(want[3], io).astype(np.float64)), what + " hist"


@pytest.mark.parametrize("seed", range(12))
def test_verify_tree_random_case(seed):
    """Random candidate trees (random parents, any number of candidates up to 64) with random acceptances."""
    rng = np.random.default_rng(9200 + seed)
    d, Kc, n = int(rng.choice([64, 128])), int(rng.integers(1, 9)), int(rng.integers(1, 65))
    B, H = int(rng.integers(1, 5)), int(rng.integers(1, 6))
    phi = "relu" if rng.random() < 0.25 else "elu1"
    eps = 0.05 if phi == "relu" else 1e-3
    parent = np.array([-1] + [int(rng.integers(-1, i)) for i in range(1, n)], dtype=np.int32)
    accept = None if rng.random() < 0.2 else rng.integers(-1, n, size=B).astype(np.int32)
    what = f"seed {seed}: d{d} Kc{Kc} n{n} B{B} H{H} {phi} accept={'none' if accept is None else accept.tolist()}"
    print(what, flush=True)
    S, z, hist = random_state(rng, B, H, d, Kc, "bf16")
    S = np.abs(S)
    q, k, v = (workloads.round_to_io(rng.standard_normal((B, H, n, d)), "bf16") for _ in range(3))
    w = workloads.conv_weights(rng, H, d, Kc)
    with oracle.feature_map(phi):
        want = oracle.verify_tree(q, k, v, parent, w, S, z, hist, accept, eps=eps)
    dt = torch.bfloat16
    state = (dev(S), dev(z), dev(hist, dt))
    acc = None if accept is None else torch.from_numpy(accept).cuda()
    out = binding.verify_tree(dev(q, dt), dev(k, dt), dev(v, dt), torch.from_numpy(parent).cuda(), dev(w), state, acc, eps, phi=phi)
    torch.cuda.synchronize()
    check(host(out), want[0], TOL["bf16"], what + " out")
    check(host(state[0]), want[1], STATE_TOL, what + " S")
    check(host(state[1]), want[2], STATE_TOL, what + " z")
    assert np.array_equal(host(state[2]), workloads.round_to_io(want[3], "bf16").astype(np.float64)), what + " hist"


@pytest.mark.parametrize("seed", range(16))
def test_verify_grouped_random_case(seed):
    """Generation with the three-branch form: random open-group lengths per batch row (so some rows complete their
    group and some drafts fall into the next one), random commit counts."""
    rng = np.random.default_rng(9300 + seed)
    io = "bf16" if rng.random() < 0.7 else "f32"
    d, Kc, kk = int(rng.choice([64, 128])), int(rng.integers(1, 9)), int(rng.integers(1, 17))
    B, H = int(rng.integers(1, 5)), int(rng.integers(1, 6))
    phi = "relu" if rng.random() < 0.25 else "elu1"
    eps = 0.05 if phi == "relu" else 1e-3
    alpha = float(rng.choice([1.0, 0.5, 2.0]))
    fill = rng.choice([0, 1, 31, 47, 48, 55, 60, 62, 63], size=B).astype(np.int32)
    n_commit = None if rng.random() < 0.3 else rng.integers(0, kk + 1, size=B).astype(np.int32)
    what = f"seed {seed}: {io} d{d} Kc{Kc} k{kk} B{B} H{H} {phi} fill={fill.tolist()} keep={'all' if n_commit is None else n_commit.tolist()}"
    print(what, flush=True)
    S, z, hist = random_state(rng, B, H, d, Kc, io)
    kwin, vwin = (workloads.round_to_io(rng.standard_normal((B, H, 64, d)), io) for _ in range(2))
    q, k, v = (workloads.round_to_io(rng.standard_normal((B, H, kk, d)), io) for _ in range(3))
    w = workloads.conv_weights(rng, H, d, Kc)
    with oracle.feature_map(phi):
        want = oracle.verify_grouped(q, k, v, w, 64, S, z, hist, kwin, vwin, fill, n_commit, alpha=alpha, eps=eps)
    dt = IO[io]
    gs = (dev(S), dev(z), dev(hist, dt), dev(kwin, dt), dev(vwin, dt), torch.from_numpy(np.repeat(fill[:, None], H, axis=1)).cuda())
    nc = None if n_commit is None else torch.from_numpy(n_commit).cuda()
    out = binding.verify_grouped(dev(q, dt), dev(k, dt), dev(v, dt), dev(w), gs, alpha, nc, eps, phi=phi)
    torch.cuda.synchronize()
    check(host(out), want[0], TOL[io], what + " out")
    check(host(gs[0]), want[1], STATE_TOL, what + " S")
    check(host(gs[1]), want[2], STATE_TOL, what + " z")
    assert np.array_equal(host(gs[2]), workloads.round_to_io(want[3], io).astype(np.float64)), what + " hist"
    assert np.array_equal(gs[5].cpu().numpy(), np.repeat(want[6][:, None], H, axis=1)), what + " rows in use"
    for b, n in enumerate(want[6]):
        assert np.array_equal(host(gs[3])[b, :, :n], want[4][b, :, :n]), what + " kwin"
        assert np.array_equal(host(gs[4])[b, :, :n], want[5][b, :, :n]), what + " vwin"
