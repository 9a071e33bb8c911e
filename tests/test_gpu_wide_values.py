"""Value rows wider than key rows (Sec. 3, Eq. 1: Q, K of width d_k, V of width d_v = m d_k) on the GPU against
the CPU oracle, through the C ABI: linattn_prefill, linattn_verify, linattn_decode."""
import numpy as np
import pytest
import torch

import oracle
from parity import STATE_TOL, TOL, check, dev, host
from paper_2406_07368_amd import binding, workloads
from test_gpu_prefill import IO

pytestmark = pytest.mark.gpu


def wide_case(seed, B, H, L, d, m, Kc, io, with_state, scale=1.0):
    rng = np.random.default_rng(seed)
    q, k = (workloads.round_to_io(rng.standard_normal((B, H, L, d)) * scale, io) for _ in range(2))
    v = workloads.round_to_io(rng.standard_normal((B, H, L, m * d)) * scale, io)
    w = workloads.conv_weights(rng, H, m * d, Kc)
    state = None
    if with_state:
        S0 = (rng.standard_normal((B, H, d, m * d)) * 3.0).astype(np.float32)
        z0 = (np.abs(rng.standard_normal((B, H, d))) * 5.0 + 1.0).astype(np.float32)
        h0 = workloads.round_to_io(rng.standard_normal((B, H, Kc - 1, m * d)), io)
        state = (S0, z0, h0)
    return q, k, v, w, state


def run_prefill(q, k, v, w, state, io, chunk=64, eps=0.0):
    dt = IO[io]
    st = None if state is None else (dev(state[0]), dev(state[1]), dev(state[2], dt))
    out, (S, z, h) = binding.prefill(dev(q, dt), dev(k, dt), dev(v, dt), dev(w), st, chunk, eps)
    torch.cuda.synchronize()
    return host(out), host(S), host(z), host(h)


def compare(got, want, io, what):
    e = check(got[0], want[0], TOL[io], what + " out")
    check(got[1], want[1], TOL[io], what + " S")
    check(got[2], want[2], TOL[io], what + " z")
    assert np.array_equal(got[3], want[3]), what + " hist"
    return e


@pytest.mark.parametrize("io", ["bf16", "f32"])
@pytest.mark.parametrize("d,m", [(64, 2), (128, 2), (64, 3)])
@pytest.mark.parametrize("L,Kc,with_state", [(1, 3, False), (65, 5, True), (300, 3, True), (333, 8, False)])
def test_prefill_with_wide_values(io, d, m, L, Kc, with_state):
    q, k, v, w, state = wide_case(8000 + L + d + m, 2, 3, L, d, m, Kc, io, with_state)
    args = () if state is None else state
    want = oracle.prefill_recurrent(q, k, v, w, *args, eps=1e-3)
    compare(run_prefill(q, k, v, w, state, io, 64, 1e-3), want, io, f"d_k={d} d_v={m * d} L={L}")


def test_prefill_with_wide_values_segmented_and_long_conv():
    """Few heads, long sequence: segments along the sequence, per value block; and 63 taps on top."""
    for Kc in (5, 63):
        q, k, v, w, state = wide_case(8100 + Kc, 1, 2, 2100, 64, 2, Kc, "bf16", True)
        want = oracle.prefill_recurrent(q, k, v, w, *state)
        compare(run_prefill(q, k, v, w, state, "bf16"), want, "bf16", f"segmented, Kc={Kc}")


@pytest.mark.parametrize("io", ["bf16", "f32"])
def test_prefill_with_wide_values_token_major(io):
    """q, k stored [B,L,H,d_k] and v, out [B,L,H,d_v]: two sets of strides."""
    B, H, L, d, m, Kc = 2, 4, 150, 64, 2, 3
    dt = IO[io]
    q, k, v, w, _ = wide_case(8200, B, H, L, d, m, Kc, io, False)
    want = oracle.prefill_recurrent(q, k, v, w)
    tq, tk, tv = (dev(np.ascontiguousarray(a.transpose(0, 2, 1, 3)), dt).transpose(1, 2) for a in (q, k, v))
    out, (S, z, h) = binding.prefill(tq, tk, tv, dev(w))
    torch.cuda.synchronize()
    assert out.stride() == tv.stride() and out.shape == tv.shape
    compare((host(out), host(S), host(z), host(h)), want, io, "token-major")


def test_prefill_refuses_what_wide_values_cannot_do():
    B, H, L, d, m, Kc = 1, 2, 70, 64, 2, 3
    q, k, v, w, state = wide_case(8300, B, H, L, d, m, Kc, "bf16", True)
    dt = torch.bfloat16
    gq, gk, gv, gw = dev(q, dt), dev(k, dt), dev(v, dt), dev(w)
    S, z, h = dev(state[0]), dev(state[1]), dev(state[2], dt)
    out = torch.empty_like(gv)
    desc = binding.make_desc(B, H, d, Kc, 64, dt, L=L, d_v=m * d)
    with pytest.raises(binding.LinattnError) as ei:       # z_out == z_in: every value block reads z_in, one writes z_out
        binding.linattn_prefill(desc, L, gq, gk, gv, gw, S, z, h, out, S, z, h)
    assert ei.value.status == 5
    with pytest.raises(binding.LinattnError) as ei:       # the three-branch form takes d_v = d only
        binding.linattn_prefill_grouped(desc, L, 1.0, gq, gk, gv, gw, None, None, None, out, None, None, None)
    assert ei.value.status == 5
    bad = binding.make_desc(B, H, d, Kc, 64, dt, L=L, d_v=96)
    with pytest.raises(binding.LinattnError) as ei:
        binding.linattn_prefill(bad, L, gq, gk, gv, gw, None, None, None, out, None, None, None)
    assert ei.value.status == 2


@pytest.mark.parametrize("io", ["bf16", "f32"])
@pytest.mark.parametrize("B,H", [(2, 3), (24, 32)])
@pytest.mark.parametrize("d,m,kk,Kc", [(64, 2, 1, 3), (64, 2, 5, 5), (128, 2, 8, 3), (64, 3, 16, 8)])
def test_verify_and_decode_with_wide_values(io, B, H, d, m, kk, Kc):
    dt = IO[io]
    rng = np.random.default_rng(8400 + kk + d + m + B)
    _, _, _, w, state = wide_case(8401 + kk + B, B, H, 1, d, m, Kc, io, True)
    S, z, hist = state
    q, k = (workloads.round_to_io(rng.standard_normal((B, H, kk, d)), io) for _ in range(2))
    v = workloads.round_to_io(rng.standard_normal((B, H, kk, m * d)), io)
    n_commit = (np.arange(B) % (kk + 1)).astype(np.int32)
    want = oracle.verify(q, k, v, w, S, z, hist, n_commit, eps=1e-3)
    st = (dev(S), dev(z), dev(hist, dt))
    out = binding.verify(dev(q, dt), dev(k, dt), dev(v, dt), dev(w), st, torch.from_numpy(n_commit).cuda(), 1e-3)
    torch.cuda.synchronize()
    check(host(out), want[0], TOL[io], "verify out")
    check(host(st[0]), want[1], STATE_TOL, "verify S")
    check(host(st[1]), want[2], STATE_TOL, "verify z")
    assert np.array_equal(host(st[2]), workloads.round_to_io(want[3], io).astype(np.float64)), "verify hist"
    want1 = oracle.decode(q[:, :, :1], k[:, :, :1], v[:, :, :1], w, S, z, hist, eps=1e-3)
    st1 = (dev(S), dev(z), dev(hist, dt))
    out1 = binding.decode(dev(q[:, :, 0], dt), dev(k[:, :, 0], dt), dev(v[:, :, 0], dt), dev(w), st1, 1e-3)
    torch.cuda.synchronize()
    check(host(out1)[:, :, None], want1[0], TOL[io], "decode out")
    check(host(st1[0]), want1[1], STATE_TOL, "decode S")
    check(host(st1[1]), want1[2], STATE_TOL, "decode z")


def test_wide_values_workloads_every_head():
    """B8 H32 L4096 d_k 64 d_v 128 bf16 at full size (the launch the bench times), then the verify workload:
    B32 H32, state from a 2048-token prefix, 8 drafts; every head against the oracle."""
    wl = workloads.CONFIGS["wide_values_prefill"]
    q, k, v, w = workloads.prefill_tensors(wl)
    out, (S, z, h) = binding.prefill(q.cuda(), k.cuda(), v.cuda(), w.cuda(), None, wl.chunk)
    torch.cuda.synchronize()
    out, S, z, h = out.cpu(), S.cpu(), z.cpu(), h.cpu()
    worst = 0.0
    for b in range(wl.B):
        sl = slice(b, b + 1)
        want = oracle.prefill_recurrent(host(q[sl]), host(k[sl]), host(v[sl]), w.numpy())
        worst = max(worst, compare((host(out[sl]), host(S[sl]), host(z[sl]), host(h[sl])), want, "bf16", f"prefill batch row {b}"))
    vw = workloads.CONFIGS["wide_values_verify"]
    pq, pk, pv, w = workloads.prefill_tensors(vw)
    _, state = binding.prefill(pq.cuda(), pk.cuda(), pv.cuda(), w.cuda(), None, vw.chunk)
    kk = 8
    dq, dk, dv = (torch.from_numpy(a).to(torch.bfloat16) for a in workloads.draft_block(vw, kk))
    n_commit = (np.arange(vw.B) % (kk + 1)).astype(np.int32)
    vout = binding.verify(dq.cuda(), dk.cuda(), dv.cuda(), w.cuda(), state, torch.from_numpy(n_commit).cuda())
    torch.cuda.synchronize()
    worst_v = 0.0
    for b in range(vw.B):
        sl = slice(b, b + 1)
        _, S1, z1, h1 = oracle.prefill_recurrent(host(pq[sl]), host(pk[sl]), host(pv[sl]), w.numpy())
        want = oracle.verify(host(dq[sl]), host(dk[sl]), host(dv[sl]), w.numpy(), S1, z1, h1, n_commit[sl])
        worst_v = max(worst_v, check(host(vout[sl]), want[0], TOL["bf16"], f"verify out, batch row {b}"))
        check(host(state[0][sl]), want[1], TOL["bf16"], f"verify S, batch row {b}")      # the prefix state is the bf16 prefill's
        check(host(state[1][sl]), want[2], TOL["bf16"], f"verify z, batch row {b}")
        assert np.array_equal(host(state[2][sl]), want[3])
    print(f"wide values: prefill {wl.B * wl.H} heads, worst out error {worst:.2e}; verify {vw.B * vw.H} heads, {worst_v:.2e}", flush=True)
