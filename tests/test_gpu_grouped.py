"""linattn_prefill_grouped (the three-branch form of Sec. 4.1) on the GPU against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from parity import TOL, check, check_unfloored, dev, host
from paper_2406_07368_amd import binding, workloads
from test_gpu_prefill import small_case

pytestmark = pytest.mark.gpu

BF = torch.bfloat16


def run_gpu(q, k, v, w, state, alpha, eps=0.0, phi="elu1", dt=BF):
    st = None if state is None else (dev(state[0]), dev(state[1]), dev(state[2], dt))
    out, (S, z, h) = binding.prefill_grouped(dev(q, dt), dev(k, dt), dev(v, dt), dev(w), alpha, st, eps, phi=phi)
    torch.cuda.synchronize()
    return host(out), host(S), host(z), host(h)


def compare(got, want, what="", io="bf16"):
    tol = TOL[io]
    e = check(got[0], want[0], tol, what + " out")
    check(got[1], want[1], tol, what + " S")
    check(got[2], want[2], tol, what + " z")
    assert np.array_equal(got[3], want[3]), what + " hist"
    return e


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("alpha", [1.0, 0.35])
@pytest.mark.parametrize("L,Kc,with_state", [(1, 3, False), (63, 3, True), (64, 1, False), (65, 5, True), (129, 2, False),
                                             (200, 3, False), (333, 8, True), (512, 2, True)])
def test_grouped_matches_oracle_small(d, alpha, L, Kc, with_state):
    """Several groups and a ragged tail, with and without an incoming state."""
    B, H = 2, 3
    q, k, v, w, state = small_case(5000 + L + d + Kc, B, H, L, d, Kc, "bf16", with_state)
    args = {} if state is None else dict(S0=state[0], z0=state[1], hist0=state[2])
    want = oracle.prefill_grouped(q, k, v, w, 64, alpha=alpha, eps=1e-3, **args)
    got = run_gpu(q, k, v, w, state, alpha, eps=1e-3)
    compare(got, want, f"L={L} d={d} alpha={alpha}")


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("L,Kc,with_state,phi", [(1, 3, False, "elu1"), (64, 1, True, "elu1"), (65, 5, True, "relu"), (200, 8, False, "elu1"),
                                                 (130, 3, True, "elu1")])
def test_grouped_fp32_rows_match_the_oracle_to_1e4(d, L, Kc, with_state, phi):
    """fp32 rows take a plain fp32 kernel: the three-branch form against the oracle at the fp32 bar."""
    B, H = 2, 2
    q, k, v, w, state = small_case(5050 + L + d + Kc, B, H, L, d, Kc, "f32", with_state)
    args = {} if state is None else dict(S0=state[0], z0=state[1], hist0=state[2])
    with oracle.feature_map(phi):
        want = oracle.prefill_grouped(q, k, v, w, 64, alpha=0.7, eps=1e-2, **args)
    got = run_gpu(q, k, v, w, state, 0.7, eps=1e-2, phi=phi, dt=torch.float32)
    compare(got, want, f"fp32 L={L} d={d}", io="f32")


@pytest.mark.parametrize("d", [64, 128])
def test_first_group_without_state_and_eps(d):
    """Nothing precedes the first group and eps = 0: the linear branch's denominator is exactly zero there and
    the branch is absent (no division by zero reaches the output)."""
    q, k, v, w, _ = small_case(5100 + d, 1, 4, 150, d, 3, "bf16", False)
    want = oracle.prefill_grouped(q, k, v, w, 64, alpha=1.0, eps=0.0)
    got = run_gpu(q, k, v, w, None, 1.0, eps=0.0)
    compare(got, want, f"d={d}")


@pytest.mark.parametrize("d,scale", [(64, 3.0), (128, 2.5)])
def test_local_branch_alone_with_peaked_weights(d, scale):
    """alpha = 0 leaves local attention + conv; large logits (|q.k|/sqrt(d) in the tens) make the weights
    nearly one-hot, which the subtraction of a query's largest logit has to survive."""
    q, k, v, w, _ = small_case(5200 + d, 2, 2, 300, d, 3, "bf16", False, scale=scale)
    want = oracle.prefill_grouped(q, k, v, w, 64, alpha=0.0)
    got = run_gpu(q, k, v, w, None, 0.0)
    compare(got, want, f"d={d} scale={scale}")


@pytest.mark.parametrize("d,L,Kc,with_state", [(128, 2100, 5, True), (64, 4099, 3, False)])
def test_few_heads_long_sequence_is_segmented(d, L, Kc, with_state):
    """B*H far below the number of compute units: segments along the sequence (which start on group
    boundaries) must give the same result."""
    B, H = 1, 2
    desc = binding.make_desc(B, H, d, Kc, 64, BF, L=L)
    assert binding.linattn_workspace_bytes(desc, L) > 0
    q, k, v, w, state = small_case(5300 + L, B, H, L, d, Kc, "bf16", with_state)
    args = {} if state is None else dict(S0=state[0], z0=state[1], hist0=state[2])
    want = oracle.prefill_grouped(q, k, v, w, 64, alpha=0.8, eps=1e-3, **args)
    got = run_gpu(q, k, v, w, state, 0.8, eps=1e-3)
    compare(got, want, f"segmented L={L}")


def test_token_major_views_and_second_feature_map():
    """[B,L,H,d] tensors passed as transposed views; phi = max(x, 0) on the linear branch."""
    B, H, L, d, Kc = 2, 4, 260, 128, 3
    q, k, v, w, _ = small_case(5400, B, H, L, d, Kc, "bf16", False)
    gq, gk, gv = (dev(np.ascontiguousarray(a.transpose(0, 2, 1, 3)), BF).transpose(1, 2) for a in (q, k, v))
    for phi in ("elu1", "relu"):
        with oracle.feature_map(phi):
            want = oracle.prefill_grouped(q, k, v, w, 64, alpha=1.0, eps=1e-2)
        out, (S, z, h) = binding.prefill_grouped(gq, gk, gv, dev(w), 1.0, None, 1e-2, phi=phi)
        torch.cuda.synchronize()
        assert out.stride() == gq.stride()
        compare((host(out), host(S), host(z), host(h)), want, phi)


def test_continuation_at_a_group_boundary():
    """Two calls cut at a multiple of 64 equal one call (the state carries everything)."""
    B, H, L, d, Kc = 1, 3, 300, 64, 4
    q, k, v, w, _ = small_case(5500, B, H, L, d, Kc, "bf16", False)
    gq, gk, gv, gw = dev(q, BF), dev(k, BF), dev(v, BF), dev(w)
    whole, st_whole = binding.prefill_grouped(gq, gk, gv, gw, 1.0, None, 1e-3)
    cut = 128
    a, st_a = binding.prefill_grouped(gq[:, :, :cut].contiguous(), gk[:, :, :cut].contiguous(), gv[:, :, :cut].contiguous(), gw, 1.0, None, 1e-3)
    b, st_b = binding.prefill_grouped(gq[:, :, cut:].contiguous(), gk[:, :, cut:].contiguous(), gv[:, :, cut:].contiguous(), gw, 1.0, st_a, 1e-3)
    torch.cuda.synchronize()
    assert torch.equal(torch.cat([a, b], dim=2), whole)
    for x, y in zip(st_b, st_whole):
        assert torch.equal(x, y)


def test_full_size_llama_shape_every_head():
    """B8 H32 L4096 d128 token-major, the launch the bench times: all 256 heads against the oracle."""
    wl = workloads.CONFIGS["cfg3_llama7b_prefill"]
    q, k, v, w = workloads.prefill_tensors(wl)
    tm = [t.transpose(1, 2).contiguous().cuda().transpose(1, 2) for t in (q, k, v)]
    out, (S, z, h) = binding.prefill_grouped(tm[0], tm[1], tm[2], w.cuda(), 1.0)
    torch.cuda.synchronize()
    del tm
    out, S, z, h = out.cpu(), S.cpu(), z.cpu(), h.cpu()
    worst, worst_p99 = 0.0, 0.0
    for b in range(wl.B):
        sl = (slice(b, b + 1), slice(None))
        want = oracle.prefill_grouped(host(q[sl]), host(k[sl]), host(v[sl]), w.numpy(), 64, alpha=1.0)
        got = (host(out[sl]), host(S[sl]), host(z[sl]), host(h[sl]))
        worst = max(worst, compare(got, want, f"batch row {b}"))
        worst_p99 = max(worst_p99, check_unfloored(got[0], want[0], TOL["bf16"], f"batch row {b} out"))
    print(f"three-branch cfg3: {wl.B * wl.H} heads, worst out error {worst:.2e}, 99th percentile of the un-floored "
          f"error {worst_p99:.2e}", flush=True)
