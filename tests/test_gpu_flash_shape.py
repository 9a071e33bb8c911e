"""The sizes of the paper's FLASH experiment on the GPU against the CPU oracle, through the C ABI: a masked
depthwise convolution of up to 63 taps (Sec. 4.1) in both prefill forms, and the three-branch form in groups of
256 tokens (Sec. 5 "Settings")."""
import numpy as np
import pytest
import torch

import oracle
from parity import TOL, check, check_unfloored, dev, host
from paper_2406_07368_amd import binding, workloads
from test_gpu_prefill import IO, small_case

pytestmark = pytest.mark.gpu


def run(q, k, v, w, state, io, chunk=64, eps=0.0, alpha=None, alias_hist=False):
    dt = IO[io]
    st = None if state is None else (dev(state[0]), dev(state[1]), dev(state[2], dt))
    if alias_hist:
        # the caller's history buffer is updated in place: hist_out is hist_in
        B, H, L, d = q.shape
        Kc = w.shape[2]
        gq, gk, gv = dev(q, dt), dev(k, dt), dev(v, dt)
        desc = binding.make_desc(B, H, d, Kc, chunk, dt, eps, L=L)
        out = torch.empty_like(gq)
        nb = binding.linattn_workspace_bytes(desc, L)
        ws = torch.empty(max(nb, 16), dtype=torch.uint8, device="cuda")
        binding.linattn_prefill(desc, L, gq, gk, gv, dev(w), st[0], st[1], st[2], out, st[0], st[1], st[2], ws, nb)
        S, z, h = st
    else:
        out, (S, z, h) = binding.prefill(dev(q, dt), dev(k, dt), dev(v, dt), dev(w), st, chunk, eps, grouped_alpha=alpha)
    torch.cuda.synchronize()
    return host(out), host(S), host(z), host(h)


def compare(got, want, io, what):
    e = check(got[0], want[0], TOL[io], what + " out")
    check(got[1], want[1], TOL[io], what + " S")
    check(got[2], want[2], TOL[io], what + " z")
    assert np.array_equal(got[3], want[3]), what + " hist"
    return e


@pytest.mark.parametrize("io", ["bf16", "f32"])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("L,Kc,with_state", [(1, 63, True), (40, 9, False), (62, 63, True), (63, 63, False), (64, 33, True),
                                             (130, 63, True), (300, 63, False), (300, 17, True)])
def test_long_conv_kernels_in_the_token_level_prefill(io, d, L, Kc, with_state):
    """More taps than the attention kernels gather themselves: sequences shorter and longer than the window, with
    and without a history of Kc - 1 rows."""
    q, k, v, w, state = small_case(7000 + L + d + Kc, 2, 3, L, d, Kc, io, with_state)
    args = () if state is None else state
    want = oracle.prefill_recurrent(q, k, v, w, *args, eps=1e-3)
    compare(run(q, k, v, w, state, io, 256, 1e-3), want, io, f"L={L} Kc={Kc}")


@pytest.mark.parametrize("L", [20, 200])
def test_long_conv_history_updated_in_place(L):
    """hist_out may be hist_in, also when the new history is part old rows, part new ones (L < Kc - 1)."""
    io, d, Kc = "bf16", 128, 63
    q, k, v, w, state = small_case(7100 + L, 2, 2, L, d, Kc, io, True)
    want = oracle.prefill_recurrent(q, k, v, w, *state)
    compare(run(q, k, v, w, state, io, alias_hist=True), want, io, f"in place, L={L}")


def test_long_conv_on_a_segmented_sequence_and_in_token_major_layout():
    """Few heads, long sequence (the attention kernel cuts the sequence into segments) with 63 taps; and the same
    call on [B,L,H,d] tensors."""
    B, H, L, d, Kc = 1, 2, 2100, 128, 63
    q, k, v, w, state = small_case(7200, B, H, L, d, Kc, "bf16", True)
    want = oracle.prefill_recurrent(q, k, v, w, *state)
    compare(run(q, k, v, w, state, "bf16", 256), want, "bf16", "segmented")
    dt = torch.bfloat16
    tq, tk, tv = (dev(np.ascontiguousarray(a.transpose(0, 2, 1, 3)), dt).transpose(1, 2) for a in (q, k, v))
    st = (dev(state[0]), dev(state[1]), dev(state[2], dt))
    out, (S, z, h) = binding.prefill(tq, tk, tv, dev(w), st, 256)
    torch.cuda.synchronize()
    assert out.stride() == tq.stride()
    compare((host(out), host(S), host(z), host(h)), want, "bf16", "token-major")


def test_long_conv_leaks_nothing_from_later_tokens():
    io, d, Kc, L = "bf16", 128, 63, 200
    q, k, v, w, _ = small_case(7300, 1, 2, L, d, Kc, io, False)
    base = run(q, k, v, w, None, io)[0]
    rng = np.random.default_rng(7301)
    for t in (0, 61, 62, 63, 130):
        q2, k2, v2 = q.copy(), k.copy(), v.copy()
        for a in (q2, k2, v2):
            a[:, :, t + 1:] = workloads.round_to_io(a[:, :, t + 1:] + 4.0 * rng.standard_normal(a[:, :, t + 1:].shape), io)
        got = run(q2, k2, v2, w, None, io)[0]
        assert np.array_equal(got[:, :, :t + 1], base[:, :, :t + 1]), f"leak into tokens <= {t}"


@pytest.mark.parametrize("io,d", [("bf16", 128), ("bf16", 64), ("f32", 64)])
@pytest.mark.parametrize("L,Kc,with_state", [(1, 3, False), (255, 63, True), (256, 5, False), (257, 63, True), (600, 63, False)])
def test_three_branch_form_in_groups_of_256(io, d, L, Kc, with_state):
    q, k, v, w, state = small_case(7400 + L + d + Kc, 2, 2, L, d, Kc, io, with_state)
    args = {} if state is None else dict(S0=state[0], z0=state[1], hist0=state[2])
    want = oracle.prefill_grouped(q, k, v, w, 256, alpha=0.7, eps=1e-3, **args)
    compare(run(q, k, v, w, state, io, 256, 1e-3, alpha=0.7), want, io, f"groups of 256, L={L} Kc={Kc}")


@pytest.mark.parametrize("B,H,L,d,Kc,with_state", [(10, 10, 1100, 128, 5, True),     # 100 heads: two segments of 3 and 2 groups
                                                    (8, 32, 600, 128, 3, True),      # 256 heads: no segments, 3 groups each
                                                    (8, 32, 300, 64, 8, False),
                                                    (1, 3, 2100, 64, 2, True)])      # 9 segments of one group
def test_three_branch_form_in_groups_of_256_launch_plans(B, H, L, d, Kc, with_state):
    """bf16 rows on the matrix cores: every way the sequence can be laid out on the chip (segments of several groups,
    of one group, none at all), with the state handed back after the last token."""
    q, k, v, w, state = small_case(7450 + B + L, B, H, L, d, Kc, "bf16", with_state)
    args = {} if state is None else dict(S0=state[0], z0=state[1], hist0=state[2])
    want = oracle.prefill_grouped(q, k, v, w, 256, alpha=1.0, eps=1e-3, **args)
    compare(run(q, k, v, w, state, "bf16", 256, 1e-3, alpha=1.0), want, "bf16", f"B{B} H{H} L{L} d{d}")


def test_three_branch_form_in_groups_of_256_details():
    """Nothing before the first group and eps = 0 (the linear branch is absent there, no division by zero reaches
    the output); the other feature map; token-major tensors; peaked softmax weights; no leak from later tokens."""
    io, dt, d = "bf16", torch.bfloat16, 128
    q, k, v, w, _ = small_case(7460, 1, 4, 700, d, 3, io, False)
    want = oracle.prefill_grouped(q, k, v, w, 256, alpha=1.0, eps=0.0)
    base = run(q, k, v, w, None, io, 256, 0.0, alpha=1.0)
    compare(base, want, io, "eps = 0")
    with oracle.feature_map("relu"):
        want = oracle.prefill_grouped(q, k, v, w, 256, alpha=0.5, eps=0.05)
    out, (S, z, h) = binding.prefill(dev(q, dt), dev(k, dt), dev(v, dt), dev(w), None, 256, 0.05, phi="relu", grouped_alpha=0.5)
    torch.cuda.synchronize()
    compare((host(out), host(S), host(z), host(h)), want, io, "relu")
    tq, tk, tv = (dev(np.ascontiguousarray(a.transpose(0, 2, 1, 3)), dt).transpose(1, 2) for a in (q, k, v))
    out, (S, z, h) = binding.prefill(tq, tk, tv, dev(w), None, 256, 0.0, grouped_alpha=1.0)
    torch.cuda.synchronize()
    assert np.array_equal(host(out), base[0]), "token-major layout"
    q3, k3, v3, w3, _ = small_case(7461, 2, 2, 500, d, 3, io, False, scale=2.5)        # logits in the tens
    want = oracle.prefill_grouped(q3, k3, v3, w3, 256, alpha=0.0)
    compare(run(q3, k3, v3, w3, None, io, 256, alpha=0.0), want, io, "peaked weights")
    rng = np.random.default_rng(7462)
    for t in (0, 100, 255, 256, 600):
        q2, k2, v2 = q.copy(), k.copy(), v.copy()
        for a in (q2, k2, v2):
            a[:, :, t + 1:] = workloads.round_to_io(a[:, :, t + 1:] + 4.0 * rng.standard_normal(a[:, :, t + 1:].shape), io)
        got = run(q2, k2, v2, w, None, io, 256, 0.0, alpha=1.0)[0]
        assert np.array_equal(got[:, :, :t + 1], base[0][:, :, :t + 1]), f"leak into tokens <= {t}"


@pytest.mark.parametrize("d", [64, 128])
def test_three_branch_form_in_groups_of_64_with_63_taps(d):
    """The matrix-core kernel of the three-branch form followed by the long convolution."""
    q, k, v, w, state = small_case(7500 + d, 2, 3, 333, d, 63, "bf16", True)
    want = oracle.prefill_grouped(q, k, v, w, 64, alpha=1.0, eps=1e-3, S0=state[0], z0=state[1], hist0=state[2])
    compare(run(q, k, v, w, state, "bf16", 64, 1e-3, alpha=1.0), want, "bf16", f"groups of 64, 63 taps, d={d}")


def test_fp32_rows_of_128_in_groups_of_256_are_refused():
    q, k, v, w, _ = small_case(7600, 1, 1, 10, 128, 3, "f32", False)
    with pytest.raises(binding.LinattnError) as ei:
        run(q, k, v, w, None, "f32", 256, alpha=1.0)
    assert ei.value.status == 5


@pytest.mark.parametrize("name", ["flash_L1024", "flash_L4096", "flash_L8192"])
def test_flash_shaped_workload_every_head(name):
    """B1 H8 d128 bf16, groups of 256, 63 taps, at full length: the token-level form (which does not depend on
    the group size) and the three-branch form in groups of 256, all heads against the oracle."""
    wl = workloads.CONFIGS[name]
    q, k, v, w = workloads.prefill_tensors(wl)
    gq, gk, gv, gw = q.cuda(), k.cuda(), v.cuda(), w.cuda()
    out, (S, z, h) = binding.prefill(gq, gk, gv, gw, None, wl.chunk)
    gout, (gS, gz, gh) = binding.prefill_grouped(gq, gk, gv, gw, 1.0, group=wl.chunk)
    torch.cuda.synchronize()
    hq, hk, hv = host(q), host(k), host(v)
    want = oracle.prefill_recurrent(hq, hk, hv, w.numpy())
    e1 = compare((host(out), host(S), host(z), host(h)), want, "bf16", name)
    p1 = check_unfloored(host(out), want[0], TOL["bf16"], name + " out")
    gwant = oracle.prefill_grouped(hq, hk, hv, w.numpy(), wl.chunk, alpha=1.0)
    e2 = compare((host(gout), host(gS), host(gz), host(gh)), gwant, "bf16", name + " three-branch form")
    print(f"{name}: token-level form {e1:.2e} (un-floored 99th percentile {p1:.2e}), three-branch form in groups of "
          f"{wl.chunk}: {e2:.2e}", flush=True)
