"""linattn_prefill on the GPU against the CPU oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

import oracle
from parity import TOL, check, check_unfloored, dev, host
from paper_2406_07368_amd import binding, workloads

pytestmark = pytest.mark.gpu

IO = {"f32": torch.float32, "bf16": torch.bfloat16}


def small_case(seed, B, H, L, d, Kc, io, with_state, scale=1.0):
    rng = np.random.default_rng(seed)
    q, k, v = (workloads.round_to_io(rng.standard_normal((B, H, L, d)) * scale, io) for _ in range(3))
    w = workloads.conv_weights(rng, H, d, Kc)
    state = None
    if with_state:
        S0 = (rng.standard_normal((B, H, d, d)) * 3.0).astype(np.float32)
        z0 = (np.abs(rng.standard_normal((B, H, d))) * 5.0 + 1.0).astype(np.float32)
        h0 = workloads.round_to_io(rng.standard_normal((B, H, Kc - 1, d)), io)
        state = (S0, z0, h0)
    return q, k, v, w, state


def run_gpu(q, k, v, w, state, io, chunk=64, eps=0.0):
    dt = IO[io]
    st = None if state is None else (dev(state[0]), dev(state[1]), dev(state[2], dt))
    out, (S, z, h) = binding.prefill(dev(q, dt), dev(k, dt), dev(v, dt), dev(w), st, chunk, eps)
    torch.cuda.synchronize()
    return host(out), host(S), host(z), host(h)


def compare(got, want, io, what=""):
    tol = TOL[io]
    e = check(got[0], want[0], tol, what + " out")
    check(got[1], want[1], tol, what + " S")
    check(got[2], want[2], tol, what + " z")
    assert np.array_equal(got[3], want[3]), what + " hist"
    return e


def test_config1_fp32_against_brute_force_quadratic():
    """B1 H4 L256 d64, all fp32, Kc 3: every output against the definition, to 1e-4."""
    wl = workloads.CONFIGS["cfg1_fp32_tiny"]
    q, k, v, w = workloads.prefill_inputs(wl)
    want = oracle.prefill_quadratic(q, k, v, w)
    got = run_gpu(q, k, v, w, None, "f32", wl.chunk)
    compare(got, want, "f32", "config 1")


@pytest.mark.parametrize("io", ["bf16", "f32"])
@pytest.mark.parametrize("d,chunk", [(64, 64), (128, 64), (128, 128), (64, 128)])
@pytest.mark.parametrize("L,Kc,with_state", [(1, 3, False), (63, 3, True), (64, 1, False), (65, 5, True),
                                             (200, 3, False), (333, 8, True), (512, 2, True)])
def test_prefill_matches_oracle_small(io, d, chunk, L, Kc, with_state):
    """Several tiles and a ragged tail, with and without an incoming state."""
    B, H = 2, 3
    q, k, v, w, state = small_case(1000 + L + d + Kc, B, H, L, d, Kc, io, with_state)
    args = () if state is None else state
    want = oracle.prefill_recurrent(q, k, v, w, *args, eps=1e-3)
    got = run_gpu(q, k, v, w, state, io, chunk, eps=1e-3)
    compare(got, want, io, f"L={L} d={d} C={chunk}")


@pytest.mark.parametrize("d,chunk,L,Kc,with_state", [(128, 64, 2100, 5, True), (64, 128, 4099, 3, False),
                                                     (128, 128, 3000, 8, True), (64, 64, 1024, 2, True)])
def test_few_heads_long_sequence_is_segmented(d, chunk, L, Kc, with_state):
    """B*H far below the number of compute units: the sequence axis is cut into segments whose start
    states come from a first pass and a prefix sum; results must not change."""
    B, H = 1, 2
    desc = binding.make_desc(B, H, d, Kc, chunk, torch.bfloat16, L=L)
    assert binding.linattn_workspace_bytes(desc, L) > 0
    q, k, v, w, state = small_case(2000 + L, B, H, L, d, Kc, "bf16", with_state)
    args = () if state is None else state
    want = oracle.prefill_recurrent(q, k, v, w, *args)
    got = run_gpu(q, k, v, w, state, "bf16", chunk)
    compare(got, want, "bf16", f"segmented L={L}")


def test_state_outputs_may_alias_state_inputs():
    """S_out/z_out/hist_out pointing at S_in/z_in/hist_in, with and without segments."""
    for (B, H, L, d, chunk, Kc) in ((2, 3, 200, 128, 64, 3), (1, 2, 2100, 64, 64, 4), (1, 1, 2, 128, 64, 5)):
        q, k, v, w, state = small_case(77 + L, B, H, L, d, Kc, "bf16", True)
        want = oracle.prefill_recurrent(q, k, v, w, *state)
        dt = torch.bfloat16
        S, z, h = dev(state[0]), dev(state[1]), dev(state[2], dt)
        out = torch.empty((B, H, L, d), dtype=dt, device="cuda")
        desc = binding.make_desc(B, H, d, Kc, chunk, dt, L=L)
        nbytes = binding.linattn_workspace_bytes(desc, L)
        ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
        binding.linattn_prefill(desc, L, dev(q, dt), dev(k, dt), dev(v, dt), dev(w), S, z, h, out, S, z, h, ws, nbytes)
        torch.cuda.synchronize()
        compare((host(out), host(S), host(z), host(h)), want, "bf16", f"aliased L={L}")


def test_config2_full():
    """GPT-2-small shape, B4 H12 L1024 d64 bf16: every head against the recurrent oracle."""
    wl = workloads.CONFIGS["cfg2_gpt2_small"]
    q, k, v, w = workloads.prefill_inputs(wl)
    want = oracle.prefill_recurrent(q, k, v, w)
    got = run_gpu(q, k, v, w, None, "bf16", wl.chunk)
    compare(got, want, "bf16", "config 2")


def _full_size_every_head(name, L=None, token_major=False, heads_per_call=32):
    """The workload at full size on the GPU; the oracle follows every head from the same inputs, a block of heads
    at a time (all host threads; whole workload: seconds)."""
    wl = workloads.CONFIGS[name]
    if L is not None:
        wl = wl.small(L=L)
    q, k, v, w = workloads.prefill_tensors(wl)
    gq, gk, gv = q.cuda(), k.cuda(), v.cuda()
    if token_major:   # [B,L,H,d] in memory, seen as [B,H,L,d]
        gq, gk, gv = (x.transpose(1, 2).contiguous().transpose(1, 2) for x in (gq, gk, gv))
    out, (S, z, h) = binding.prefill(gq, gk, gv, w.cuda(), None, wl.chunk)
    assert out.stride() == gq.stride()
    torch.cuda.synchronize()
    del gq, gk, gv
    out, S, z, h = out.cpu(), S.cpu(), z.cpu(), h.cpu()
    worst, worst_p99 = 0.0, 0.0
    for b in range(wl.B):
        for h0 in range(0, wl.H, heads_per_call):
            sl = (slice(b, b + 1), slice(h0, min(h0 + heads_per_call, wl.H)))
            want = oracle.prefill_recurrent(host(q[sl]), host(k[sl]), host(v[sl]), w[sl[1]].numpy())
            got = (host(out[sl]), host(S[sl]), host(z[sl]), host(h[sl]))
            worst = max(worst, compare(got, want, "bf16", f"{name} batch row {b} heads {h0}.."))
            worst_p99 = max(worst_p99, check_unfloored(got[0], want[0], TOL["bf16"], f"{name} batch row {b} heads {h0}.. out"))
    print(f"{name}{' token-major' if token_major else ''}: {wl.B * wl.H} heads, worst out error {worst:.2e}, "
          f"99th percentile of the un-floored error {worst_p99:.2e}", flush=True)
    return worst


def test_config3_full_size_every_head():
    """LLaMA-2-7B layer shape B8 H32 L4096 d128 bf16 at full size; all 256 heads against the oracle."""
    _full_size_every_head("cfg3_llama7b_prefill")


def test_config3_full_size_token_major_every_head():
    """The same workload with q, k, v, out laid out [B,L,H,d] (what a projection GEMM writes and
    what bench.py times); all 256 heads against the oracle."""
    _full_size_every_head("cfg3_llama7b_prefill", token_major=True)


def test_config5_long_context_every_head():
    """B1 H32 L65536 d128, chunk 128, Kc 5 at full length; all 32 heads against the oracle."""
    _full_size_every_head("cfg5_long_context", heads_per_call=16)


def test_workspace_does_not_grow_with_length():
    wl = workloads.CONFIGS["cfg5_long_context"]
    sizes = []
    for L in (8192, 16384, 32768, 65536):
        desc = binding.make_desc(wl.B, wl.H, wl.d, wl.conv_k, wl.chunk, torch.bfloat16, L=L)
        sizes.append(binding.linattn_workspace_bytes(desc, L))
    assert len(set(sizes)) == 1


@pytest.mark.parametrize("io,d,chunk", [("bf16", 128, 64), ("bf16", 64, 128), ("f32", 64, 64)])
def test_split_invariance_on_gpu(io, d, chunk):
    """prefill(L) == prefill(L1) then prefill(L - L1) from the handed-over state (to rounding)."""
    B, H, L, Kc = 1, 4, 300, 3
    q, k, v, w, _ = small_case(55, B, H, L, d, Kc, io, False)
    full = run_gpu(q, k, v, w, None, io, chunk)
    for L1 in (1, 64, 130):
        a = run_gpu(q[:, :, :L1], k[:, :, :L1], v[:, :, :L1], w, None, io, chunk)
        st = (a[1].astype(np.float32), a[2].astype(np.float32), a[3].astype(np.float32))
        b = run_gpu(q[:, :, L1:], k[:, :, L1:], v[:, :, L1:], w, st, io, chunk)
        tol = 1e-5 if io == "f32" else 1.2e-2
        check(np.concatenate([a[0], b[0]], axis=2), full[0], tol, f"split {L1} out")
        check(b[1], full[1], tol, f"split {L1} S")
        check(b[2], full[2], tol, f"split {L1} z")
        assert np.array_equal(b[3], full[3])


@pytest.mark.parametrize("io,d", [("bf16", 128), ("f32", 64)])
def test_empty_sequence_copies_the_state_through(io, d):
    B, H, Kc = 2, 2, 3
    q, k, v, w, state = small_case(56, B, H, 0, d, Kc, io, True)
    got = run_gpu(q, k, v, w, state, io)
    assert got[0].shape[2] == 0
    for g, s in zip(got[1:], state):
        assert np.array_equal(g, s.astype(np.float64))


@pytest.mark.parametrize("io,d,chunk", [("bf16", 128, 64), ("bf16", 128, 128), ("f32", 64, 64)])
def test_no_leak_from_later_tokens_on_gpu(io, d, chunk):
    """Changing tokens after t (finite values) leaves outputs up to t bit-identical, inside a
    group and across groups."""
    B, H, L, Kc = 1, 2, 200, 3
    q, k, v, w, _ = small_case(57, B, H, L, d, Kc, io, False)
    base = run_gpu(q, k, v, w, None, io, chunk)[0]
    rng = np.random.default_rng(570)
    for t in (0, 17, 63, 64, 130, 198):
        q2, k2, v2 = q.copy(), k.copy(), v.copy()
        for a in (q2, k2, v2):
            a[:, :, t + 1:] = workloads.round_to_io(a[:, :, t + 1:] + 4.0 * rng.standard_normal(a[:, :, t + 1:].shape), io)
        got = run_gpu(q2, k2, v2, w, None, io, chunk)[0]
        assert np.array_equal(got[:, :, :t + 1], base[:, :, :t + 1]), f"leak into tokens <= {t}"
        assert not np.array_equal(got[:, :, t + 1:], base[:, :, t + 1:])


def test_prefill_is_deterministic():
    B, H, L, d, Kc = 2, 8, 700, 128, 3
    q, k, v, w, _ = small_case(58, B, H, L, d, Kc, "bf16", False)
    a = run_gpu(q, k, v, w, None, "bf16")
    b = run_gpu(q, k, v, w, None, "bf16")
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


@pytest.mark.parametrize("io", ["bf16", "f32"])
def test_strided_token_major_layout(io):
    """q, k, v, out stored as [B, L, H, d] (the layout a fused QKV projection leaves behind)."""
    B, H, L, d, Kc = 2, 4, 150, 64, 3
    dt = IO[io]
    q, k, v, w, _ = small_case(59, B, H, L, d, Kc, io, False)
    want = oracle.prefill_recurrent(q, k, v, w)
    tq, tk, tv = (dev(np.ascontiguousarray(a.transpose(0, 2, 1, 3)), dt) for a in (q, k, v))   # [B,L,H,d]
    out = torch.empty_like(tq)
    S = torch.empty((B, H, d, d), device="cuda")
    z = torch.empty((B, H, d), device="cuda")
    h = torch.empty((B, H, Kc - 1, d), device="cuda", dtype=dt)
    desc = binding.make_desc(B, H, d, Kc, 64, dt, strides=(L * H * d, d, H * d))
    nbytes = binding.linattn_workspace_bytes(desc, L)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
    binding.linattn_prefill(desc, L, tq, tk, tv, dev(w), None, None, None, out, S, z, h, ws, nbytes)
    torch.cuda.synchronize()
    got = (host(out).transpose(0, 2, 1, 3), host(S), host(z), host(h))
    compare(got, want, io, "token-major")


def test_prefill_then_verify_equals_longer_prefill():
    """Sec. 5.3 (a shared prefix is computed once): prefill(P) -> verify(k) == last k rows of prefill(P + k)."""
    B, H, d, Kc, P, kk = 2, 4, 128, 3, 190, 8
    q, k, v, w, _ = small_case(60, B, H, P + kk, d, Kc, "bf16", False)
    dt = torch.bfloat16
    _, state = binding.prefill(dev(q[:, :, :P], dt), dev(k[:, :, :P], dt), dev(v[:, :, :P], dt), dev(w))
    out = binding.verify(dev(q[:, :, P:], dt), dev(k[:, :, P:], dt), dev(v[:, :, P:], dt), dev(w), state)
    torch.cuda.synchronize()
    want = oracle.prefill_recurrent(q, k, v, w)
    check(host(out), want[0][:, :, P:], TOL["bf16"], "verify after prefill")
    check(host(state[0]), want[1], TOL["bf16"], "S")
    check(host(state[1]), want[2], TOL["bf16"], "z")
    assert np.array_equal(host(state[2]), want[3])


@pytest.mark.parametrize("grouped", [False, True])
@pytest.mark.parametrize("L", [40, 300])
def test_a_wait_that_gives_up_shows_as_nan(grouped, L):
    """The waves of a bf16 prefill workgroup wait for each other with bounded polling.  With the limit set so that
    every wait gives up at once (from the host; the kernel still runs to its end), nothing that was computed from
    operands that were not waited for may come back as a number: every output row, S and z are NaN, the history
    (a copy of input rows) is exact.  Back at the default limit the same call is correct again."""
    B, H, d, Kc = 2, 4, 128, 3
    q, k, v, w, _ = small_case(61, B, H, L, d, Kc, "bf16", False)
    dt = torch.bfloat16
    args = (dev(q, dt), dev(k, dt), dev(v, dt), dev(w))
    alpha = 0.5 if grouped else None
    prev = binding.linattn_set_wait_limit(-1)
    try:
        assert prev == 1 << 20
        out, (S, z, h) = binding.prefill(*args, grouped_alpha=alpha)
        torch.cuda.synchronize()
    finally:
        assert binding.linattn_set_wait_limit(0) == -1
    assert torch.isnan(out).all() and torch.isnan(S).all() and torch.isnan(z).all()
    assert np.array_equal(host(h), v[:, :, L - (Kc - 1):])
    out, (S, z, h) = binding.prefill(*args, grouped_alpha=alpha)
    torch.cuda.synchronize()
    want = oracle.prefill_grouped(q, k, v, w, 64, alpha=alpha) if grouped else oracle.prefill_recurrent(q, k, v, w)
    compare((host(out), host(S), host(z), host(h)), want, "bf16", "default limit")
