"""linattn_verify / linattn_decode on the GPU against the CPU oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

import oracle
from parity import STATE_TOL, TOL, check, dev, host
from paper_2406_07368_amd import binding, workloads

pytestmark = pytest.mark.gpu

IO = {"f32": torch.float32, "bf16": torch.bfloat16}


def make_case(seed, B, H, d, Kc, kk, io, prefix=40, scale=1.0):
    """Drafts plus a state that a short seeded prefix leaves behind (oracle, then rounded to fp32)."""
    rng = np.random.default_rng(seed)
    shp = (B, H, prefix, d)
    pq, pk, pv = (workloads.round_to_io(rng.standard_normal(shp) * scale, io) for _ in range(3))
    w = workloads.conv_weights(rng, H, d, Kc)
    _, S, z, hist = oracle.prefill_recurrent(pq, pk, pv, w)
    S, z = S.astype(np.float32), z.astype(np.float32)          # the state the GPU is handed is fp32
    hist = workloads.round_to_io(hist, io)
    q, k, v = (workloads.round_to_io(rng.standard_normal((B, H, kk, d)) * scale, io) for _ in range(3))
    return q, k, v, w, S, z, hist


def run_gpu(q, k, v, w, S, z, hist, io, n_commit=None, eps=0.0):
    dt = IO[io]
    state = (dev(S), dev(z), dev(hist, dt))
    nc = None if n_commit is None else torch.from_numpy(np.asarray(n_commit, dtype=np.int32)).cuda()
    out = binding.verify(dev(q, dt), dev(k, dt), dev(v, dt), dev(w), state, nc, eps)
    torch.cuda.synchronize()
    return host(out), host(state[0]), host(state[1]), host(state[2])


@pytest.mark.parametrize("io", ["bf16", "f32"])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("kk,Kc", [(1, 3), (2, 1), (4, 3), (5, 5), (8, 3), (13, 8), (16, 2)])
def test_verify_matches_oracle_small(io, d, kk, Kc):
    B, H = 2, 3
    q, k, v, w, S, z, hist = make_case(100 + kk + d, B, H, d, Kc, kk, io)
    n_commit = np.array([kk, kk // 2], dtype=np.int32)
    want = oracle.verify(q, k, v, w, S, z, hist, n_commit, eps=1e-3)
    got = run_gpu(q, k, v, w, S, z, hist, io, n_commit, eps=1e-3)
    tol = TOL[io]
    check(got[0], want[0], tol, "out")
    check(got[1], want[1], 1e-5, "S")          # the state is fp32 on both sides of the call
    check(got[2], want[2], 1e-5, "z")
    assert np.array_equal(got[3], workloads.round_to_io(want[3], io).astype(np.float64)), "hist"


@pytest.mark.parametrize("BH,expect_split", [((24, 32), 1), ((16, 32), 2), ((2, 32), 4)])
def test_verify_every_column_split(BH, expect_split):
    """B*H decides over how many workgroups a head's columns are spread; all variants must agree with the oracle."""
    B, H = BH
    d, Kc, kk, io = 64, 3, 4, "bf16"
    q, k, v, w, S, z, hist = make_case(7, B, H, d, Kc, kk, io, prefix=8)
    n_commit = (np.arange(B) % (kk + 1)).astype(np.int32)
    want = oracle.verify(q, k, v, w, S, z, hist, n_commit)
    got = run_gpu(q, k, v, w, S, z, hist, io, n_commit)
    check(got[0], want[0], TOL[io], "out")
    # whole heads of bf16 drafts take the matrix-core kernel (phi(k) as two bf16 terms), the others the
    # column-split kernel (fp32 products): the same state either way
    check(got[1], want[1], STATE_TOL, "S")
    check(got[2], want[2], STATE_TOL, "z")
    assert np.array_equal(got[3], workloads.round_to_io(want[3], io).astype(np.float64))


# ---- the matrix-core kernel: bf16 drafts, B*H >= 768 (whole heads per workgroup) -------------------
MB, MH = 24, 32


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("kk,Kc", [(1, 3), (2, 1), (4, 3), (5, 5), (8, 3), (13, 8), (16, 2)])
def test_verify_whole_heads_on_the_matrix_cores(d, kk, Kc):
    io = "bf16"
    q, k, v, w, S, z, hist = make_case(300 + kk + d, MB, MH, d, Kc, kk, io, prefix=12)
    n_commit = (np.arange(MB) * 5 % (kk + 1)).astype(np.int32)
    want = oracle.verify(q, k, v, w, S, z, hist, n_commit, eps=1e-3)
    got = run_gpu(q, k, v, w, S, z, hist, io, n_commit, eps=1e-3)
    check(got[0], want[0], TOL[io], "out")
    check(got[1], want[1], STATE_TOL, "S")
    check(got[2], want[2], STATE_TOL, "z")
    assert np.array_equal(got[3], workloads.round_to_io(want[3], io).astype(np.float64)), "hist"
    for b in np.nonzero(n_commit == 0)[0]:       # nothing accepted: the state comes back bit-unchanged
        assert np.array_equal(got[1][b], S[b].astype(np.float64))
        assert np.array_equal(got[2][b], z[b].astype(np.float64))
        assert np.array_equal(got[3][b], hist[b].astype(np.float64))


def test_matrix_core_verify_equals_sequential_decode_and_leaks_nothing():
    """Sec. 4.2 on the matrix-core kernel: one call over kk drafts == kk decode calls, and changing
    later drafts leaves the outputs of earlier ones bit-identical."""
    io, d, Kc, kk = "bf16", 128, 3, 6
    dt = IO[io]
    q, k, v, w, S, z, hist = make_case(17, MB, MH, d, Kc, kk, io, prefix=12)
    got = run_gpu(q, k, v, w, S, z, hist, io)
    state = (dev(S), dev(z), dev(hist, dt))
    outs = []
    for j in range(kk):
        outs.append(host(binding.decode(dev(q[:, :, j], dt), dev(k[:, :, j], dt), dev(v[:, :, j], dt), dev(w), state)))
    torch.cuda.synchronize()
    seq = np.stack(outs, axis=2)
    # the same terms, grouped differently (bf16-rounded S for the read-out in both): output rounding apart
    check(seq, got[0], 1.2e-2, "decode chain out")
    check(host(state[0]), got[1], 1e-5, "decode chain S")
    check(host(state[1]), got[2], 1e-5, "decode chain z")
    assert np.array_equal(host(state[2]), got[3])
    for j in (0, 3):
        q2, k2, v2 = q.copy(), k.copy(), v.copy()
        for a in (q2, k2, v2):
            a[:, :, j + 1:] = workloads.round_to_io(-2.0 * a[:, :, j + 1:] + 1.0, io)
        other = run_gpu(q2, k2, v2, w, S, z, hist, io)[0]
        assert np.array_equal(other[:, :, :j + 1], got[0][:, :, :j + 1]), f"draft {j} saw a later draft"


def test_fp32_drafts_on_whole_heads_keep_the_exact_update():
    """fp32 drafts never take the matrix-core kernel: B*H >= 768 runs the streaming kernel unsplit (fp32 products)."""
    B, H, d, Kc, kk, io = MB, MH, 64, 3, 5, "f32"
    q, k, v, w, S, z, hist = make_case(19, B, H, d, Kc, kk, io, prefix=8)
    n_commit = (np.arange(B) % (kk + 1)).astype(np.int32)
    want = oracle.verify(q, k, v, w, S, z, hist, n_commit)
    got = run_gpu(q, k, v, w, S, z, hist, io, n_commit)
    check(got[0], want[0], TOL[io], "out")
    check(got[1], want[1], 1e-5, "S")
    check(got[2], want[2], 1e-5, "z")
    assert np.array_equal(got[3], want[3])


def test_rejected_drafts_leave_no_trace():
    """n_commit = 0 hands the state back bit-unchanged; outputs are still produced."""
    B, H, d, Kc, kk, io = 3, 4, 128, 3, 8, "bf16"
    q, k, v, w, S, z, hist = make_case(11, B, H, d, Kc, kk, io)
    n_commit = np.array([0, 3, 0], dtype=np.int32)
    got = run_gpu(q, k, v, w, S, z, hist, io, n_commit)
    for b in (0, 2):
        assert np.array_equal(got[1][b], S[b].astype(np.float64))
        assert np.array_equal(got[2][b], z[b].astype(np.float64))
        assert np.array_equal(got[3][b], hist[b].astype(np.float64))
    want = oracle.verify(q, k, v, w, S, z, hist, n_commit)
    check(got[0], want[0], TOL[io], "out")
    check(got[1], want[1], 1e-5, "S")


def test_out_of_range_commit_counts_are_clamped():
    B, H, d, Kc, kk, io = 2, 2, 64, 3, 4, "f32"
    q, k, v, w, S, z, hist = make_case(12, B, H, d, Kc, kk, io)
    got = run_gpu(q, k, v, w, S, z, hist, io, np.array([-3, 99], dtype=np.int32))
    want = oracle.verify(q, k, v, w, S, z, hist, np.array([0, kk], dtype=np.int32))
    check(got[1], want[1], 1e-5, "S")
    check(got[2], want[2], 1e-5, "z")


@pytest.mark.parametrize("io", ["bf16", "f32"])
def test_verify_equals_sequential_decode_on_gpu(io):
    """Sec. 4.2: one call over kk drafts == kk decode calls (outputs and final state), on the GPU itself."""
    B, H, d, Kc, kk = 2, 5, 128, 3, 6
    dt = IO[io]
    q, k, v, w, S, z, hist = make_case(13, B, H, d, Kc, kk, io)
    got = run_gpu(q, k, v, w, S, z, hist, io)
    state = (dev(S), dev(z), dev(hist, dt))
    outs = []
    for j in range(kk):
        o = binding.decode(dev(q[:, :, j], dt), dev(k[:, :, j], dt), dev(v[:, :, j], dt), dev(w), state)
        outs.append(host(o))
    torch.cuda.synchronize()
    seq = np.stack(outs, axis=2)
    # same arithmetic in a different order: equal to rounding of the output dtype
    check(seq, got[0], 1e-5 if io == "f32" else 8e-3, "decode chain out")
    check(host(state[0]), got[1], 1e-6, "decode chain S")
    check(host(state[1]), got[2], 1e-6, "decode chain z")
    assert np.array_equal(host(state[2]), got[3])
    want = oracle.verify(q, k, v, w, S, z, hist)
    check(seq, want[0], TOL[io], "decode chain vs oracle")


def test_no_leak_between_drafts_on_gpu():
    B, H, d, Kc, kk, io = 1, 4, 128, 3, 8, "bf16"
    q, k, v, w, S, z, hist = make_case(14, B, H, d, Kc, kk, io)
    base = run_gpu(q, k, v, w, S, z, hist, io)[0]
    for j in (0, 3, 6):
        q2, k2, v2 = q.copy(), k.copy(), v.copy()
        for a in (q2, k2, v2):
            a[:, :, j + 1:] = workloads.round_to_io(-2.0 * a[:, :, j + 1:] + 1.0, io)
        got = run_gpu(q2, k2, v2, w, S, z, hist, io)[0]
        assert np.array_equal(got[:, :, :j + 1], base[:, :, :j + 1]), f"draft {j} saw a later draft"
        assert not np.array_equal(got[:, :, j + 1:], base[:, :, j + 1:])


def test_decode_entry_point_shapes():
    """[B,H,d] tensors through linattn_decode."""
    B, H, d, Kc, io = 2, 3, 64, 5, "bf16"
    q, k, v, w, S, z, hist = make_case(15, B, H, d, Kc, 1, io)
    dt = IO[io]
    state = (dev(S), dev(z), dev(hist, dt))
    o = binding.decode(dev(q[:, :, 0], dt), dev(k[:, :, 0], dt), dev(v[:, :, 0], dt), dev(w), state)
    torch.cuda.synchronize()
    want = oracle.decode(q, k, v, w, S, z, hist)
    check(host(o)[:, :, None], want[0], TOL[io], "out")
    check(host(state[0]), want[1], 1e-5, "S")
    check(host(state[1]), want[2], 1e-5, "z")


def oracle_prefix_states(pq, pk, pv, w):
    """(S, z, hist) of every head after the prefix, by the oracle, a batch row at a time (all host threads)."""
    B, H, _, d = pq.shape
    Kc = w.shape[2]
    S = np.empty((B, H, d, d))
    z = np.empty((B, H, d))
    hist = np.empty((B, H, Kc - 1, d))
    for b in range(B):
        sl = slice(b, b + 1)
        _, S[sl], z[sl], hist[sl] = oracle.prefill_recurrent(host(pq[sl]), host(pk[sl]), host(pv[sl]), w.numpy())
    return S, z, hist


@pytest.fixture(scope="module")
def cfg4_prefix():
    """The 2048-token prefix of the B32 H32 d128 workload, the state linattn_prefill builds from it on the GPU, and the
    state the oracle builds from the same prefix for every head."""
    wl = workloads.CONFIGS["cfg4_llama7b_verify"]
    pq, pk, pv, w = workloads.prefill_tensors(wl)
    _, state = binding.prefill(pq.cuda(), pk.cuda(), pv.cuda(), w.cuda(), chunk=wl.chunk)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    ostate = oracle_prefix_states(pq, pk, pv, w)
    return wl, w, state, ostate


@pytest.mark.parametrize("kk", [1, 4, 8])
def test_config4_full_size_every_head(cfg4_prefix, kk):
    """B32 H32 d128, state from a 2048-token bf16 prefix built by linattn_prefill on the GPU at
    full size; the oracle follows all 1024 heads from the same inputs (prefix and drafts)."""
    wl, w, state0, (S1, z1, h1) = cfg4_prefix
    dt = IO[wl.io_dtype]
    state = tuple(t.clone() for t in state0)
    dq, dk, dv = (torch.from_numpy(a).to(dt) for a in workloads.draft_block(wl, kk))
    n_commit = (np.arange(wl.B) % (kk + 1)).astype(np.int32)
    out = binding.verify(dq.cuda(), dk.cuda(), dv.cuda(), w.cuda(), state, torch.from_numpy(n_commit).cuda())
    torch.cuda.synchronize()
    want = oracle.verify(host(dq), host(dk), host(dv), w.numpy(), S1, z1, h1, n_commit)
    e = check(host(out), want[0], TOL["bf16"], "out")
    check(host(state[0]), want[1], TOL["bf16"], "S")      # the prefix state is the bf16 prefill's: its bar
    check(host(state[1]), want[2], TOL["bf16"], "z")
    assert np.array_equal(host(state[2]), want[3]), "hist"
    print(f"config 4, k = {kk}: {wl.B * wl.H} heads, worst out error {e:.2e}", flush=True)


def test_long_decode_chain_from_the_config4_state(cfg4_prefix):
    """Sec. 4.2 over a long generation: 1008 sequential steps (decode, 4-draft and 8-draft verification with
    per-row commit counts, mixed) on 768 of the 1024 heads (24 batch rows: still whole heads on the matrix cores,
    and the oracle's share stays under a minute), every step through the C ABI, the oracle taking the same steps
    from the same fp32 state.  The state lives through all of them: S and z at the end to 1e-4, the
    outputs along the way to the bf16 bar."""
    wl, w, state0, _ = cfg4_prefix
    dt = IO[wl.io_dtype]
    B = 24
    state = tuple(t[:B].clone() for t in state0)
    S, z, hist = host(state[0]), host(state[1]), host(state[2])          # both sides start from the GPU's fp32 state
    gw, wn = w.cuda(), w.numpy()
    g = torch.Generator(device="cpu").manual_seed(wl.seed + 5)
    rng = np.random.default_rng(wl.seed + 5)
    pattern = (1, 1, 4, 1, 8, 1, 1, 4)                                   # drafts per step; 126 rounds = 1008 steps
    steps, tokens, worst = 0, 0, 0.0
    for rnd in range(126):
        for kk in pattern:
            dq, dk, dv = (torch.randn((B, wl.H, kk, wl.d), generator=g).to(dt) for _ in range(3))
            n_commit = None if kk == 1 else rng.integers(0, kk + 1, size=B).astype(np.int32)
            if kk == 1:
                out = binding.decode(dq[:, :, 0].cuda(), dk[:, :, 0].cuda(), dv[:, :, 0].cuda(), gw, state)[:, :, None]
            else:
                out = binding.verify(dq.cuda(), dk.cuda(), dv.cuda(), gw, state, torch.from_numpy(n_commit).cuda())
            want, S, z, hist = oracle.verify(host(dq), host(dk), host(dv), wn, S, z, hist, n_commit)
            steps += 1
            tokens += kk if n_commit is None else int(n_commit.mean())
            if steps % 48 == 0 or steps == 1008:
                worst = max(worst, check(host(out), want, TOL["bf16"], f"out at step {steps}"))
        if rnd % 25 == 0:
            print(f"decode chain: step {steps}", flush=True)
    torch.cuda.synchronize()
    assert steps == 1008
    eS = check(host(state[0]), S, 1e-4, "S after 1008 steps")
    ez = check(host(state[1]), z, 1e-4, "z after 1008 steps")
    assert np.array_equal(host(state[2]), hist), "hist after 1008 steps"
    print(f"decode chain: {steps} steps, about {tokens} tokens kept per row; S error {eS:.2e}, z error {ez:.2e}, "
          f"worst sampled out error {worst:.2e}", flush=True)
