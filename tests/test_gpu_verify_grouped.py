"""linattn_verify_grouped (generation with the three-branch form) on the GPU against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from parity import STATE_TOL, TOL, check, dev, host
from paper_2406_07368_amd import binding, workloads

pytestmark = pytest.mark.gpu

IO = {"f32": torch.float32, "bf16": torch.bfloat16}
C = 64


def make_state(rng, B, H, d, Kc, io, fill):
    """A state as a prefix would leave it: non-negative S (sums of positive features times values of either sign
    are of either sign, but z is positive), history and an open group with `fill[b]` rows in use."""
    S = (rng.standard_normal((B, H, d, d)) * 3).astype(np.float32)
    z = (np.abs(rng.standard_normal((B, H, d))) * 5 + 1).astype(np.float32)
    hist = workloads.round_to_io(rng.standard_normal((B, H, Kc - 1, d)), io)
    kwin = workloads.round_to_io(rng.standard_normal((B, H, C, d)), io)
    vwin = workloads.round_to_io(rng.standard_normal((B, H, C, d)), io)
    return S, z, hist, kwin, vwin, np.asarray(fill, dtype=np.int32)


def to_gpu(state, io):
    dt = IO[io]
    S, z, hist, kwin, vwin, fill = state
    H = S.shape[1]
    return dev(S), dev(z), dev(hist, dt), dev(kwin, dt), dev(vwin, dt), torch.from_numpy(np.repeat(fill[:, None], H, axis=1)).cuda()


def compare_state(got, want, io, what, fill_in):
    """S, z to the bar; history and the rows in use of the open group bit for bit (rows at or beyond fill are not
    part of the state)."""
    check(host(got[0]), want[0], STATE_TOL, what + " S")
    check(host(got[1]), want[1], STATE_TOL, what + " z")
    assert np.array_equal(host(got[2]), workloads.round_to_io(want[2], io).astype(np.float64)), what + " hist"
    assert np.array_equal(got[5].cpu().numpy(), np.repeat(want[5][:, None], got[5].shape[1], axis=1)), what + " fill (per head)"
    for b, n in enumerate(want[5]):
        assert np.array_equal(host(got[3])[b, :, :n], want[3][b, :, :n]), what + f" kwin, batch row {b}"
        assert np.array_equal(host(got[4])[b, :, :n], want[4][b, :, :n]), what + f" vwin, batch row {b}"


@pytest.mark.parametrize("io", ["bf16", "f32"])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("kk,Kc,fill", [(1, 3, (0, 17)), (1, 1, (63, 62)), (2, 3, (62, 10)), (3, 2, (63, 40)), (4, 3, (30, 61)), (5, 5, (59, 60)), (8, 2, (0, 63)),
                                        (13, 8, (50, 55)), (16, 3, (47, 48)), (16, 4, (63, 5)), (6, 1, (20, 63))])
def test_verify_grouped_matches_oracle(io, d, kk, Kc, fill):
    """Groups that stay open, groups that are completed by the kept drafts, drafts beyond the end of the group.
    bf16 with four or more drafts runs on the matrix cores, everything else on the vector ALUs."""
    B, H = 2, 3
    rng = np.random.default_rng(6000 + kk + d + Kc)
    state = make_state(rng, B, H, d, Kc, io, fill)
    q, k, v = (workloads.round_to_io(rng.standard_normal((B, H, kk, d)), io) for _ in range(3))
    w = workloads.conv_weights(rng, H, d, Kc)
    n_commit = np.array([kk, kk // 2], dtype=np.int32)
    want = oracle.verify_grouped(q, k, v, w, C, *state, n_commit=n_commit, alpha=0.8, eps=1e-3)
    gs = to_gpu(state, io)
    dt = IO[io]
    out = binding.verify_grouped(dev(q, dt), dev(k, dt), dev(v, dt), dev(w), gs, 0.8, torch.from_numpy(n_commit).cuda(), 1e-3)
    torch.cuda.synchronize()
    check(host(out), want[0], TOL[io], "out")
    compare_state(gs, want[1:], io, f"kk={kk} fill={fill}", fill)


def test_nothing_kept_leaves_everything_untouched():
    B, H, d, Kc, kk = 3, 2, 128, 3, 6
    rng = np.random.default_rng(6100)
    state = make_state(rng, B, H, d, Kc, "bf16", (5, 60, 63))
    q, k, v = (workloads.round_to_io(rng.standard_normal((B, H, kk, d)), "bf16") for _ in range(3))
    w = workloads.conv_weights(rng, H, d, Kc)
    gs = to_gpu(state, "bf16")
    before = [t.clone() for t in gs]
    bf = torch.bfloat16
    out = binding.verify_grouped(dev(q, bf), dev(k, bf), dev(v, bf), dev(w), gs, 1.0, torch.zeros(B, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    want = oracle.verify_grouped(q, k, v, w, C, *state, n_commit=np.zeros(B, dtype=np.int32))
    check(host(out), want[0], TOL["bf16"], "out")
    for a, b in zip(gs, before):
        assert torch.equal(a, b)


@pytest.mark.parametrize("io,d,block", [("bf16", 128, 1), ("bf16", 64, 7), ("f32", 64, 16), ("bf16", 128, 16)])
def test_generation_reproduces_the_grouped_prefill(io, d, block):
    """A sequence fed through verify_grouped from an empty state, block by block with everything kept, against the
    whole-sequence oracle; then the same after a GPU prefill of the first 128 tokens."""
    B, H, Kc, L = 2, 2, 3, 200
    rng = np.random.default_rng(6200 + d + block)
    q, k, v = (workloads.round_to_io(rng.standard_normal((B, H, L, d)), io) for _ in range(3))
    w = workloads.conv_weights(rng, H, d, Kc)
    want = oracle.prefill_grouped(q, k, v, w, C, alpha=1.0, eps=1e-3)
    dt = IO[io]
    gq, gk, gv, gw = dev(q, dt), dev(k, dt), dev(v, dt), dev(w)
    starts = [(0, binding.grouped_state(B, H, d, Kc, dt))]
    if io == "bf16":
        _, st = binding.prefill_grouped(gq[:, :, :128].contiguous(), gk[:, :, :128].contiguous(), gv[:, :, :128].contiguous(), gw, 1.0, None, 1e-3)
        starts.append((128, binding.grouped_state(B, H, d, Kc, dt, prefill_state=st)))
    for t_start, gs in starts:
        outs = []
        for t0 in range(t_start, L, block):
            sl = slice(t0, min(t0 + block, L))
            outs.append(binding.verify_grouped(gq[:, :, sl].contiguous(), gk[:, :, sl].contiguous(), gv[:, :, sl].contiguous(), gw, gs, 1.0, None, 1e-3))
        torch.cuda.synchronize()
        check(host(torch.cat(outs, dim=2)), want[0][:, :, t_start:], TOL[io], f"outputs from token {t_start}")
        assert gs[5].cpu().tolist() == [[L % C] * H] * B
        # completed groups + the open group's rows = the running sum of the whole sequence
        S_open = np.einsum("bhti,bhtc->bhic", oracle.phi(host(gs[3])[:, :, :L % C]), host(gs[4])[:, :, :L % C])
        check(host(gs[0]) + S_open, want[1], TOL[io], "S")


def test_whole_model_shape_one_token():
    """B32 H32 d128, one token per head (the decode step the bench times), open groups of different lengths."""
    B, H, d, Kc = 32, 32, 128, 3
    rng = np.random.default_rng(6300)
    fill = (np.arange(B) * 5) % C
    state = make_state(rng, B, H, d, Kc, "bf16", fill)
    q, k, v = (workloads.round_to_io(rng.standard_normal((B, H, 1, d)), "bf16") for _ in range(3))
    w = workloads.conv_weights(rng, H, d, Kc)
    bf = torch.bfloat16
    gs = to_gpu(state, "bf16")
    out = binding.verify_grouped(dev(q, bf), dev(k, bf), dev(v, bf), dev(w), gs, 1.0)
    torch.cuda.synchronize()
    rows = [0, 7, 13, 31]                                          # fill 0, 35, 1 (65 % 64), 27; row 13 of 5*13 = 65 -> 1
    sub = tuple(a[rows] for a in state)
    want = oracle.verify_grouped(q[rows], k[rows], v[rows], w, C, *sub)
    check(host(out)[rows], want[0], TOL["bf16"], "out")
    check(host(gs[0])[rows], want[1], STATE_TOL, "S")
    assert gs[5].cpu().numpy()[rows, 0].tolist() == want[6].tolist()
