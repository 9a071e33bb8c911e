"""The entry points under HIP graph capture: a serving loop replays decode / verify steps as a graph.

The library allocates nothing and keeps no state between calls, so a captured sequence of calls must give,
on every replay, what the same calls give when issued eagerly."""
import numpy as np
import pytest
import torch

from parity import dev, host
from paper_2406_07368_amd import binding, workloads
from test_gpu_verify import make_case

pytestmark = pytest.mark.gpu
BF = torch.bfloat16


def test_decode_verify_and_tree_steps_replay_as_a_graph():
    B, H, d, Kc = 24, 32, 128, 3                       # whole heads: the matrix-core kernels
    q, k, v, w, S, z, hist = make_case(71, B, H, d, Kc, 8, "bf16", prefix=12)
    gw = dev(w)
    dq, dk, dv = dev(q, BF), dev(k, BF), dev(v, BF)
    parent = torch.from_numpy(workloads.candidate_tree(8, 5, 3)).cuda()
    accept = torch.from_numpy((np.arange(B) % 8).astype(np.int32)).cuda()
    n_commit = torch.from_numpy((np.arange(B) % 5).astype(np.int32)).cuda()
    desc = binding.make_desc(B, H, d, Kc, 64, BF, L=1)

    def new_state():
        return dev(S), dev(z), dev(hist, BF)

    outs = [torch.empty((B, H, 1, d), dtype=BF, device="cuda"), torch.empty((B, H, 4, d), dtype=BF, device="cuda"),
            torch.empty((B, H, 8, d), dtype=BF, device="cuda")]

    # the inputs of the captured calls must outlive the capture: slice once, outside
    d1 = tuple(x[:, :, :1].contiguous() for x in (dq, dk, dv))
    d4 = tuple(x[:, :, 1:5].contiguous() for x in (dq, dk, dv))

    def steps_fixed(state, o):
        Ss, zs, hs = state
        binding.linattn_decode(desc, d1[0], d1[1], d1[2], gw, Ss, zs, hs, o[0])
        binding.linattn_verify(desc, 4, d4[0], d4[1], d4[2], gw, Ss, zs, hs, n_commit, o[1])
        binding.linattn_verify_tree(desc, 8, dq, dk, dv, parent, gw, Ss, zs, hs, accept, o[2])

    graph_state, eager_state = new_state(), new_state()
    eager_outs = [torch.empty_like(o) for o in outs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up on the capture stream, then restore the state
        steps_fixed(graph_state, outs)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for t, s0 in zip(graph_state, (S, z, hist)):
        t.copy_(dev(s0, t.dtype))
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        steps_fixed(graph_state, outs)
    torch.cuda.synchronize()
    for t, s0 in zip(graph_state, (S, z, hist)):       # capture does not execute: still the initial state
        assert torch.equal(t, dev(s0, t.dtype))
    for replay in range(4):
        g.replay()
        steps_fixed(eager_state, eager_outs)           # the program's own eager work between the replays
        torch.cuda.synchronize()
        for a, b in zip(outs, eager_outs):
            assert torch.equal(a, b), f"replay {replay}: outputs differ from the eager calls"
        for a, b in zip(graph_state, eager_state):
            assert torch.equal(a, b), f"replay {replay}: state differs from the eager calls"
    assert not np.array_equal(host(graph_state[0]), S.astype(np.float64))   # the state did move


@pytest.mark.parametrize("grouped", [False, True])
def test_prefill_replays_as_a_graph(grouped):
    """grouped: the three-branch form (same launch plan, its own kernel for the full pass)."""
    wl = workloads.CONFIGS["cfg2_gpt2_small"]        # segmented: three kernels and a workspace per call
    q, k, v, w = workloads.prefill_tensors(wl)
    gq, gk, gv, gw = q.cuda(), k.cuda(), v.cuda(), w.cuda()
    desc = binding.make_desc(wl.B, wl.H, wl.d, wl.conv_k, wl.chunk, BF, L=wl.L)
    nb = binding.linattn_workspace_bytes(desc, wl.L)
    assert nb > 0
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    mk = lambda: (torch.empty_like(gq), torch.empty((wl.B, wl.H, wl.d, wl.d), device="cuda"),
                  torch.empty((wl.B, wl.H, wl.d), device="cuda"),
                  torch.empty((wl.B, wl.H, wl.conv_k - 1, wl.d), dtype=BF, device="cuda"))
    want, got = mk(), mk()

    def call(dst):
        if grouped:
            binding.linattn_prefill_grouped(desc, wl.L, 0.75, gq, gk, gv, gw, None, None, None, *dst, ws, nb)
        else:
            binding.linattn_prefill(desc, wl.L, gq, gk, gv, gw, None, None, None, *dst, ws, nb)
    call(want)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        call(got)
    for replay in range(3):
        for t in got:
            t.zero_()
        ws.zero_()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(got, want):
            assert torch.equal(a, b), f"replay {replay} differs from the eager call"


def test_three_branch_generation_replays_as_a_graph():
    """A decode step and an eight-draft step of the three-branch form (vector-ALU and matrix-core kernels) captured
    once and replayed: the open groups grow, and on the later replays they are completed and re-opened."""
    B, H, d, Kc = 8, 32, 128, 3
    rng = np.random.default_rng(72)
    gw = dev(workloads.conv_weights(rng, H, d, Kc))
    q1, k1, v1 = (dev(workloads.round_to_io(rng.standard_normal((B, H, 1, d)), "bf16"), BF) for _ in range(3))
    q8, k8, v8 = (dev(workloads.round_to_io(rng.standard_normal((B, H, 8, d)), "bf16"), BF) for _ in range(3))
    n_commit = torch.from_numpy((np.arange(B) % 9).astype(np.int32)).cuda()
    desc = binding.make_desc(B, H, d, Kc, 64, BF, L=1)

    def new_state():
        st = list(binding.grouped_state(B, H, d, Kc, BF))
        st[5].fill_(40)                                   # 40 rows in use: the third replay completes some groups
        torch.manual_seed(5)
        st[3].copy_(torch.randn(st[3].shape, device="cuda").to(BF))
        st[4].copy_(torch.randn(st[4].shape, device="cuda").to(BF))
        st[1].fill_(3.0)
        return st

    def steps(st, o):
        binding.linattn_verify_grouped(desc, 1, 1.0, q1, k1, v1, gw, *st, None, o[0])
        binding.linattn_verify_grouped(desc, 8, 1.0, q8, k8, v8, gw, *st, n_commit, o[1])

    graph_state, eager_state = new_state(), new_state()
    outs = [torch.empty_like(q1), torch.empty_like(q8)]
    eager_outs = [torch.empty_like(o) for o in outs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        steps(graph_state, outs)
    torch.cuda.synchronize()
    for replay in range(5):
        g.replay()
        steps(eager_state, eager_outs)
        torch.cuda.synchronize()
        for a, b in zip(outs, eager_outs):
            assert torch.equal(a, b), f"replay {replay}: outputs differ from the eager calls"
        for a, b in zip(graph_state, eager_state):
            assert torch.equal(a, b), f"replay {replay}: state differs from the eager calls"
    assert int(graph_state[5].min()) < 40                 # some groups were completed and re-opened


def test_training_step_replays_as_a_graph():
    """Forward and gradient of the three-branch form (groups of 256, 63 taps: a dozen launches and two workspaces)
    captured once and replayed, outputs and workspaces cleared between the replays."""
    wl = workloads.CONFIGS["flash_L1024"]
    q, k, v, w = workloads.prefill_tensors(wl)
    gq, gk, gv, gw = q.cuda(), k.cuda(), v.cuda(), w.cuda()
    gdo = workloads.upstream_gradient_tensor(wl).cuda()
    desc = binding.make_desc(wl.B, wl.H, wl.d, wl.conv_k, wl.chunk, BF, L=wl.L)
    nf, nb = binding.linattn_workspace_bytes(desc, wl.L), binding.linattn_backward_workspace_bytes(desc, wl.L)
    wsf, wsb = torch.empty(nf, dtype=torch.uint8, device="cuda"), torch.empty(nb, dtype=torch.uint8, device="cuda")
    mk = lambda: [torch.empty_like(gq) for _ in range(4)] + [torch.empty_like(gw)]
    want, got = mk(), mk()

    def call(dst):
        out, dq, dk, dv, dw = dst
        binding.linattn_prefill_grouped(desc, wl.L, 1.0, gq, gk, gv, gw, None, None, None, out, None, None, None, wsf, nf)
        binding.linattn_prefill_grouped_backward(desc, wl.L, 1.0, gq, gk, gv, gw, gdo, dq, dk, dv, dw, wsb, nb)
    call(want)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        call(got)
    for replay in range(3):
        for t in got:
            t.zero_()
        wsf.zero_()
        wsb.zero_()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip(got, want):
            assert torch.equal(a, b), f"replay {replay} differs from the eager call"


FIRST_CALL_UNDER_CAPTURE = r"""
import sys, torch
sys.path.insert(0, sys.argv[1])
from paper_2406_07368_amd import binding, workloads
wl = workloads.CONFIGS["flash_L1024"]
q, k, v, w = (t.cuda() for t in workloads.prefill_tensors(wl))
do = workloads.upstream_gradient_tensor(wl).cuda()
desc = binding.make_desc(wl.B, wl.H, wl.d, wl.conv_k, wl.chunk, torch.bfloat16, L=wl.L)
nb = binding.linattn_backward_workspace_bytes(desc, wl.L)
ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
mk = lambda: [torch.empty_like(q) for _ in range(3)] + [torch.empty_like(w)]
got, want = mk(), mk()
side = torch.cuda.Stream()
g = torch.cuda.CUDAGraph()
with torch.cuda.graph(g, stream=side):          # the library's very first call in this process
    binding.linattn_prefill_grouped_backward(desc, wl.L, 1.0, q, k, v, w, do, *got, ws, nb)
g.replay()
torch.cuda.synchronize()
binding.linattn_prefill_grouped_backward(desc, wl.L, 1.0, q, k, v, w, do, *want, ws, nb)   # eager: makes the side stream
torch.cuda.synchronize()
assert all(torch.equal(a, b) for a, b in zip(got, want)), "captured first call differs from the eager call"
for t in got:
    t.zero_()
g.replay()
torch.cuda.synchronize()
assert all(torch.equal(a, b) for a, b in zip(got, want)), "replay after the eager call differs"
print("ok")
"""


def test_gradient_captured_as_the_first_call_of_a_process():
    """The gradient forks part of its work onto a stream the library makes at its first such call -- unless that call
    is being captured: then everything stays on the caller's stream.  A fresh process captures the gradient before any
    eager call, replays it, and compares with the eager call (which then does make the side stream)."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, "-c", FIRST_CALL_UNDER_CAPTURE, root], capture_output=True, text=True, timeout=280)
    assert res.returncode == 0 and res.stdout.strip().endswith("ok"), res.stdout[-2000:] + res.stderr[-4000:]

