"""The second feature map, phi(x) = max(x, 0) (LINATTN_PHI_RELU), on every entry point against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from parity import STATE_TOL, TOL, check, dev, host
from paper_2406_07368_amd import binding, workloads
from test_gpu_prefill import small_case
from test_gpu_verify import make_case

pytestmark = pytest.mark.gpu

IO = {"f32": torch.float32, "bf16": torch.bfloat16}
EPS = 0.05      # the denominator of this map can vanish


@pytest.mark.parametrize("io", ["bf16", "f32"])
@pytest.mark.parametrize("d,L,B,H", [(64, 65, 2, 3), (128, 130, 2, 3), (128, 2100, 1, 2)])
def test_relu_prefill(io, d, L, B, H):
    Kc = 3
    q, k, v, w, state = small_case(800 + d + L, B, H, L, d, Kc, io, True)
    with oracle.feature_map("relu"):
        want = oracle.prefill_recurrent(q, k, v, w, *state, eps=EPS)
    dt = IO[io]
    st = (dev(state[0]), dev(state[1]), dev(state[2], dt))
    out, (S, z, h) = binding.prefill(dev(q, dt), dev(k, dt), dev(v, dt), dev(w), st, 64, EPS, phi="relu")
    torch.cuda.synchronize()
    tol = TOL[io]
    check(host(out), want[0], tol, "out")
    check(host(S), want[1], tol, "S")
    check(host(z), want[2], tol, "z")
    assert np.array_equal(host(h), want[3])


@pytest.mark.parametrize("io,B,H", [("bf16", 2, 3), ("f32", 2, 3), ("bf16", 24, 32)])
def test_relu_verify_and_decode(io, B, H):
    d, Kc, kk = 128, 3, 6
    q, k, v, w, S, z, hist = make_case(810 + B, B, H, d, Kc, kk, io, prefix=12)
    z = np.abs(z)                     # a state this map could have produced: no negative mass
    n_commit = (np.arange(B) % (kk + 1)).astype(np.int32)
    with oracle.feature_map("relu"):
        want = oracle.verify(q, k, v, w, S, z, hist, n_commit, eps=EPS)
        want1 = oracle.decode(q[:, :, :1], k[:, :, :1], v[:, :, :1], w, S, z, hist, eps=EPS)
    dt = IO[io]
    state = (dev(S), dev(z), dev(hist, dt))
    out = binding.verify(dev(q, dt), dev(k, dt), dev(v, dt), dev(w), state, torch.from_numpy(n_commit).cuda(), EPS, phi="relu")
    state1 = (dev(S), dev(z), dev(hist, dt))
    out1 = binding.decode(dev(q[:, :, 0], dt), dev(k[:, :, 0], dt), dev(v[:, :, 0], dt), dev(w), state1, EPS, phi="relu")
    torch.cuda.synchronize()
    tol = TOL[io]
    check(host(out), want[0], tol, "verify out")
    check(host(state[0]), want[1], STATE_TOL, "verify S")
    check(host(state[1]), want[2], STATE_TOL, "verify z")
    check(host(out1)[:, :, None], want1[0], tol, "decode out")
    check(host(state1[0]), want1[1], STATE_TOL, "decode S")


def test_relu_tree_verify():
    B, H, d, Kc, n = 2, 3, 128, 4, 40
    q, k, v, w, S, z, hist = make_case(820, B, H, d, Kc, n, "bf16", prefix=12)
    z = np.abs(z)
    parent = workloads.candidate_tree(n, 25, 5)
    accept = np.array([n - 1, 7], dtype=np.int32)
    with oracle.feature_map("relu"):
        want = oracle.verify_tree(q, k, v, parent, w, S, z, hist, accept, eps=EPS)
    dt = torch.bfloat16
    state = (dev(S), dev(z), dev(hist, dt))
    out = binding.verify_tree(dev(q, dt), dev(k, dt), dev(v, dt), torch.from_numpy(parent).cuda(), dev(w), state,
                              torch.from_numpy(accept).cuda(), EPS, phi="relu")
    torch.cuda.synchronize()
    check(host(out), want[0], TOL["bf16"], "out")
    check(host(state[0]), want[1], STATE_TOL, "S")
    check(host(state[1]), want[2], STATE_TOL, "z")
    assert np.array_equal(host(state[2]), workloads.round_to_io(want[3], "bf16").astype(np.float64))
