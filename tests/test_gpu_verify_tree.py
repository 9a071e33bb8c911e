"""linattn_verify_tree on the GPU against the CPU oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

import oracle
from parity import STATE_TOL, TOL, check, dev, host
from paper_2406_07368_amd import binding, workloads
from test_gpu_verify import make_case

pytestmark = pytest.mark.gpu

IO = "bf16"
BF = torch.bfloat16


def random_tree(rng, n, roots=0.15):
    return np.array([-1] + [(-1 if rng.random() < roots else int(rng.integers(0, i))) for i in range(1, n)], dtype=np.int32)


def run_gpu(q, k, v, parent, w, S, z, hist, accept=None, eps=0.0):
    state = (dev(S), dev(z), dev(hist, BF))
    acc = None if accept is None else torch.from_numpy(np.asarray(accept, dtype=np.int32)).cuda()
    out = binding.verify_tree(dev(q, BF), dev(k, BF), dev(v, BF), torch.from_numpy(parent).cuda(), dev(w), state, acc, eps)
    torch.cuda.synchronize()
    return host(out), host(state[0]), host(state[1]), host(state[2])


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("n,Kc", [(1, 3), (2, 1), (5, 2), (17, 3), (32, 5), (33, 3), (47, 8), (64, 3), (64, 8)])
def test_tree_matches_oracle(d, n, Kc):
    B, H = 3, 4
    rng = np.random.default_rng(500 + n + d + Kc)
    q, k, v, w, S, z, hist = make_case(600 + n + d, B, H, d, Kc, n, IO, prefix=24)
    parent = random_tree(rng, n)
    accept = np.array([n - 1, -1, int(rng.integers(0, n))], dtype=np.int32)
    want = oracle.verify_tree(q, k, v, parent, w, S, z, hist, accept, eps=1e-3)
    got = run_gpu(q, k, v, parent, w, S, z, hist, accept, eps=1e-3)
    check(got[0], want[0], TOL[IO], "out")
    check(got[1], want[1], STATE_TOL, "S")
    check(got[2], want[2], STATE_TOL, "z")
    assert np.array_equal(got[3], workloads.round_to_io(want[3], IO).astype(np.float64)), "hist"
    # nothing accepted: that row's state comes back bit-unchanged
    assert np.array_equal(got[1][1], S[1].astype(np.float64))
    assert np.array_equal(got[2][1], z[1].astype(np.float64))
    assert np.array_equal(got[3][1], hist[1].astype(np.float64))


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("n,Kc", [(1, 3), (2, 1), (5, 2), (17, 3), (33, 5), (47, 8), (64, 3), (64, 8)])
def test_tree_of_fp32_candidates_matches_oracle(d, n, Kc):
    """fp32 candidates: exact fp32 multiply-adds on the vector ALUs, held to the fp32 bar."""
    B, H = 3, 4
    rng = np.random.default_rng(520 + n + d + Kc)
    q, k, v, w, S, z, hist = make_case(620 + n + d, B, H, d, Kc, n, "f32", prefix=24)
    parent = random_tree(rng, n)
    accept = np.array([n - 1, -1, int(rng.integers(0, n))], dtype=np.int32)
    want = oracle.verify_tree(q, k, v, parent, w, S, z, hist, accept, eps=1e-3)
    state = (dev(S), dev(z), dev(hist))
    out = binding.verify_tree(dev(q), dev(k), dev(v), torch.from_numpy(parent).cuda(), dev(w), state,
                              torch.from_numpy(accept).cuda(), 1e-3)
    torch.cuda.synchronize()
    check(host(out), want[0], TOL["f32"], "out")
    check(host(state[0]), want[1], STATE_TOL, "S")
    check(host(state[1]), want[2], STATE_TOL, "z")
    assert np.array_equal(host(state[2]), want[3]), "hist"
    assert np.array_equal(host(state[0])[1], S[1].astype(np.float64))      # nothing accepted: bit-unchanged
    assert np.array_equal(host(state[1])[1], z[1].astype(np.float64))


def test_fp32_tree_that_is_a_chain_equals_plain_verify():
    B, H, d, Kc, n = 4, 6, 128, 3, 11
    q, k, v, w, S, z, hist = make_case(43, B, H, d, Kc, n, "f32", prefix=12)
    chain = np.arange(n, dtype=np.int32) - 1
    n_commit = (np.arange(B) * 3 % (n + 1)).astype(np.int32)
    ts = (dev(S), dev(z), dev(hist))
    tout = binding.verify_tree(dev(q), dev(k), dev(v), torch.from_numpy(chain).cuda(), dev(w), ts, torch.from_numpy(n_commit - 1).cuda())
    vs = (dev(S), dev(z), dev(hist))
    vout = binding.verify(dev(q), dev(k), dev(v), dev(w), vs, torch.from_numpy(n_commit).cuda())
    torch.cuda.synchronize()
    check(host(tout), host(vout), 1e-5, "out")
    check(host(ts[0]), host(vs[0]), 1e-5, "S")
    check(host(ts[1]), host(vs[1]), 1e-5, "z")
    assert torch.equal(ts[2], vs[2])


def test_chain_shaped_tree_equals_plain_verify_on_the_gpu():
    """parent[i] = i - 1: the same outputs and state as linattn_verify with n_commit = accept + 1."""
    B, H, d, Kc, n = 24, 32, 128, 3, 13           # whole heads: both calls run on the matrix cores
    q, k, v, w, S, z, hist = make_case(41, B, H, d, Kc, n, IO, prefix=12)
    chain = np.arange(n, dtype=np.int32) - 1
    n_commit = (np.arange(B) * 3 % (n + 1)).astype(np.int32)
    tree = run_gpu(q, k, v, chain, w, S, z, hist, n_commit - 1)
    state = (dev(S), dev(z), dev(hist, BF))
    out = binding.verify(dev(q, BF), dev(k, BF), dev(v, BF), dev(w), state, torch.from_numpy(n_commit).cuda())
    torch.cuda.synchronize()
    check(tree[0], host(out), 1.2e-2, "out")      # the same terms grouped differently, output rounding apart
    check(tree[1], host(state[0]), 1e-5, "S")
    check(tree[2], host(state[1]), 1e-5, "z")
    assert np.array_equal(tree[3], host(state[2]))


def test_candidates_off_the_root_path_are_invisible_on_the_gpu():
    B, H, d, Kc, n = 1, 4, 128, 4, 40
    rng = np.random.default_rng(43)
    q, k, v, w, S, z, hist = make_case(44, B, H, d, Kc, n, IO, prefix=12)
    parent = random_tree(rng, n)
    base = run_gpu(q, k, v, parent, w, S, z, hist)[0]
    for i in (0, 7, 21, 39):
        on = set()
        a = i
        while a >= 0:
            on.add(a)
            a = int(parent[a])
        off = [c for c in range(n) if c not in on]
        q2, k2, v2 = q.copy(), k.copy(), v.copy()
        for x in (q2, k2, v2):
            x[:, :, off] = workloads.round_to_io(-2.0 * x[:, :, off] + 1.0, IO)
        other = run_gpu(q2, k2, v2, parent, w, S, z, hist)[0]
        assert np.array_equal(other[:, :, i], base[:, :, i]), f"candidate {i} saw a candidate off its root path"
        assert not np.array_equal(np.delete(other, sorted(on), axis=2), np.delete(base, sorted(on), axis=2))


def test_malformed_tree_entries_are_read_as_roots():
    B, H, d, Kc, n = 1, 2, 64, 3, 6
    q, k, v, w, S, z, hist = make_case(45, B, H, d, Kc, n, IO, prefix=12)
    bad = np.array([-1, 0, 7, -5, 4, 2], dtype=np.int32)          # 7 >= 2, -5 < -1, 4 >= 4
    good = np.array([-1, 0, -1, -1, -1, 2], dtype=np.int32)
    a = run_gpu(q, k, v, bad, w, S, z, hist, np.array([5], dtype=np.int32))
    b = run_gpu(q, k, v, good, w, S, z, hist, np.array([5], dtype=np.int32))
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


@pytest.fixture(scope="module")
def tree_workload():
    """B32 H32 d128, state from a 2048-token bf16 prefix built by linattn_prefill on the GPU at full size, and the
    oracle's state from the same prefix for every head."""
    from test_gpu_verify import oracle_prefix_states
    wl = workloads.CONFIGS["tree_verify_64x42"]
    pq, pk, pv, w = workloads.prefill_tensors(wl)
    _, state = binding.prefill(pq.cuda(), pk.cuda(), pv.cuda(), w.cuda(), chunk=wl.chunk)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    return wl, w, state, oracle_prefix_states(pq, pk, pv, w)


def test_tree_workload_full_size_every_head(tree_workload):
    """64 speculated tokens in a seeded tree with 42 root-to-leaf candidates (the shape of Sec. 5.3, Tab. 9)
    on 1024 heads; the oracle follows every head from the same inputs (prefix and candidates)."""
    wl, w, state0, (S1, z1, h1) = tree_workload
    n, leaves = wl.draft_k
    parent = workloads.candidate_tree(n, leaves, wl.seed)
    dq, dk, dv = (torch.from_numpy(a).to(BF) for a in workloads.draft_block(wl, n))
    state = tuple(t.clone() for t in state0)
    accept = ((np.arange(wl.B) * 7) % (n + 1) - 1).astype(np.int32)
    out = binding.verify_tree(dq.cuda(), dk.cuda(), dv.cuda(), torch.from_numpy(parent).cuda(), w.cuda(), state,
                              torch.from_numpy(accept).cuda())
    torch.cuda.synchronize()
    want = oracle.verify_tree(host(dq), host(dk), host(dv), parent, w.numpy(), S1, z1, h1, accept)
    e = check(host(out), want[0], TOL[IO], "out")
    check(host(state[0]), want[1], TOL[IO], "S")          # the prefix state is the bf16 prefill's: its bar
    check(host(state[1]), want[2], TOL[IO], "z")
    assert np.array_equal(host(state[2]), want[3]), "hist"
    print(f"tree workload: {wl.B * wl.H} heads, worst out error {e:.2e}", flush=True)
