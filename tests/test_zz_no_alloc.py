"""linattn_prefill_noalloc (the entry point that allocates nothing: its scratch is a static device array) against
linattn_prefill on the same inputs, through the C ABI: two calls in a row, the second on a smaller input."""
import numpy as np
import pytest
import torch

from parity import dev
from paper_2406_07368_amd import binding, workloads

pytestmark = pytest.mark.gpu

BF = torch.bfloat16


def both_entry_points(seed, B, H, L, d, Kc, with_state):
    rng = np.random.default_rng(seed)
    q, k, v = (dev(workloads.round_to_io(rng.standard_normal((B, H, L, d)), "bf16"), BF) for _ in range(3))
    w = dev(workloads.conv_weights(rng, H, d, Kc))
    st = (None, None, None)
    if with_state:
        st = (dev((rng.standard_normal((B, H, d, d)) * 3).astype(np.float32)),
              dev((np.abs(rng.standard_normal((B, H, d))) * 5 + 1).astype(np.float32)),
              dev(workloads.round_to_io(rng.standard_normal((B, H, Kc - 1, d)), "bf16"), BF))
    desc = binding.make_desc(B, H, d, Kc, 64, BF, L=L)
    need = binding.linattn_workspace_bytes(desc, L)
    assert 0 < need <= binding.linattn_noalloc_scratch_bytes(), "the case must be one that uses the scratch"
    res = []
    for noalloc in (False, True):
        out = torch.full_like(q, float("nan"))
        S = torch.full((B, H, d, d), float("nan"), device="cuda")
        z = torch.full((B, H, d), float("nan"), device="cuda")
        h = torch.zeros((B, H, Kc - 1, d), device="cuda", dtype=BF)
        if noalloc:
            binding.linattn_prefill_noalloc(desc, L, q, k, v, w, *st, out, S, z, h)
        else:
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            binding.linattn_prefill(desc, L, q, k, v, w, *st, out, S, z, h, ws, need)
        torch.cuda.synchronize()
        res.append((out, S, z, h))
    return res


def test_noalloc_prefill_equals_prefill_twice_in_a_row():
    """The same kernels on the same plan: bit-identical outputs and state.  The second call is smaller than the first
    (fewer segments, smaller head dimension) and finds the first call's contents in the scratch."""
    for seed, shape in ((71, (1, 2, 4200, 128, 5, True)), (72, (2, 3, 1100, 64, 3, False))):
        want, got = both_entry_points(seed, *shape)
        for name, a, b in zip(("out", "S", "z", "hist"), want, got):
            assert torch.isfinite(a.float()).all(), name
            assert torch.equal(a, b), f"{name} differs between linattn_prefill and linattn_prefill_noalloc for {shape}"


def test_noalloc_prefill_without_segments_needs_no_scratch():
    """B*H fills the chip: no workspace in either entry point; results identical as well."""
    B, H, L, d, Kc = 8, 32, 200, 128, 3
    rng = np.random.default_rng(73)
    q, k, v = (dev(workloads.round_to_io(rng.standard_normal((B, H, L, d)), "bf16"), BF) for _ in range(3))
    w = dev(workloads.conv_weights(rng, H, d, Kc))
    desc = binding.make_desc(B, H, d, Kc, 64, BF, L=L)
    assert binding.linattn_workspace_bytes(desc, L) == 0
    o1, o2 = torch.empty_like(q), torch.empty_like(q)
    binding.linattn_prefill(desc, L, q, k, v, w, None, None, None, o1, None, None, None, None, 0)
    binding.linattn_prefill_noalloc(desc, L, q, k, v, w, None, None, None, o2, None, None, None)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2)
