"""Gradient of the three-branch form (the training direction of the FLASH-shaped row, Sec. 5.3) on the GPU against the
CPU oracle, through the C ABI: dq, dk, dv element by element, the conv-weight gradient summed over the batch."""
import numpy as np
import pytest
import torch

import oracle
from parity import TOL, check, check_unfloored, dev, host
from paper_2406_07368_amd import binding, workloads

pytestmark = pytest.mark.gpu

# dw is a sum of fp32 products of bf16 numbers in fp32, in a fixed order: the fp32 bar
DW_TOL = TOL["f32"]


def case(seed, B, H, L, d, Kc, scale=1.0):
    rng = np.random.default_rng(seed)
    q, k, v = (workloads.round_to_io(rng.standard_normal((B, H, L, d)) * scale, "bf16") for _ in range(3))
    w = workloads.conv_weights(rng, H, d, Kc)
    dout = workloads.upstream_gradient((B, H, L, d), "bf16", seed + 1)
    return q, k, v, w, dout


def run(q, k, v, w, dout, group, alpha=1.0, eps=0.0, phi="elu1"):
    bf = torch.bfloat16
    dq, dk, dv, dw = binding.prefill_grouped_backward(dev(q, bf), dev(k, bf), dev(v, bf), dev(w), dev(dout, bf), alpha, eps,
                                                      phi=phi, group=group)
    torch.cuda.synchronize()
    return {"dq": host(dq), "dk": host(dk), "dv": host(dv), "dw": host(dw)}


def compare(got, want, what):
    for name in ("dq", "dk", "dv"):
        check(got[name], want[name], TOL["bf16"], f"{what} {name}")
    scale = max(float(np.sqrt(np.mean(want["dw"] ** 2))), 1e-30)
    err = float(np.max(np.abs(got["dw"] - want["dw"]))) / scale
    assert err <= DW_TOL, f"{what} dw: max abs err / rms {err:.3e} > {DW_TOL:.1e}"


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("group", [64, 256])
@pytest.mark.parametrize("L,Kc", [(1, 3), (31, 1), (64, 3), (65, 8), (256, 5), (257, 3), (300, 63), (700, 17), (1024, 3)])
def test_gradient_against_the_oracle(d, group, L, Kc):
    """Several groups and a ragged last one, one token, exactly one group, conv windows longer than the sequence."""
    q, k, v, w, dout = case(9000 + L + d + group + Kc, 2, 3, L, d, Kc)
    want = oracle.prefill_grouped_backward(q, k, v, w, dout, group, alpha=0.8, eps=1e-3)
    compare(run(q, k, v, w, dout, group, 0.8, 1e-3), want, f"d={d} group={group} L={L} Kc={Kc}")


@pytest.mark.parametrize("group", [64, 256])
def test_gradient_with_eps_zero_and_alpha_zero(group):
    """eps = 0: the first group has no grouped branch (its denominator is exactly zero) and nothing may divide by it;
    alpha = 0: the grouped branch is gone, and with it every path through the group-level sums."""
    q, k, v, w, dout = case(9100 + group, 2, 2, 600, 128, 3)
    for alpha in (1.0, 0.0):
        want = oracle.prefill_grouped_backward(q, k, v, w, dout, group, alpha=alpha, eps=0.0)
        compare(run(q, k, v, w, dout, group, alpha, 0.0), want, f"group={group} alpha={alpha}")


@pytest.mark.parametrize("d,group", [(64, 64), (128, 256)])
def test_gradient_with_the_relu_feature_map(d, group):
    q, k, v, w, dout = case(9200 + d, 2, 2, 500, d, 3)
    with oracle.feature_map("relu"):
        want = oracle.prefill_grouped_backward(q, k, v, w, dout, group, alpha=1.2, eps=0.5)
    compare(run(q, k, v, w, dout, group, 1.2, 0.5, phi="relu"), want, f"relu d={d}")


def test_gradient_of_token_major_tensors():
    """[B, L, H, d] in memory, handed over as strided [B, H, L, d] views: the layout a projection GEMM writes."""
    B, H, L, d, Kc, group = 2, 3, 520, 128, 5, 256
    q, k, v, w, dout = case(9300, B, H, L, d, Kc)
    want = oracle.prefill_grouped_backward(q, k, v, w, dout, group, alpha=1.0, eps=1e-3)
    bf = torch.bfloat16
    tm = [dev(np.ascontiguousarray(a.transpose(0, 2, 1, 3)), bf).transpose(1, 2) for a in (q, k, v, dout)]
    dq, dk, dv, dw = binding.prefill_grouped_backward(tm[0], tm[1], tm[2], dev(w), tm[3], 1.0, 1e-3, group=group)
    torch.cuda.synchronize()
    assert dq.stride() == tm[0].stride()
    compare({"dq": host(dq), "dk": host(dk), "dv": host(dv), "dw": host(dw)}, want, "token-major")


def test_gradient_is_reproducible_bit_for_bit():
    """No atomics anywhere: two calls give the same bits, also for the sums over the batch."""
    q, k, v, w, dout = case(9400, 3, 2, 700, 128, 63)
    a = run(q, k, v, w, dout, 256)
    b = run(q, k, v, w, dout, 256)
    for name in a:
        assert np.array_equal(a[name], b[name]), name


@pytest.mark.parametrize("group,L", [(64, 1536), (256, 3000)])
def test_gradient_with_more_workgroups_than_the_chip_holds(group, L):
    """48 heads x dozens of groups: every kernel of the call runs in several rounds, and the sums over the batch
    rows that share a head's conv weights have six terms."""
    q, k, v, w, dout = case(9600 + group, 6, 8, L, 128, 3, scale=0.5)
    want = oracle.prefill_grouped_backward(q, k, v, w, dout, group, alpha=1.0, eps=0.0)
    compare(run(q, k, v, w, dout, group, 1.0, 0.0), want, f"group={group} L={L}")


def test_conv_weight_gradient_not_wanted():
    """dconv_w = NULL: the other three gradients are the same bits, and the conv-weight pass does not run."""
    q, k, v, w, dout = case(9500, 2, 2, 300, 64, 5)
    bf = torch.bfloat16
    args = (dev(q, bf), dev(k, bf), dev(v, bf), dev(w), dev(dout, bf))
    with_dw = binding.prefill_grouped_backward(*args, group=64)
    without = binding.prefill_grouped_backward(*args, group=64, want_dw=False)
    torch.cuda.synchronize()
    assert without[3] is None
    for a, b in zip(with_dw[:3], without[:3]):
        assert torch.equal(a, b)


def test_no_tokens():
    bf = torch.bfloat16
    empty = torch.empty((2, 3, 0, 128), dtype=bf, device="cuda")
    w = dev(workloads.conv_weights(np.random.default_rng(1), 3, 128, 3))
    dq, dk, dv, dw = binding.prefill_grouped_backward(empty, empty, empty, w, empty, group=256)
    torch.cuda.synchronize()
    assert dq.shape == empty.shape and torch.all(dw == 0)


@pytest.mark.parametrize("name", ["flash_L1024", "flash_L4096", "flash_L8192"])
def test_flash_shapes_every_head(name):
    """The sizes of the paper's FLASH experiment (groups of 256, 63 taps, batch 1), every head, every element."""
    wl = workloads.CONFIGS[name]
    q, k, v, w = workloads.prefill_tensors(wl)
    dout = workloads.upstream_gradient_tensor(wl)
    dq, dk, dv, dw = binding.prefill_grouped_backward(q.cuda(), k.cuda(), v.cuda(), w.cuda(), dout.cuda(), 1.0, group=wl.chunk)
    torch.cuda.synchronize()
    want = oracle.prefill_grouped_backward(q.double().numpy(), k.double().numpy(), v.double().numpy(), w.double().numpy(),
                                           dout.double().numpy(), wl.chunk, alpha=1.0)
    got = {"dq": host(dq), "dk": host(dk), "dv": host(dv), "dw": host(dw)}
    compare(got, want, name)
    for n in ("dq", "dk", "dv"):
        check_unfloored(got[n], want[n], TOL["bf16"], f"{name} {n}")


def test_flash_shape_on_a_batch_one_head_of_every_batch_row():
    """B8 H8 L8192: 2048 groups, several rounds of every kernel.  The oracle follows one head through all eight batch
    rows: dq, dk, dv of those rows and the conv-weight gradient of that head (a sum over the batch), forward and back."""
    wl = workloads.CONFIGS["flash_B8_L8192"]
    hsel = 5
    q, k, v, w = workloads.prefill_tensors(wl)
    dout = workloads.upstream_gradient_tensor(wl)
    gq, gk, gv, gw, gd = q.cuda(), k.cuda(), v.cuda(), w.cuda(), dout.cuda()
    out, (S, z, hist) = binding.prefill_grouped(gq, gk, gv, gw, 1.0, group=wl.chunk)
    dq, dk, dv, dw = binding.prefill_grouped_backward(gq, gk, gv, gw, gd, 1.0, group=wl.chunk)
    torch.cuda.synchronize()
    sl = slice(hsel, hsel + 1)
    hq, hk, hv, hd = (t[:, sl].double().numpy() for t in (q, k, v, dout))
    hw = w[sl].double().numpy()
    fwant = oracle.prefill_grouped(hq, hk, hv, hw, wl.chunk, alpha=1.0)
    check(host(out[:, sl]), fwant[0], TOL["bf16"], "forward out")
    check(host(S[:, sl]), fwant[1], TOL["bf16"], "forward S")
    check(host(z[:, sl]), fwant[2], TOL["bf16"], "forward z")
    want = oracle.prefill_grouped_backward(hq, hk, hv, hw, hd, wl.chunk, alpha=1.0)
    got = {"dq": host(dq[:, sl]), "dk": host(dk[:, sl]), "dv": host(dv[:, sl]), "dw": host(dw[sl])}
    compare(got, want, f"{wl.name} head {hsel}")
    for n in ("dq", "dk", "dv"):
        check_unfloored(got[n], want[n], TOL["bf16"], f"{wl.name} head {hsel} {n}")
