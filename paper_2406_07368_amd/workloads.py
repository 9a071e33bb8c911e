"""Seeded synthetic inputs with the shapes of the five workloads.

This module holds none of the method's arithmetic: it only draws random
numbers and rounds them to the i/o dtype, so that the very same arrays can be
handed to the GPU library and to whatever it is checked against.

The workloads stand in for the activations of the models the paper measures
(LLaMA-2-7B: 32 heads of 128; GPT-2-small: 12 heads of 64; group size 64 for
LLaMA, Sec. 5 "Settings"); no dataset, prompt or trained weight is used.

Recipe: ``numpy.random.default_rng(seed)``; standard normals drawn in the
fixed order Q, K, V, conv weights; Q, K, V multiplied by ``scale``; conv
weights multiplied by ``Kc ** -0.5`` (variance 1/Kc); everything cast to
float32 and Q, K, V rounded once to the i/o dtype (round-to-nearest-even for
bf16).  Arrays are returned as float32 numpy arrays holding exactly
representable values of the i/o dtype.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    mode: str          # "prefill", "verify" or "verify_tree"
    B: int
    H: int
    L: int             # prefill length, or prefix length for verify workloads
    d: int
    io_dtype: str      # "f32" or "bf16"
    chunk: int
    conv_k: int
    scale: float
    seed: int
    draft_k: tuple = ()
    d_v: int = 0       # width of the value rows when it differs from d (a multiple of d); 0: d

    def small(self, **kw) -> "Workload":
        return replace(self, **kw)


CONFIGS = {
    # config 1: tiny all-fp32 prefill, checked against the brute-force quadratic form
    "cfg1_fp32_tiny": Workload("cfg1_fp32_tiny", "prefill", 1, 4, 256, 64, "f32", 64, 3, 1.0, 1001),
    # config 2: GPT-2-small-shaped prefill
    "cfg2_gpt2_small": Workload("cfg2_gpt2_small", "prefill", 4, 12, 1024, 64, "bf16", 64, 3, 1.0, 1002),
    # config 3: LLaMA-2-7B-shaped layer prefill (inputs scaled by d**-0.5)
    "cfg3_llama7b_prefill": Workload("cfg3_llama7b_prefill", "prefill", 8, 32, 4096, 128, "bf16", 64, 3,
                                     128 ** -0.5, 1003),
    # config 4: decode + speculative verify on a state built from a 2048-token prefix
    "cfg4_llama7b_verify": Workload("cfg4_llama7b_verify", "verify", 32, 32, 2048, 128, "bf16", 64, 3, 1.0,
                                    1004, (1, 4, 8)),
    # tree-structured verify on the state of config 4: 64 speculated tokens, 42 sequence candidates
    # (root-to-leaf paths), the shape of the paper's single-batch comparison (Sec. 5.3, Tab. 9)
    "tree_verify_64x42": Workload("tree_verify_64x42", "verify_tree", 32, 32, 2048, 128, "bf16", 64, 3, 1.0,
                                  1006, (64, 42)),
    # the shape of the paper's FLASH experiment (Sec. 4.1: masked DWConv of kernel size 63; Sec. 5 "Settings" and
    # Sec. 5.3: groups of 256 tokens, batch 1, sequences of 1K / 4K / 8K tokens), as eight heads of 128
    "flash_L1024": Workload("flash_L1024", "prefill", 1, 8, 1024, 128, "bf16", 256, 63, 128 ** -0.5, 1011),
    "flash_L4096": Workload("flash_L4096", "prefill", 1, 8, 4096, 128, "bf16", 256, 63, 128 ** -0.5, 1012),
    "flash_L8192": Workload("flash_L8192", "prefill", 1, 8, 8192, 128, "bf16", 256, 63, 128 ** -0.5, 1013),
    # the same layer on a batch of eight sequences: 2048 groups of 256 tokens, several per compute unit -- the size
    # at which the kernels of the FLASH shape are bound by the chip and not by the latency of a few launches
    "flash_B8_L8192": Workload("flash_B8_L8192", "prefill", 8, 8, 8192, 128, "bf16", 256, 63, 128 ** -0.5, 1014),
    # value rows wider than key rows (Sec. 3, Eq. 1: d_k and d_v are separate): the LLaMA-2-7B layer shape with the
    # query/key width halved, prefill and verify
    "wide_values_prefill": Workload("wide_values_prefill", "prefill", 8, 32, 4096, 64, "bf16", 64, 3, 64 ** -0.5, 1021, (), 128),
    "wide_values_verify": Workload("wide_values_verify", "verify", 32, 32, 2048, 64, "bf16", 64, 3, 1.0, 1022, (1, 4, 8), 128),
    # config 5: long-context prefill
    "cfg5_long_context": Workload("cfg5_long_context", "prefill", 1, 32, 65536, 128, "bf16", 128, 5, 1.0, 1005),
}


def round_to_io(a: np.ndarray, io_dtype: str) -> np.ndarray:
    """float32 array whose values are exactly representable in ``io_dtype``."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if io_dtype == "f32":
        return a
    if io_dtype == "bf16":
        return torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    raise ValueError(f"unknown io dtype {io_dtype!r}")


def torch_dtype(io_dtype: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[io_dtype]


def conv_weights(rng, H: int, d: int, conv_k: int) -> np.ndarray:
    return (rng.standard_normal((H, d, conv_k)) * conv_k ** -0.5).astype(np.float32)


def prefill_inputs(wl: Workload, seed: int | None = None):
    """Returns q, k, v [B,H,L,d] and conv weights w [H,d,Kc] (float32 numpy)."""
    rng = np.random.default_rng(wl.seed if seed is None else seed)
    shape = (wl.B, wl.H, wl.L, wl.d)
    q, k, v = (round_to_io(rng.standard_normal(shape) * wl.scale, wl.io_dtype) for _ in range(3))
    w = conv_weights(rng, wl.H, wl.d, wl.conv_k)
    return q, k, v, w


def draft_block(wl: Workload, kk: int, step: int = 0, seed: int | None = None):
    """q, k, v [B,H,kk,d] for one verify/decode step (seed + 100*(step+1))."""
    base = wl.seed if seed is None else seed
    rng = np.random.default_rng(base + 100 * (step + 1))
    return tuple(round_to_io(rng.standard_normal((wl.B, wl.H, kk, width)) * wl.scale, wl.io_dtype)
                 for width in (wl.d, wl.d, wl.d_v or wl.d))


def candidate_tree(n: int, leaves: int, seed: int) -> np.ndarray:
    """parent[n] (int32) of a seeded tree with ``n`` candidates of which exactly ``leaves`` have no child,
    i.e. ``leaves`` root-to-leaf sequence candidates.  parent[i] < i; -1 marks a candidate that follows the
    verified sequence directly.  The n - leaves inner candidates come first (each hangs under an earlier inner
    candidate or under the verified sequence, so the tree is a few steps deep and bushy near the root, like
    the hand-made trees of tree-based speculative decoders); every inner candidate without a child
    then gets a leaf, and the remaining leaves pick an inner candidate at random.  Only the shape is modelled: no decoder's
    actual tree is reproduced.
    """
    inner = n - leaves
    if not (0 <= inner <= leaves and n >= 1):
        raise ValueError("need n >= 1 and at most as many inner candidates as leaves")
    rng = np.random.default_rng(seed)
    parent = np.full(n, -1, dtype=np.int32)
    has_child = np.zeros(max(inner, 1), dtype=bool)
    for i in range(1, inner):
        parent[i] = int(rng.integers(-1, i))
        if parent[i] >= 0:
            has_child[parent[i]] = True
    childless = [i for i in range(inner) if not has_child[i]]
    for j in range(inner, n):
        if childless:
            parent[j] = childless.pop(0)
        elif inner:
            parent[j] = int(rng.integers(0, inner))
    return parent


def random_state(wl: Workload, tokens: int, seed: int | None = None):
    """A plausible running state without running any attention code.

    S, z and hist with the magnitudes a ``tokens``-long prefix of unit-normal
    inputs would leave behind: S ~ N(0, tokens * 1.6), z ~ tokens * 0.95 +
    N(0, tokens * 0.5); used only where the *values* of the state do not
    matter (bandwidth measurements).  float32, hist rounded to the io dtype.
    """
    rng = np.random.default_rng((wl.seed if seed is None else seed) + 7)
    S = (rng.standard_normal((wl.B, wl.H, wl.d, wl.d)) * (1.6 * tokens) ** 0.5).astype(np.float32)
    z = (0.95 * tokens + rng.standard_normal((wl.B, wl.H, wl.d)) * (0.5 * tokens) ** 0.5).astype(np.float32)
    hist = round_to_io(rng.standard_normal((wl.B, wl.H, wl.conv_k - 1, wl.d)) * wl.scale, wl.io_dtype)
    return S, z, hist


def upstream_gradient(shape, io_dtype: str, seed: int) -> np.ndarray:
    """Seeded stand-in for d loss / d out of a training step: N(0, 1), exactly representable in ``io_dtype``."""
    return round_to_io(np.random.default_rng(seed).standard_normal(shape), io_dtype)


def upstream_gradient_tensor(wl: Workload, seed: int | None = None):
    """Full-size variant (torch CPU tensor in the i/o dtype, ``torch.Generator``), shape of the outputs of ``wl``."""
    g = torch.Generator(device="cpu").manual_seed((wl.seed if seed is None else seed) + 7919)
    return torch.randn((wl.B, wl.H, wl.L, wl.d_v or wl.d), generator=g, dtype=torch.float32).to(torch_dtype(wl.io_dtype))


def prefill_tensors(wl: Workload, seed: int | None = None):
    """Full-size variant of ``prefill_inputs``: torch CPU tensors already in the i/o dtype.

    Same distribution and scale, drawn with ``torch.Generator`` (float32 normals, order Q, K, V)
    because numpy's float64 stream is too slow and too large for the 10^8..10^9-element
    workloads.  Conv weights come from ``conv_weights(default_rng(seed))`` as above.
    """
    s = wl.seed if seed is None else seed
    g = torch.Generator(device="cpu").manual_seed(s)
    dt = torch_dtype(wl.io_dtype)
    q, k, v = ((torch.randn((wl.B, wl.H, wl.L, width), generator=g, dtype=torch.float32) * wl.scale).to(dt)
               for width in (wl.d, wl.d, wl.d_v or wl.d))
    w = torch.from_numpy(conv_weights(np.random.default_rng(s), wl.H, wl.d_v or wl.d, wl.conv_k))
    return q, k, v, w
