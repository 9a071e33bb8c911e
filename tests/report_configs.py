#!/usr/bin/env python3
"""Runs the five workloads on the GPU and prints one table row each: time, rate, fraction of the
HBM and MFMA roofs, worst error against the oracle (all heads where that takes seconds, a sample
of heads at the full-size workloads), and the oracle's own time on one and on all host threads.

    python tests/report_configs.py          (needs the GPU; about a minute)

Not collected by pytest; the parity tests assert the same errors against their bars.
"""
from __future__ import annotations

import os
import statistics
import sys
import time

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, HERE)
sys.path.insert(0, os.path.dirname(HERE))

import oracle  # noqa: E402
from parity import err_stats, host, rel_err  # noqa: E402
from paper_2406_07368_amd import binding, workloads  # noqa: E402

HBM, MFMA = 8.0e12, 2.5e15


def gpu_time(fn, warm=60, n=60):
    """Median launch duration in seconds once the clocks have settled."""
    for _ in range(warm):
        fn()
    ev = []
    for _ in range(n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); fn(); e1.record()
        ev.append((e0, e1))
    torch.cuda.synchronize()
    return statistics.median(a.elapsed_time(b) for a, b in ev) * 1e-3


def oracle_time(fn_heads, threads_all):
    """Seconds per head on one thread and on all threads (heads are independent)."""
    oracle.set_num_threads(1)
    t0 = time.perf_counter(); fn_heads(1); t1 = time.perf_counter() - t0
    oracle.set_num_threads(threads_all)
    t0 = time.perf_counter(); fn_heads(threads_all); tn = (time.perf_counter() - t0) / threads_all
    return t1, tn


def prefill_row(name, sample, grouped=False):
    """grouped: the three-branch form (groups of 64, alpha 1) on the same tensors."""
    wl = workloads.CONFIGS[name]
    io = torch.float32 if wl.io_dtype == "f32" else torch.bfloat16
    q, k, v, w = workloads.prefill_tensors(wl)
    gq, gk, gv, gw = q.cuda(), k.cuda(), v.cuda(), w.cuda()
    out, (S, z, h) = binding.prefill(gq, gk, gv, gw, None, wl.chunk, grouped_alpha=1.0 if grouped else None)
    torch.cuda.synchronize()
    heads = sample if sample is not None else [(b, hh) for b in range(wl.B) for hh in range(wl.H)]
    worst, extra = 0.0, (0.0, 0.0)
    ref = oracle.prefill_quadratic if name.startswith("cfg1") else oracle.prefill_recurrent
    if grouped:
        def ref(q_, k_, v_, w_):
            return oracle.prefill_grouped(q_, k_, v_, w_, 64, alpha=1.0)
    for b, hh in heads:
        sl = (slice(b, b + 1), slice(hh, hh + 1))
        want = ref(host(q[sl]), host(k[sl]), host(v[sl]), w[hh:hh + 1].numpy())
        worst = max(worst, rel_err(host(out[sl]), want[0]), rel_err(host(S[sl]), want[1]), rel_err(host(z[sl]), want[2]))
        _, ma, p999 = err_stats(host(out[sl]), want[0])
        extra = (max(extra[0], ma), max(extra[1], p999))
    desc = binding.make_desc(wl.B, wl.H, wl.d, wl.conv_k, wl.chunk, io, L=wl.L)
    nb = binding.linattn_workspace_bytes(desc, wl.L)
    ws = torch.empty(max(nb, 16), dtype=torch.uint8, device="cuda")
    if grouped:
        t = gpu_time(lambda: binding.linattn_prefill_grouped(desc, wl.L, 1.0, gq, gk, gv, gw, None, None, None, out, S, z, h, ws, nb))
    else:
        t = gpu_time(lambda: binding.linattn_prefill(desc, wl.L, gq, gk, gv, gw, None, None, None, out, S, z, h, ws, nb))
    esz = 4 if wl.io_dtype == "f32" else 2
    nbytes = 4 * wl.B * wl.H * wl.L * wl.d * esz
    ht = wl.B * wl.H * wl.L
    fc, fd = ht * (2 * (wl.chunk + 1) * wl.d + 4 * wl.d * wl.d), ht * (4 * wl.chunk * wl.d + 4 * wl.d * wl.d)
    threads = oracle.num_threads()
    rng = np.random.default_rng(1)

    def run_heads(n):
        shp = (1, n, wl.L, wl.d)
        a, b_, c = (workloads.round_to_io(rng.standard_normal(shp) * wl.scale, wl.io_dtype) for _ in range(3))
        ref(a, b_, c, workloads.conv_weights(rng, n, wl.d, wl.conv_k))
    t1, tn = oracle_time(run_heads, threads)
    nh = wl.B * wl.H
    mf = "-" if wl.io_dtype == "f32" else f"{100 * fc / t / MFMA:.1f} / {100 * fd / t / MFMA:.1f}"
    if grouped:
        name += ", three-branch form"
        fc = fd = ht * (4 * wl.chunk * wl.d + 4 * wl.d * wl.d)
    return (f"| {name} | {t * 1e6:.1f} µs | {wl.B * wl.L / t / 1e6:.2f} M tokens/s | {100 * nbytes / t / HBM:.1f} | {mf} | "
            f"{t1 * nh:.2f} s | {tn * nh:.2f} s ({threads}) | {worst:.1e} ({'all' if sample is None else len(sample)} heads); "
            f"out: max abs {extra[0]:.1e}, p99.9 rel {extra[1]:.1e} |")


def verify_rows():
    wl = workloads.CONFIGS["cfg4_llama7b_verify"]
    pq, pk, pv, w = workloads.prefill_tensors(wl)
    gw = w.cuda()
    _, state0 = binding.prefill(pq.cuda(), pk.cuda(), pv.cuda(), gw, chunk=wl.chunk)
    torch.cuda.synchronize()
    sample = [(0, 0), (3, 17), (15, 31), (31, 5)]
    pre = {}
    for b, h in sample:
        sl = (slice(b, b + 1), slice(h, h + 1))
        pre[(b, h)] = oracle.prefill_recurrent(host(pq[sl]), host(pk[sl]), host(pv[sl]), w[h:h + 1].numpy())[1:]
    sets = [tuple(t.clone() for t in state0) for _ in range(16)]     # 1.1 GB: no call finds its state in cache
    rows = []
    threads = oracle.num_threads()
    for kk in (8, 4, 1):
        dq, dk, dv = (torch.from_numpy(a).to(torch.bfloat16) for a in workloads.draft_block(wl, kk))
        gq, gk, gv = dq.cuda(), dk.cuda(), dv.cuda()
        state = tuple(t.clone() for t in state0)
        out = binding.verify(gq, gk, gv, gw, state)
        torch.cuda.synchronize()
        worst, extra = 0.0, (0.0, 0.0)
        for b, h in sample:
            sl = (slice(b, b + 1), slice(h, h + 1))
            S1, z1, h1 = pre[(b, h)]
            want = oracle.verify(host(dq[sl]), host(dk[sl]), host(dv[sl]), w[h:h + 1].numpy(), S1, z1, h1)
            worst = max(worst, rel_err(host(out[sl]), want[0]), rel_err(host(state[0][sl]), want[1]))
            _, ma, p999 = err_stats(host(out[sl]), want[0])
            extra = (max(extra[0], ma), max(extra[1], p999))
        desc = binding.make_desc(wl.B, wl.H, wl.d, wl.conv_k, wl.chunk, torch.bfloat16, L=1)
        o = torch.empty_like(gq)
        i = [0]

        def call():
            S, z, h = sets[i[0] % len(sets)]
            i[0] += 1
            binding.linattn_verify(desc, kk, gq, gk, gv, gw, S, z, h, None, o)
        t = gpu_time(call)
        heads = wl.B * wl.H
        nbytes = heads * ((wl.d * wl.d + wl.d) * 8 + kk * wl.d * 8 + (wl.conv_k - 1) * wl.d * 4)
        S1, z1, h1 = pre[sample[0]]

        def run_heads(n):
            a = np.repeat(host(dq[:1, :1]), n, axis=1)
            oracle.verify(a, a, a, np.repeat(w[:1].numpy(), n, axis=0), np.repeat(S1, n, axis=1), np.repeat(z1, n, axis=1),
                          np.repeat(h1, n, axis=1))
        t1, tn = oracle_time(run_heads, threads)
        rows.append(f"| cfg4 verify k={kk} | {t * 1e6:.1f} µs | {wl.B * kk / t / 1e6:.2f} M draft tokens/s | {100 * nbytes / t / HBM:.1f} | - | "
                    f"{t1 * heads * 1e3:.1f} ms | {tn * heads * 1e3:.1f} ms ({threads}) | {worst:.1e} ({len(sample)} heads); "
                    f"out: max abs {extra[0]:.1e}, p99.9 rel {extra[1]:.1e} |")
    # tree-structured verify on the same state: 64 candidates, 42 root-to-leaf paths
    tw = workloads.CONFIGS["tree_verify_64x42"]
    n, leaves = tw.draft_k
    parent = workloads.candidate_tree(n, leaves, tw.seed)
    dq, dk, dv = (torch.from_numpy(a).to(torch.bfloat16) for a in workloads.draft_block(tw, n))
    gq, gk, gv, gp = dq.cuda(), dk.cuda(), dv.cuda(), torch.from_numpy(parent).cuda()
    accept = torch.from_numpy(((np.arange(tw.B) * 7) % n).astype(np.int32))
    state = tuple(t.clone() for t in state0)
    out = binding.verify_tree(gq, gk, gv, gp, gw, state, accept.cuda())
    torch.cuda.synchronize()
    worst, extra = 0.0, (0.0, 0.0)
    for b, h in sample:
        sl = (slice(b, b + 1), slice(h, h + 1))
        S1, z1, h1 = pre[(b, h)]
        want = oracle.verify_tree(host(dq[sl]), host(dk[sl]), host(dv[sl]), parent, w[h:h + 1].numpy(), S1, z1, h1,
                                  accept[b:b + 1].numpy())
        worst = max(worst, rel_err(host(out[sl]), want[0]), rel_err(host(state[0][sl]), want[1]))
        _, ma, p999 = err_stats(host(out[sl]), want[0])
        extra = (max(extra[0], ma), max(extra[1], p999))
    desc = binding.make_desc(tw.B, tw.H, tw.d, tw.conv_k, tw.chunk, torch.bfloat16, L=1)
    o = torch.empty_like(gq)
    ga = accept.cuda()
    i = [0]

    def call_tree():
        S, z, h = sets[i[0] % len(sets)]
        i[0] += 1
        binding.linattn_verify_tree(desc, n, gq, gk, gv, gp, gw, S, z, h, ga, o)
    t = gpu_time(call_tree)
    heads = tw.B * tw.H
    nbytes = heads * ((tw.d * tw.d + tw.d) * 8 + n * tw.d * 8 + (tw.conv_k - 1) * tw.d * 4)
    S1, z1, h1 = pre[sample[0]]

    def run_tree_heads(m):
        a = np.repeat(host(dq[:1, :1]), m, axis=1)
        oracle.verify_tree(a, a, a, parent, np.repeat(w[:1].numpy(), m, axis=0), np.repeat(S1, m, axis=1),
                           np.repeat(z1, m, axis=1), np.repeat(h1, m, axis=1))
    t1, tn = oracle_time(run_tree_heads, threads)
    rows.append(f"| tree verify, {n} candidates / {leaves} paths | {t * 1e6:.1f} µs | {tw.B * n / t / 1e6:.2f} M candidate tokens/s | "
                f"{100 * nbytes / t / HBM:.1f} | - | {t1 * heads * 1e3:.1f} ms | {tn * heads * 1e3:.1f} ms ({threads}) | "
                f"{worst:.1e} ({len(sample)} heads); out: max abs {extra[0]:.1e}, p99.9 rel {extra[1]:.1e} |")
    # generation with the three-branch form: one token per head, open groups of 32 rows, on the same completed-group state
    rng = np.random.default_rng(77)
    C = 64
    fill = np.full(wl.B, 32, dtype=np.int32)
    kwin, vwin = (torch.from_numpy(workloads.round_to_io(rng.standard_normal((wl.B, wl.H, C, wl.d)), "bf16")).to(torch.bfloat16) for _ in range(2))
    dq, dk, dv = (torch.from_numpy(a).to(torch.bfloat16) for a in workloads.draft_block(wl, 1))
    gq, gk, gv = dq.cuda(), dk.cuda(), dv.cuda()

    def gstate(st):
        return (st[0].clone(), st[1].clone(), st[2].clone(), kwin.cuda(), vwin.cuda(),
                torch.from_numpy(np.repeat(fill[:, None], wl.H, axis=1)).cuda())
    gs = gstate(state0)
    out = binding.verify_grouped(gq, gk, gv, gw, gs)
    torch.cuda.synchronize()
    worst, extra = 0.0, (0.0, 0.0)
    for b, h in sample:
        sl = (slice(b, b + 1), slice(h, h + 1))
        S1, z1, h1 = pre[(b, h)]
        want = oracle.verify_grouped(host(dq[sl]), host(dk[sl]), host(dv[sl]), w[h:h + 1].numpy(), C, S1, z1, h1,
                                     host(kwin[sl]), host(vwin[sl]), fill[b:b + 1])
        worst = max(worst, rel_err(host(out[sl]), want[0]))
        _, ma, p999 = err_stats(host(out[sl]), want[0])
        extra = (max(extra[0], ma), max(extra[1], p999))
    gsets = [gstate(st) for st in sets]
    desc = binding.make_desc(wl.B, wl.H, wl.d, wl.conv_k, 64, torch.bfloat16, L=1)
    o = torch.empty_like(gq)
    nothing = torch.zeros(wl.B, dtype=torch.int32, device="cuda")     # nothing kept: every call sees the same 32 rows
    i = [0]

    def call_g():
        S, z, h, kw, vwn, fl = gsets[i[0] % len(gsets)]
        i[0] += 1
        binding.linattn_verify_grouped(desc, 1, 1.0, gq, gk, gv, gw, S, z, h, kw, vwn, fl, nothing, o)
    t = gpu_time(call_g)
    heads = wl.B * wl.H
    nbytes = heads * ((wl.d * wl.d + wl.d) * 4 + 2 * 32 * wl.d * 2 + 4 * wl.d * 2 + (wl.conv_k - 1) * wl.d * 2)
    S1, z1, h1 = pre[sample[0]]

    def run_g_heads(m):
        a = np.repeat(host(dq[:1, :1]), m, axis=1)
        kw1 = np.repeat(host(kwin[:1, :1]), m, axis=1)
        oracle.verify_grouped(a, a, a, np.repeat(w[:1].numpy(), m, axis=0), C, np.repeat(S1, m, axis=1), np.repeat(z1, m, axis=1),
                              np.repeat(h1, m, axis=1), kw1, kw1, fill[:1])
    t1, tn = oracle_time(run_g_heads, threads)
    rows.append(f"| cfg4 shape, three-branch generation step (1 token, 32 rows open, nothing kept) | {t * 1e6:.1f} µs | {wl.B / t / 1e6:.2f} M tokens/s | "
                f"{100 * nbytes / t / HBM:.1f} | - | {t1 * heads * 1e3:.1f} ms | {tn * heads * 1e3:.1f} ms ({threads}) | "
                f"{worst:.1e} ({len(sample)} heads; out only); out: max abs {extra[0]:.1e}, p99.9 rel {extra[1]:.1e} |")
    return rows


def main():
    binding.load()
    print("| workload | GPU time | rate | % of 8 TB/s | % of 2.5 PF (causal / full tiles) | oracle, 1 thread | oracle, all threads | max rel err (floored by the head's rms; worst of out, S, z) |")
    print("|---|---|---|---|---|---|---|---|")
    print(prefill_row("cfg1_fp32_tiny", None), flush=True)
    print(prefill_row("cfg2_gpt2_small", None), flush=True)
    print(prefill_row("cfg3_llama7b_prefill", [(0, 0), (3, 31), (7, 16)]), flush=True)
    for r in verify_rows():
        print(r, flush=True)
    print(prefill_row("cfg5_long_context", [(0, 0), (0, 31)]), flush=True)
    print(prefill_row("cfg3_llama7b_prefill", [(0, 0), (3, 31), (7, 16)], grouped=True), flush=True)


if __name__ == "__main__":
    main()
