#!/usr/bin/env python3
"""Benchmark of the linear-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One *step* is one pass over every stage of the path on synthetic, seeded inputs
already resident in HBM:

    linattn_prefill   LLaMA-2-7B layer shape  B8 H32 L4096 d128 bf16, chunk 64, Kc 3,
                      q, k, v, out token-major [B,L,H,d] as a projection GEMM writes them
                      (--layout bhld for head-major; that time is reported beside it anyway)
    linattn_verify    B32 H32 d128, fp32 state, k = 8 drafts  (state updated in place)
    linattn_verify    same, k = 4
    linattn_decode    same, one token

The headline ``value`` is prefill tokens/s (B*L divided by the mean duration of the
prefill launches, measured with events on the launch stream inside the timed
region); the verify/decode step times are reported beside it in microseconds with
their own HBM roofline; the tree-structured verify (64 candidates) and the three-branch form of
the prefill with its one-token generation step are timed after the steps and reported as ``tree_verify``,
``prefill_grouped`` and ``verify_grouped`` (one token = decode, and eight drafts); the prefill workloads of
configs 1, 2 and 5 likewise, as ``other_configs``.  Between steps the verify state rotates over 32 separate
state sets (2.1 GB) and the prefill inputs over 2 sets (2.1 GB) so that nothing is
served from the 256 MB last-level cache.

Prints ONE JSON line.  ``roofline`` is for the dominant kernel (prefill):
algorithmic bytes per launch / measured mean launch duration against 8 TB/s.
``cpu_baseline`` is the fp64 CPU oracle timed on this machine's host cores on a
bounded sample of the same prefill workload: a baseline, not a target.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import glob
import sys
import threading
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2406_07368_amd import binding, workloads  # noqa: E402


class BoardTelemetry:
    """The board's own sensors (sysfs: socket power in microwatts, the core clock level marked with '*'), read from a
    thread every 20 ms between start() and stop().  Not a profiler and not part of any timing: it says whether the
    timed steps ran at the power limit and at which core clock.  Sensors that cannot be read are left out."""

    def __init__(self):
        self.power = next(iter(sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") +
                                      glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average"))), None)
        self.sclk = next(iter(sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))), None)
        cap = self.power and os.path.join(os.path.dirname(self.power), "power1_cap")
        self.cap_w = self._read_float(cap, 1e-6) if cap and os.path.exists(cap) else None
        self.watts, self.mhz, self._stop, self._thread = [], [], threading.Event(), None

    @staticmethod
    def _read_float(path, scale):
        try:
            with open(path) as f:
                return float(f.read().split()[0]) * scale
        except (OSError, ValueError, IndexError):
            return None

    def _sample(self):
        if self.power:
            w = self._read_float(self.power, 1e-6)
            if w is not None:
                self.watts.append(w)
        if self.sclk:
            try:
                with open(self.sclk) as f:
                    m = re.search(r"(\d+)\s*Mhz\s*\*", f.read(), re.I)
                if m:
                    self.mhz.append(float(m.group(1)))
            except OSError:
                pass

    def start(self):
        if not (self.power or self.sclk):
            return

        def loop():
            while not self._stop.wait(0.02):
                self._sample()
        self._thread = threading.Thread(target=loop, daemon=True)
        self._thread.start()

    def stop(self):
        self._stop.set()
        if self._thread:
            self._thread.join()
        out = {"what": "board sensors sampled every 20 ms over the settling and the timed steps (not a measurement of any kernel)"}
        if self.watts:
            out["socket_power_w"] = {"mean": sum(self.watts) / len(self.watts), "max": max(self.watts), "samples": len(self.watts),
                                     "limit": self.cap_w}
        if self.mhz:
            out["core_clock_mhz"] = {"mean": sum(self.mhz) / len(self.mhz), "min": min(self.mhz), "samples": len(self.mhz)}
        return out if len(out) > 1 else None

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix throughput
SETTLE_WINDOW = 20             # launches whose durations must agree before the timed region starts
SETTLE_CAP = 400               # untimed settling steps at most


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100,
                    help="untimed steps first; the clocks of a GPU that was idle take some tens of launches to settle")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--only", choices=["all", "prefill", "verify"], default="all",
                    help="restrict the step to one stage (for profiling runs)")
    ap.add_argument("--state-sets", type=int, default=32)
    ap.add_argument("--no-telemetry", action="store_true", help="do not sample the board's power and clock sensors")
    ap.add_argument("--prefill-workload", default="cfg3_llama7b_prefill",
                    choices=["cfg2_gpt2_small", "cfg3_llama7b_prefill", "cfg5_long_context"],
                    help="prefill workload of the step (the headline is cfg3; the others are for side measurements)")
    ap.add_argument("--length", type=int, default=0, help="override L of the prefill workload (length sweeps)")
    ap.add_argument("--layout", choices=["blhd", "bhld"], default="blhd",
                    help="memory layout of q, k, v, out: blhd = token-major [B,L,H,d], the layout a projection "
                         "GEMM writes (default); bhld = head-major [B,H,L,d]")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one elementwise kernel that reads 1 GiB and writes 1 GiB "
                         "(reference dispatch for scaling the HBM byte counters)")
    return ap.parse_args()


def prefill_bytes(wl):
    """Algorithmic HBM bytes of one prefill call: read Q, K, V, write out (state and weights are negligible)."""
    return 4 * wl.B * wl.H * wl.L * wl.d * 2


def prefill_flops(wl):
    """Per head-token: 2(C+1)d + 4d^2 (causal count) and 4Cd + 4d^2 (full tiles)."""
    ht = wl.B * wl.H * wl.L
    return ht * (2 * (wl.chunk + 1) * wl.d + 4 * wl.d * wl.d), ht * (4 * wl.chunk * wl.d + 4 * wl.d * wl.d)


def verify_bytes(wl, kk):
    """S and z read and written once, q/k/v read, out written, history read and written."""
    heads = wl.B * wl.H
    state = heads * (wl.d * wl.d + wl.d) * 4 * 2
    io = heads * kk * wl.d * 2 * 4
    hist = heads * (wl.conv_k - 1) * wl.d * 2 * 2
    return state + io + hist


def layouts(wl):
    """Tensor shape in memory and (batch, head, token) element strides of the two layouts."""
    B, H, L, d = wl.B, wl.H, wl.L, wl.d
    return {"blhd": ((B, L, H, d), (L * H * d, d, H * d)),
            "bhld": ((B, H, L, d), (H * L * d, L * d, d))}


# rocprofv3 counter summaries of the prefill workloads (all launches of one call summed)
TRAFFIC_FILES = {"cfg3_llama7b_prefill": "prefill_mfma_cfg3_pmc.txt", "cfg5_long_context": "prefill_cfg5_pmc.txt",
                 "cfg2_gpt2_small": "prefill_cfg2_pmc.txt"}


def read_traffic(name):
    """HBM bytes per launch measured with rocprofv3 counters, if a summary is committed under profiles/."""
    if not name:
        return None
    path = os.path.join(ROOT, "profiles", name)
    try:
        m = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read())
        return float(m.group(1)) if m else None
    except OSError:
        return None


def cpu_baseline(wl, seconds):
    """The oracle as it stands, all host threads, on whole heads of the prefill workload."""
    import oracle
    threads = oracle.num_threads()
    rng = np.random.default_rng(wl.seed)

    def run(heads):
        shp = (1, heads, wl.L, wl.d)
        q, k, v = (workloads.round_to_io(rng.standard_normal(shp) * wl.scale, wl.io_dtype) for _ in range(3))
        w = workloads.conv_weights(rng, heads, wl.d, wl.conv_k)
        t0 = time.perf_counter()
        oracle.prefill_recurrent(q, k, v, w)
        return time.perf_counter() - t0

    oracle.set_num_threads(1)
    t_one = run(1)                                           # one head on one thread
    oracle.set_num_threads(threads)
    t_probe = run(threads)                                   # one head per thread
    heads = int(max(threads, min(wl.B * wl.H, threads * round(seconds / max(t_probe, 1e-3)))))
    heads -= heads % threads
    t = run(heads)
    head_tokens_per_s = heads * wl.L / t
    return {"value": head_tokens_per_s / wl.H, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "value_one_thread": wl.L / t_one / wl.H,
            "sample": f"{heads} of {wl.B * wl.H} heads x L={wl.L} (fp64 recurrent form), {t:.1f} s; "
                      f"scaled to a {wl.H}-head layer"}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    binding.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.Stream(device=dev)

    pw = workloads.CONFIGS[args.prefill_workload]
    if args.length > 0:
        pw = pw.small(L=args.length)
    vw = workloads.CONFIGS["cfg4_llama7b_verify"]
    do_prefill = args.only in ("all", "prefill")
    do_verify = args.only in ("all", "verify")

    # ---- inputs, resident in HBM before anything is timed -------------------------------------------
    g = torch.Generator(device=dev).manual_seed(pw.seed)
    n_in = 2 if do_prefill else 0
    pin = []
    # the values are i.i.d., so drawing them straight into either layout gives the same workload
    shape, strides = layouts(pw)[args.layout]
    for _ in range(n_in):
        q, k, v = ((torch.randn(shape, generator=g, device=dev) * pw.scale).to(torch.bfloat16) for _ in range(3))
        pin.append((q, k, v, torch.empty_like(q)))
    pwts = torch.from_numpy(workloads.conv_weights(np.random.default_rng(pw.seed), pw.H, pw.d, pw.conv_k)).to(dev)
    pdesc = binding.make_desc(pw.B, pw.H, pw.d, pw.conv_k, pw.chunk, torch.bfloat16, strides=strides)
    ws_bytes = binding.linattn_workspace_bytes(pdesc, pw.L)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
    S_out = torch.empty((pw.B, pw.H, pw.d, pw.d), device=dev)
    z_out = torch.empty((pw.B, pw.H, pw.d), device=dev)
    h_out = torch.empty((pw.B, pw.H, pw.conv_k - 1, pw.d), device=dev, dtype=torch.bfloat16)

    vwts = torch.from_numpy(workloads.conv_weights(np.random.default_rng(vw.seed), vw.H, vw.d, vw.conv_k)).to(dev)
    vdesc = binding.make_desc(vw.B, vw.H, vw.d, vw.conv_k, vw.chunk, torch.bfloat16, L=1)
    states, drafts = [], {}
    if do_verify:
        # one real state from the 2048-token prefix, then copies with a small seeded perturbation
        q, k, v, _ = workloads.prefill_tensors(vw)
        _, st0 = binding.prefill(q.to(dev), k.to(dev), v.to(dev), vwts, chunk=vw.chunk)
        del q, k, v
        for i in range(args.state_sets):
            S = st0[0] * (1.0 + 0.001 * i)
            states.append((S, st0[1].clone(), st0[2].clone()))
        for kk in (8, 4, 1):
            dq, dk, dv = (torch.from_numpy(a).to(torch.bfloat16).to(dev) for a in workloads.draft_block(vw, kk))
            drafts[kk] = (dq, dk, dv, torch.empty_like(dq))
    torch.cuda.synchronize()

    ev = {name: [] for name in ("prefill", "verify8", "verify4", "decode")}

    def timed(name, fn, record):
        if record:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fn()
            e1.record(stream)
            ev[name].append((e0, e1))
        else:
            fn()

    def step(i, record):
        if do_prefill:
            q, k, v, out = pin[i % len(pin)]
            timed("prefill", lambda: binding.linattn_prefill(pdesc, pw.L, q, k, v, pwts, None, None, None, out,
                                                             S_out, z_out, h_out, ws, ws_bytes, stream), record)
        if do_verify:
            # every call gets a state set of its own, so none finds its state in the last-level cache
            for j, (name, kk) in enumerate((("verify8", 8), ("verify4", 4))):
                S, z, h = states[(3 * i + j) % len(states)]
                dq, dk, dv, o = drafts[kk]
                timed(name, lambda: binding.linattn_verify(vdesc, kk, dq, dk, dv, vwts, S, z, h, None, o, stream), record)
            S, z, h = states[(3 * i + 2) % len(states)]
            dq, dk, dv, o = drafts[1]
            timed("decode", lambda: binding.linattn_decode(vdesc, dq, dk, dv, vwts, S, z, h, o, stream), record)

    for i in range(args.warmup):
        step(i, False)
    # Whatever --warmup says, untimed steps go on until the duration of the dominant launch has settled:
    # a GPU that was idle runs its first launches at boost clock, is then pulled down hard by the power
    # management and recovers over some tens of launches.  Settled = every duration of the last window lies
    # within +-5 % of the window's median, and the medians of the last four windows lie within 1 % of each other
    # (the recovery is a slow drift, about 1 % per window towards its end: three windows each within 1 % of the one
    # before it still let a run start 8 % above the level it reached 100 steps later, on a GPU that another job
    # had just left warm).  The unsettled figures are reported beside the settled ones.
    settle_name = "prefill" if do_prefill else "verify8"
    settle_steps, settle_hist, meds = 0, [], []
    sensors = BoardTelemetry()
    if not args.no_telemetry:
        sensors.start()
    while settle_steps < SETTLE_CAP:
        n0 = len(ev[settle_name])
        for i in range(SETTLE_WINDOW):
            step(args.warmup + settle_steps + i, True)
        stream.synchronize()
        settle_steps += SETTLE_WINDOW
        last = [a.elapsed_time(b) for a, b in ev[settle_name][n0:]]
        settle_hist.extend(last)
        med = float(np.median(last))
        meds.append(med)
        if (len(meds) >= 4 and max(meds[-4:]) - min(meds[-4:]) <= 0.01 * med
                and max(abs(t - med) for t in last) <= 0.05 * med):
            break
    # the timed region follows at once (an idle gap of a few milliseconds would send the clock through its hump
    # again): the settling records stay in the lists and are skipped when the durations are read
    n_settled = {name: len(lst) for name, lst in ev.items()}
    first_step = args.warmup + settle_steps
    if args.copy_calibration:
        # a plain elementwise kernel of known traffic (reads 1 GiB, writes 1 GiB): the reference
        # against which the FETCH_SIZE / WRITE_SIZE counters of the same run are scaled
        with torch.cuda.stream(stream):
            a = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
            b = torch.empty_like(a)
            torch.add(a, 1.0, out=b)
    stream.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(first_step + i, True)
    stream.synchronize()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    telemetry = sensors.stop()

    other_layout_ms = None
    if do_prefill and args.only == "all":
        # the same prefill in the other memory layout, outside the timed region, for the record
        other = "bhld" if args.layout == "blhd" else "blhd"
        shape2, strides2 = layouts(pw)[other]
        desc2 = binding.make_desc(pw.B, pw.H, pw.d, pw.conv_k, pw.chunk, torch.bfloat16, strides=strides2)
        pin2 = [tuple(t.view(shape2) for t in s4) for s4 in pin]   # same memory, read in the other order
        ev2 = []
        for i in range(3 + min(args.steps, 10)):
            q, k, v, out = pin2[i % len(pin2)]
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            binding.linattn_prefill(desc2, pw.L, q, k, v, pwts, None, None, None, out, S_out, z_out, h_out, ws,
                                    ws_bytes, stream)
            e1.record(stream)
            if i >= 3:
                ev2.append((e0, e1))
        stream.synchronize()
        other_layout_ms = {"layout": other, "mean": sum(a.elapsed_time(b) for a, b in ev2) / len(ev2),
                           "min": min(a.elapsed_time(b) for a, b in ev2)}

    grouped = None
    if do_prefill and args.only == "all" and pw.chunk == 64:
        # next row of the scope (not part of the step): the three-branch form of the same prefill (grouped linear
        # attention + local softmax attention + masked conv), same inputs, same layout, same algorithmic bytes
        ev4 = []
        for i in range(20 + min(args.steps, 50)):
            q, k, v, out = pin[i % len(pin)]
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            binding.linattn_prefill_grouped(pdesc, pw.L, 1.0, q, k, v, pwts, None, None, None, out, S_out, z_out, h_out,
                                            ws, ws_bytes, stream)
            e1.record(stream)
            if i >= 20:
                ev4.append((e0, e1))
        stream.synchronize()
        t_ms = [a.elapsed_time(b) for a, b in ev4]
        t_mean = sum(t_ms) / len(t_ms)
        nb = prefill_bytes(pw)
        grouped = {"workload": f"{pw.name} B{pw.B} H{pw.H} L{pw.L} d{pw.d} bf16, groups of 64, Kc{pw.conv_k}, alpha 1, same tensors "
                               "and layout as the prefill of the step",
                   "ms": {"mean": t_mean, "median": float(np.median(t_ms)), "min": min(t_ms)},
                   "tokens_per_s": pw.B * pw.L / (t_mean * 1e-3),
                   "roofline": {"bound": "hbm", "achieved": nb / t_mean / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                "frac": nb / t_mean / 1e6 / HBM_PEAK_GBS, "algorithmic_bytes": nb,
                                "traffic_from_profiles": read_traffic("prefill_grouped_cfg3_pmc.txt") if pw.name.startswith("cfg3") and not args.length else None}}

    tree = None
    if do_verify and args.only == "all":
        # next row of the scope (not part of the step): tree-structured verify, 64 speculated tokens / 42
        # sequence candidates on the same 1024 heads; each call takes a state set of its own and every batch row
        # accepts one root path, so the whole state is written back as in the chain case
        tw = workloads.CONFIGS["tree_verify_64x42"]
        n_nodes, n_leaves = tw.draft_k
        parent = torch.from_numpy(workloads.candidate_tree(n_nodes, n_leaves, tw.seed)).to(dev)
        tq, tk, tv = (torch.from_numpy(a).to(torch.bfloat16).to(dev) for a in workloads.draft_block(tw, n_nodes))
        tout = torch.empty_like(tq)
        accept = torch.from_numpy(((np.arange(tw.B) * 7) % n_nodes).astype(np.int32)).to(dev)
        ev3 = []
        for i in range(10 + min(args.steps, 50)):
            S, z, h = states[i % len(states)]
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            binding.linattn_verify_tree(vdesc, n_nodes, tq, tk, tv, parent, vwts, S, z, h, accept, tout, stream)
            e1.record(stream)
            if i >= 10:
                ev3.append((e0, e1))
        stream.synchronize()
        t_us = [a.elapsed_time(b) * 1e3 for a, b in ev3]
        heads = tw.B * tw.H
        nb = heads * ((tw.d * tw.d + tw.d) * 8 + n_nodes * tw.d * 8 + (tw.conv_k - 1) * tw.d * 4)
        t_mean = sum(t_us) / len(t_us)
        tree = {"workload": f"{tw.name}: B{tw.B} H{tw.H} d{tw.d}, {n_nodes} candidates, {n_leaves} root-to-leaf paths, "
                            "every row accepts one path",
                "us": {"mean": t_mean, "min": min(t_us)},
                "roofline": {"bound": "hbm", "achieved": nb / t_mean / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": nb / t_mean / 1e3 / HBM_PEAK_GBS, "algorithmic_bytes": nb,
                             "traffic_from_profiles": read_traffic("tree_verify_64x42_pmc.txt")}}

    gdecode = None
    if do_verify and args.only == "all":
        # generation with the three-branch form (not part of the step): one token, then eight drafts, per head on the
        # same 1024 heads, every open group half full (32 of 64 rows) when a measurement starts; each call takes a
        # state set of its own and keeps its tokens, so the groups grow each time a set comes round again
        fill0 = 32
        wins = [(torch.randn((vw.B, vw.H, 64, vw.d), generator=g, device=dev).to(torch.bfloat16),
                 torch.randn((vw.B, vw.H, 64, vw.d), generator=g, device=dev).to(torch.bfloat16),
                 torch.full((vw.B, vw.H), fill0, dtype=torch.int32, device=dev)) for _ in states]
        gdesc = binding.make_desc(vw.B, vw.H, vw.d, vw.conv_k, 64, torch.bfloat16, L=1)
        gdecode = {}
        for key, kk in (("k1", 1), ("k8", 8)):
            for _, _, fl in wins:
                fl.fill_(fill0)
            dq, dk, dv, o = drafts[kk]
            ev5, nb_total = [], 0
            n_warm, n_timed = 10, min(args.steps, 50)
            for i in range(n_warm + n_timed):
                S, z, h = states[i % len(states)]
                kw, vwn, fl = wins[i % len(states)]
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                binding.linattn_verify_grouped(gdesc, kk, 1.0, dq, dk, dv, vwts, S, z, h, kw, vwn, fl, None, o, stream)
                e1.record(stream)
                if i >= n_warm:
                    ev5.append((e0, e1))
                    rows_in_use = fill0 + kk * (i // len(states))
                    # read: S, z, the rows in use of both windows, q k v, history, taps, count; write: out, the new rows, history, count
                    nb_total += vw.B * vw.H * ((vw.d * vw.d + vw.d) * 4 + 2 * rows_in_use * vw.d * 2 + 3 * kk * vw.d * 2 + kk * vw.d * 2
                                             + 2 * kk * vw.d * 2 + 2 * (vw.conv_k - 1) * vw.d * 2 + vw.conv_k * vw.d * 4 + 8)
            stream.synchronize()
            t_us = [a.elapsed_time(b) * 1e3 for a, b in ev5]
            t_mean = sum(t_us) / len(t_us)
            nb = nb_total / len(t_us)
            gdecode[key] = {"workload": f"B{vw.B} H{vw.H} d{vw.d} bf16, {kk} token(s) per head, all kept, open groups {fill0}+ of 64 rows, "
                                        "completed-group state from the 2048-token prefix of cfg4, alpha 1",
                            "kernel": "verify_grouped_kernel (vector ALUs)" if kk < 4 else "verify_grouped_mfma_kernel",
                            "us": {"mean": t_mean, "median": float(np.median(t_us)), "min": min(t_us)},
                            "roofline": {"bound": "hbm", "achieved": nb / t_mean / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                         "frac": nb / t_mean / 1e3 / HBM_PEAK_GBS, "algorithmic_bytes": nb,
                                         "traffic_from_profiles": read_traffic(f"verify_grouped_cfg4_{key}_pmc.txt")}}

    side = None
    if args.only == "all" and not args.length:
        # the other prefill workloads (not part of the step): configs 1, 2 and 5, head-major as the parity tests
        # run them, two input sets each (config 2's 25 MB would otherwise be served from the last-level cache)
        side = {}
        for name in ("cfg1_fp32_tiny", "cfg2_gpt2_small", "cfg5_long_context"):
            wl = workloads.CONFIGS[name]
            sdt = workloads.torch_dtype(wl.io_dtype)
            gs = torch.Generator(device=dev).manual_seed(wl.seed)
            sets = []
            for _ in range(2 if name != "cfg2_gpt2_small" else 16):
                q, k, v = ((torch.randn((wl.B, wl.H, wl.L, wl.d), generator=gs, device=dev) * wl.scale).to(sdt) for _ in range(3))
                sets.append((q, k, v, torch.empty_like(q)))
            swts = torch.from_numpy(workloads.conv_weights(np.random.default_rng(wl.seed), wl.H, wl.d, wl.conv_k)).to(dev)
            sdesc = binding.make_desc(wl.B, wl.H, wl.d, wl.conv_k, wl.chunk, sdt, L=wl.L)
            sws_bytes = binding.linattn_workspace_bytes(sdesc, wl.L)
            sws = torch.empty(max(sws_bytes, 16), dtype=torch.uint8, device=dev)
            sS = torch.empty((wl.B, wl.H, wl.d, wl.d), device=dev)
            sz = torch.empty((wl.B, wl.H, wl.d), device=dev)
            sh = torch.empty((wl.B, wl.H, wl.conv_k - 1, wl.d), device=dev, dtype=sdt)
            evs = []
            n_warm, n_timed = 20, min(max(args.steps, 20), 50)
            for i in range(n_warm + n_timed):
                q, k, v, out = sets[i % len(sets)]
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                binding.linattn_prefill(sdesc, wl.L, q, k, v, swts, None, None, None, out, sS, sz, sh, sws, sws_bytes, stream)
                e1.record(stream)
                if i >= n_warm:
                    evs.append((e0, e1))
            stream.synchronize()
            t_ms = [a.elapsed_time(b) for a, b in evs]
            t_mean = sum(t_ms) / len(t_ms)
            esz = 4 if wl.io_dtype == "f32" else 2
            nb = 4 * wl.B * wl.H * wl.L * wl.d * esz
            side[name] = {"workload": f"B{wl.B} H{wl.H} L{wl.L} d{wl.d} {wl.io_dtype} chunk{wl.chunk} Kc{wl.conv_k}, head-major",
                          "ms": {"mean": t_mean, "median": float(np.median(t_ms)), "min": min(t_ms)},
                          "tokens_per_s": wl.B * wl.L / (t_mean * 1e-3), "workspace_bytes": sws_bytes,
                          "roofline": {"bound": "hbm", "achieved": nb / t_mean / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                       "frac": nb / t_mean / 1e6 / HBM_PEAK_GBS, "algorithmic_bytes": nb,
                                       "traffic_from_profiles": read_traffic(TRAFFIC_FILES.get(name, ""))}}
            del sets, sws, sS, sz, sh
        torch.cuda.empty_cache()

    flash = None
    if args.only == "all" and not args.length:
        # next row of the scope (not part of the step): the sizes of the paper's FLASH experiment -- 63-tap masked
        # DWConv, groups of 256 tokens, batch 1, 1K / 4K / 8K tokens, as eight heads of 128.  Token-level form
        # (matrix-core attention kernel + the long-convolution pass) and the three-branch form in groups of 256
        # (its own matrix-core kernel + the same long-convolution pass).  Eight heads cannot fill the chip: these
        # are latency figures, a few launches of some tens of microseconds each.  The last row is the same layer on a
        # batch of eight sequences (2048 groups): the size at which the chip, not the launch chain, is the bound.
        flash = {}
        for name in ("flash_L1024", "flash_L4096", "flash_L8192", "flash_B8_L8192"):
            wl = workloads.CONFIGS[name]
            few = wl.B > 1                                  # the batch row: milliseconds per call, fewer of them
            gs = torch.Generator(device=dev).manual_seed(wl.seed)
            q, k, v = ((torch.randn((wl.B, wl.H, wl.L, wl.d), generator=gs, device=dev) * wl.scale).to(torch.bfloat16) for _ in range(3))
            out = torch.empty_like(q)
            fw = torch.from_numpy(workloads.conv_weights(np.random.default_rng(wl.seed), wl.H, wl.d, wl.conv_k)).to(dev)
            fdesc = binding.make_desc(wl.B, wl.H, wl.d, wl.conv_k, wl.chunk, torch.bfloat16, L=wl.L)
            fws_bytes = binding.linattn_workspace_bytes(fdesc, wl.L)
            fws = torch.empty(max(fws_bytes, 16), dtype=torch.uint8, device=dev)
            fS = torch.empty((wl.B, wl.H, wl.d, wl.d), device=dev)
            fz = torch.empty((wl.B, wl.H, wl.d), device=dev)
            fh = torch.empty((wl.B, wl.H, wl.conv_k - 1, wl.d), device=dev, dtype=torch.bfloat16)
            nb = 4 * wl.B * wl.H * wl.L * wl.d * 2
            row = {"workload": f"B{wl.B} H{wl.H} L{wl.L} d{wl.d} bf16, groups of {wl.chunk}, Kc{wl.conv_k}, head-major"}
            for key, n_warm, n_timed, call in (
                    ("token_level", 5 if few else 10, 10 if few else 30, lambda: binding.linattn_prefill(fdesc, wl.L, q, k, v, fw, None, None, None, out, fS, fz, fh, fws, fws_bytes, stream)),
                    ("three_branch", 5 if few else 10, 10 if few else 30, lambda: binding.linattn_prefill_grouped(fdesc, wl.L, 1.0, q, k, v, fw, None, None, None, out, fS, fz, fh, fws, fws_bytes, stream))):
                evs = []
                for i in range(n_warm + n_timed):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                    call()
                    e1.record(stream)
                    if i >= n_warm:
                        evs.append((e0, e1))
                stream.synchronize()
                t_ms = [a.elapsed_time(b) for a, b in evs]
                t_mean = sum(t_ms) / len(t_ms)
                row[key] = {"ms": {"mean": t_mean, "min": min(t_ms)}, "tokens_per_s": wl.B * wl.L / (t_mean * 1e-3),
                            "roofline": {"bound": "hbm", "achieved": nb / t_mean / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                         "frac": nb / t_mean / 1e6 / HBM_PEAK_GBS, "algorithmic_bytes": nb}}
            # the training direction of the same shape (Sec. 5.3 times forward + backward): gradient of the three-branch
            # form, dout seeded; algorithmic bytes = q, k, v, dout read, dq, dk, dv written
            dout = torch.randn((wl.B, wl.H, wl.L, wl.d), generator=gs, device=dev).to(torch.bfloat16)
            dq, dk, dv = (torch.empty_like(q) for _ in range(3))
            dw = torch.empty_like(fw)
            bws_bytes = binding.linattn_backward_workspace_bytes(fdesc, wl.L)
            bws = torch.empty(max(bws_bytes, 16), dtype=torch.uint8, device=dev)
            evs = []
            bwarm, btimed = (5, 10) if few else (10, 30)
            for i in range(bwarm + btimed):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                binding.linattn_prefill_grouped_backward(fdesc, wl.L, 1.0, q, k, v, fw, dout, dq, dk, dv, dw, bws, bws_bytes, stream)
                e1.record(stream)
                if i >= bwarm:
                    evs.append((e0, e1))
            stream.synchronize()
            t_ms = [a.elapsed_time(b) for a, b in evs]
            t_mean = sum(t_ms) / len(t_ms)
            nbb = 7 * wl.B * wl.H * wl.L * wl.d * 2
            row["three_branch_backward"] = {"ms": {"mean": t_mean, "min": min(t_ms)}, "tokens_per_s": wl.B * wl.L / (t_mean * 1e-3),
                                            "workspace_bytes": bws_bytes,
                                            "roofline": {"bound": "hbm", "achieved": nbb / t_mean / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                                         "frac": nbb / t_mean / 1e6 / HBM_PEAK_GBS, "algorithmic_bytes": nbb}}
            row["training_step_ms"] = row["three_branch"]["ms"]["mean"] + t_mean
            flash[name] = row
            del q, k, v, out, fws, dout, dq, dk, dv, bws
        torch.cuda.empty_cache()

    wide = None
    if args.only == "all" and not args.length:
        # next row of the scope (not part of the step): value rows wider than key rows, d_k 64 / d_v 128 on the
        # LLaMA layer shape -- prefill (two value blocks per head on the matrix-core kernel, q and k read by both)
        # and an 8-draft verify step (streaming kernel: column slices of the 64 x 128 state)
        wide = {}
        wl = workloads.CONFIGS["wide_values_prefill"]
        gs = torch.Generator(device=dev).manual_seed(wl.seed)
        sets = []
        for _ in range(2):
            q, k = ((torch.randn((wl.B, wl.H, wl.L, wl.d), generator=gs, device=dev) * wl.scale).to(torch.bfloat16) for _ in range(2))
            v = (torch.randn((wl.B, wl.H, wl.L, wl.d_v), generator=gs, device=dev) * wl.scale).to(torch.bfloat16)
            sets.append((q, k, v, torch.empty_like(v)))
        ww = torch.from_numpy(workloads.conv_weights(np.random.default_rng(wl.seed), wl.H, wl.d_v, wl.conv_k)).to(dev)
        wdesc = binding.make_desc(wl.B, wl.H, wl.d, wl.conv_k, wl.chunk, torch.bfloat16, L=wl.L, d_v=wl.d_v)
        wS = torch.empty((wl.B, wl.H, wl.d, wl.d_v), device=dev)
        wz = torch.empty((wl.B, wl.H, wl.d), device=dev)
        wh = torch.empty((wl.B, wl.H, wl.conv_k - 1, wl.d_v), device=dev, dtype=torch.bfloat16)
        evs = []
        for i in range(20 + 30):
            q, k, v, out = sets[i % 2]
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            binding.linattn_prefill(wdesc, wl.L, q, k, v, ww, None, None, None, out, wS, wz, wh, None, 0, stream)
            e1.record(stream)
            if i >= 20:
                evs.append((e0, e1))
        stream.synchronize()
        t_ms = [a.elapsed_time(b) for a, b in evs]
        t_mean = sum(t_ms) / len(t_ms)
        nb = wl.B * wl.H * wl.L * (2 * wl.d + 2 * wl.d_v) * 2
        wide["prefill"] = {"workload": f"B{wl.B} H{wl.H} L{wl.L} d_k{wl.d} d_v{wl.d_v} bf16 chunk{wl.chunk} Kc{wl.conv_k}, head-major",
                           "ms": {"mean": t_mean, "median": float(np.median(t_ms)), "min": min(t_ms)},
                           "tokens_per_s": wl.B * wl.L / (t_mean * 1e-3),
                           "roofline": {"bound": "hbm", "achieved": nb / t_mean / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                        "frac": nb / t_mean / 1e6 / HBM_PEAK_GBS, "algorithmic_bytes": nb}}
        del sets
        if do_verify:
            vwl = workloads.CONFIGS["wide_values_verify"]
            kk = 8
            wstates = [(torch.randn((vwl.B, vwl.H, vwl.d, vwl.d_v), generator=gs, device=dev) * 50.0,
                        torch.rand((vwl.B, vwl.H, vwl.d), generator=gs, device=dev) * 100.0 + 1900.0,
                        torch.randn((vwl.B, vwl.H, vwl.conv_k - 1, vwl.d_v), generator=gs, device=dev).to(torch.bfloat16))
                       for _ in range(args.state_sets)]
            dq, dk = (torch.randn((vwl.B, vwl.H, kk, vwl.d), generator=gs, device=dev).to(torch.bfloat16) for _ in range(2))
            dv = torch.randn((vwl.B, vwl.H, kk, vwl.d_v), generator=gs, device=dev).to(torch.bfloat16)
            do = torch.empty_like(dv)
            vdesc2 = binding.make_desc(vwl.B, vwl.H, vwl.d, vwl.conv_k, 64, torch.bfloat16, L=kk, d_v=vwl.d_v)
            evs = []
            for i in range(10 + 40):
                S, z, h = wstates[i % len(wstates)]
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                binding.linattn_verify(vdesc2, kk, dq, dk, dv, ww, S, z, h, None, do, stream)
                e1.record(stream)
                if i >= 10:
                    evs.append((e0, e1))
            stream.synchronize()
            t_us = [a.elapsed_time(b) * 1e3 for a, b in evs]
            t_mean = sum(t_us) / len(t_us)
            heads = vwl.B * vwl.H
            nb = heads * ((vwl.d * vwl.d_v + vwl.d) * 8 + kk * (2 * vwl.d + 2 * vwl.d_v) * 2 + (vwl.conv_k - 1) * vwl.d_v * 4)
            wide["verify_k8"] = {"workload": f"B{vwl.B} H{vwl.H} d_k{vwl.d} d_v{vwl.d_v} bf16, 8 drafts, all kept, synthetic state of the "
                                             "magnitude a 2048-token prefix leaves",
                                 "us": {"mean": t_mean, "median": float(np.median(t_us)), "min": min(t_us)},
                                 "roofline": {"bound": "hbm", "achieved": nb / t_mean / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                              "frac": nb / t_mean / 1e3 / HBM_PEAK_GBS, "algorithmic_bytes": nb}}
            del wstates
        torch.cuda.empty_cache()

    copy_ref = None
    if args.only == "all":
        # for reference (not a kernel of the library): what a plain elementwise kernel reaches on this GPU, reading
        # 1 GiB and writing 1 GiB per launch over rotating buffers -- the practical ceiling under the published peak
        with torch.cuda.stream(stream):
            bufs = [torch.zeros(1 << 28, dtype=torch.float32, device=dev) for _ in range(4)]
            evs = []
            for i in range(5 + 20):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                torch.add(bufs[i % 4], 1.0, out=bufs[(i + 1) % 4])
                e1.record(stream)
                if i >= 5:
                    evs.append((e0, e1))
        stream.synchronize()
        t_ms = [a.elapsed_time(b) for a, b in evs]
        t_mean = sum(t_ms) / len(t_ms)
        copy_ref = {"kernel": "torch.add(x, 1, out=y), 1 GiB read + 1 GiB written per launch", "ms": {"mean": t_mean, "min": min(t_ms)},
                    "achieved": 2 * (1 << 30) / t_mean / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": 2 * (1 << 30) / t_mean / 1e6 / HBM_PEAK_GBS}
        del bufs
        torch.cuda.empty_cache()

    timed_ms = {n: [a.elapsed_time(b) for a, b in lst[n_settled[n]:]] for n, lst in ev.items() if len(lst) > n_settled[n]}
    mean_ms = {n: sum(t) / len(t) for n, t in timed_ms.items()}
    min_ms = {n: min(t) for n, t in timed_ms.items()}
    med_ms = {n: float(np.median(t)) for n, t in timed_ms.items()}

    result = {
        "metric": "linear-attn prefill tokens/s (LLaMA-7B layer shape) + spec-verify step us, % roofline",
        "value": None, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "settle_steps": settle_steps,
        "settle": {"kernel": settle_name, "rule": f"untimed steps in windows of {SETTLE_WINDOW} until every duration of a window lies within 5 % "
                                                  f"of its median and the medians of four windows in a row within 1 % of each other (at most {SETTLE_CAP})",
                   "unsettled_ms": {"first": settle_hist[0], "max": max(settle_hist), "mean_first_window": float(np.mean(settle_hist[:SETTLE_WINDOW]))},
                   "settled_window_ms": float(np.median(settle_hist[-SETTLE_WINDOW:])),
                   "window_medians_ms": [float(np.median(settle_hist[i:i + SETTLE_WINDOW])) for i in range(0, len(settle_hist), SETTLE_WINDOW)]},
        "telemetry": telemetry,
        "ms_per_step": wall_ms / args.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{pw.name} B{pw.B} H{pw.H} L{pw.L} d{pw.d} bf16 chunk{pw.chunk} Kc{pw.conv_k} (prefill) + "
                               "cfg4_llama7b_verify B32 H32 d128 fp32-state k=8,4,1 (verify/decode)",
                   "step": "prefill + verify k=8 + verify k=4 + decode", "only": args.only,
                   "layout": {"blhd": "q,k,v,out token-major [B,L,H,d]", "bhld": "q,k,v,out head-major [B,H,L,d]"}[args.layout]},
    }
    if do_prefill:
        t = mean_ms["prefill"] * 1e-3
        nbytes = prefill_bytes(pw)
        fc, fd = prefill_flops(pw)
        result["value"] = pw.B * pw.L / t
        result["prefill_ms"] = {"mean": mean_ms["prefill"], "median": med_ms["prefill"], "min": min_ms["prefill"]}
        if other_layout_ms:
            result["prefill_ms_other_layout"] = other_layout_ms
        if grouped:
            result["prefill_grouped"] = grouped
        result["roofline"] = {"bound": "hbm", "achieved": nbytes / t / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": nbytes / t / 1e9 / HBM_PEAK_GBS,
                              "traffic_from_profiles": read_traffic(TRAFFIC_FILES.get(pw.name, "")) if not args.length else None,
                              "kernel": "prefill_mfma_ws_kernel (+ state-only pass and scan when the sequence is segmented)",
                              "algorithmic_bytes": nbytes, "workspace_bytes": ws_bytes}
        result["mfma"] = {"tflops_causal": fc / t / 1e12, "tflops_dense_tiles": fd / t / 1e12,
                          "peak": MFMA_BF16_PEAK_TFLOPS, "frac_causal": fc / t / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                          "frac_dense_tiles": fd / t / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                          "note": "HBM-bound op: at d=128, chunk 64 it moves 1024 B for <= 98304 flop per head-token, so "
                                  "the HBM roof caps the MFMA fraction near 0.31"}
    if do_verify:
        us = {}
        roof = {}
        for name, kk in (("verify8", 8), ("verify4", 4), ("decode", 1)):
            t = mean_ms[name] * 1e-3
            nb = verify_bytes(vw, kk)
            us[f"k{kk}"] = {"mean": mean_ms[name] * 1e3, "median": med_ms[name] * 1e3, "min": min_ms[name] * 1e3}
            roof[f"k{kk}"] = {"bound": "hbm", "achieved": nb / t / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": nb / t / 1e9 / HBM_PEAK_GBS, "algorithmic_bytes": nb,
                              "traffic_from_profiles": read_traffic(f"verify_cfg4_k{kk}_pmc.txt")}
        result["verify_us_per_step"] = us
        result["roofline_verify"] = roof
        if tree:
            result["tree_verify"] = tree
        if gdecode:
            result["verify_grouped"] = gdecode
        if not do_prefill:
            result["value"] = us["k8"]["mean"]
            result["unit"] = "us/step (verify k=8)"
            result["higher_is_better"] = False
    if side:
        result["other_configs"] = side
    if flash:
        result["flash_shape"] = flash
    if wide:
        result["wide_values"] = wide
    if copy_ref:
        result["hbm_copy_reference"] = copy_ref
    if not args.no_cpu_baseline and do_prefill:
        result["cpu_baseline"] = cpu_baseline(pw, args.cpu_seconds)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
