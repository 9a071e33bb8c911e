"""Calls on several HIP streams at once: the library keeps nothing between calls and owns no buffers, so calls that
work on different buffers may overlap freely and must give what they give one after the other."""
import numpy as np
import pytest
import torch

from parity import dev
from paper_2406_07368_amd import binding, workloads

pytestmark = pytest.mark.gpu
BF = torch.bfloat16


def test_calls_on_four_streams_overlap_without_interfering():
    B, H, d, Kc, L = 2, 16, 128, 3, 700
    rng = np.random.default_rng(81)
    gw = dev(workloads.conv_weights(rng, H, d, Kc))
    jobs = []
    for i in range(4):
        q, k, v = (dev(workloads.round_to_io(rng.standard_normal((B, H, L, d)), "bf16"), BF) for _ in range(3))
        dq, dk, dv = (dev(workloads.round_to_io(rng.standard_normal((B, H, 6, d)), "bf16"), BF) for _ in range(3))
        jobs.append((q, k, v, dq, dk, dv))

    def run(job, stream):
        """a segmented prefill, a chain verify on its state, a three-branch prefill and a generation step on that"""
        q, k, v, dq, dk, dv = job
        out, st = binding.prefill(q, k, v, gw, stream=stream)
        vo = binding.verify(dq, dk, dv, gw, st, stream=stream)
        gout, gst = binding.prefill_grouped(q[:, :, :640].contiguous(), k[:, :, :640].contiguous(), v[:, :, :640].contiguous(), gw,
                                            0.9, stream=stream)
        gs = binding.grouped_state(B, H, d, Kc, BF, prefill_state=gst)
        go = binding.verify_grouped(dq, dk, dv, gw, gs, 0.9, stream=stream)
        return [out, vo, gout, go, *st, *gs]

    torch.cuda.synchronize()
    want = [run(job, torch.cuda.current_stream()) for job in jobs]      # one after the other
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in jobs]
    got = []
    for _ in range(3):                                                    # several rounds, all four in flight together
        got = []
        for job, s in zip(jobs, streams):
            with torch.cuda.stream(s):
                got.append(run(job, s))
        torch.cuda.synchronize()
        for a_list, b_list in zip(got, want):
            for a, b in zip(a_list, b_list):
                assert torch.equal(a, b)


def test_gradient_calls_from_two_streams_and_two_host_threads():
    """The gradient forks part of its work to a stream of the library's own (one per host thread and device) and joins it
    before it returns: calls of one thread on two streams share that stream, calls of two threads do not, and all give
    the bits that one call after the other gives."""
    import threading
    B, H, d, Kc, L = 2, 4, 128, 63, 1100
    rng = np.random.default_rng(82)
    gw = dev(workloads.conv_weights(rng, H, d, Kc))
    jobs = [tuple(dev(workloads.round_to_io(rng.standard_normal((B, H, L, d)), "bf16"), BF) for _ in range(4)) for _ in range(4)]

    def grad(job, stream):
        q, k, v, dout = job
        return binding.prefill_grouped_backward(q, k, v, gw, dout, 0.9, 1e-3, stream=stream, group=256)

    torch.cuda.synchronize()
    want = [grad(job, torch.cuda.current_stream()) for job in jobs]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in jobs]
    got = [None] * len(jobs)

    def worker(idx):                       # two jobs per thread, each on a stream of its own, three rounds
        for _ in range(3):
            for i in idx:
                with torch.cuda.stream(streams[i]):
                    got[i] = grad(jobs[i], streams[i])
            for i in idx:
                streams[i].synchronize()

    threads = [threading.Thread(target=worker, args=(idx,)) for idx in ((0, 1), (2, 3))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    for a_list, b_list in zip(got, want):
        for a, b in zip(a_list, b_list):
            assert torch.equal(a, b)
