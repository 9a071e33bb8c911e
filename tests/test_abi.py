"""The C-ABI library: loads, exports what the header declares, refuses bad arguments.

Runs without a GPU: every call made here is rejected by validation before anything
could be enqueued.
"""
import ctypes
import os
import re

import pytest

from paper_2406_07368_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = open(os.path.join(ROOT, "include", "linattn.h")).read()
P = 0x10000  # a 16-byte aligned non-null fake device address; never dereferenced on these paths


def declared_symbols():
    code = re.sub(r"/\*.*?\*/", "", HEADER, flags=re.S)
    return sorted(set(re.findall(r"\b(linattn_[a-z_0-9]+)\s*\(", code)))


def test_header_symbols_are_exported():
    lib = binding.load()
    names = declared_symbols()
    assert set(names) == set(binding.SYMBOLS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings():
    assert binding.load().linattn_version() >= 100
    seen = {binding.status_string(s) for s in range(8)}
    assert len(seen) == 8 and binding.status_string(0) == "ok"
    assert binding.status_string(99) == "unknown status"


def test_wait_limit_setting_round_trips():
    lib = binding.load()
    assert lib.linattn_set_wait_limit(5) == 1 << 20
    assert lib.linattn_set_wait_limit(-1) == 5
    assert lib.linattn_set_wait_limit(0) == -1          # 0 restores the default
    assert lib.linattn_set_wait_limit(0) == 1 << 20


def good_desc(**kw):
    d = binding.make_desc(2, 4, 128, 3, 64, L=256)
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def prefill_status(desc, L=256, **over):
    lib = binding.load()
    a = dict(q=P, k=P, v=P, conv_w=P, S_in=None, z_in=None, hist_in=None, out=P, S_out=P, z_out=P, hist_out=P,
             ws=P, ws_bytes=1 << 40)
    a.update(over)
    return lib.linattn_prefill(ctypes.byref(desc) if desc is not None else None, L, a["q"], a["k"], a["v"],
                               a["conv_w"], a["S_in"], a["z_in"], a["hist_in"], a["out"], a["S_out"], a["z_out"],
                               a["hist_out"], a["ws"], a["ws_bytes"], None)


@pytest.mark.parametrize("field,value,status", [
    ("d", 96, 2), ("d", 0, 2), ("B", 0, 2), ("H", -1, 2), ("conv_k", 0, 2), ("conv_k", 64, 2),
    ("chunk", 32, 2), ("stride_t", (1 << 22) + 8, 2), ("io_dtype", 7, 3), ("phi", 2, 3), ("eps", -1.0, 2), ("eps", float("nan"), 2),
    ("stride_t", 64, 2), ("stride_t", 132, 2), ("stride_h", 12, 2),
])
def test_prefill_rejects_bad_descriptor(field, value, status):
    assert prefill_status(good_desc(**{field: value})) == status


def test_prefill_rejects_bad_pointers_and_sizes():
    d = good_desc()
    assert prefill_status(None) == 1
    assert prefill_status(d, L=-1) == 2
    assert prefill_status(d, q=None) == 1
    assert prefill_status(d, conv_w=None) == 1
    assert prefill_status(d, out=None) == 1
    assert prefill_status(d, v=P + 8) == 4
    assert prefill_status(d, S_out=P + 4) == 4
    # the incoming state is all-or-nothing
    assert prefill_status(d, S_in=P) == 1
    assert prefill_status(d, S_in=P, z_in=P) == 1


def test_workspace_is_constant_in_L_and_checked():
    lib = binding.load()
    d = binding.make_desc(1, 32, 128, 5, 128, L=65536)
    sizes = [binding.linattn_workspace_bytes(d, L) for L in (8192, 16384, 32768, 65536)]
    assert len(set(sizes)) == 1, sizes
    per_state = (128 * 128 + 128) * 4
    # at most 64 segment start states per (b, h) plus 8 staged history rows
    assert 0 < sizes[0] <= 32 * (64 * per_state + 8 * 128 * 2)
    if sizes[0]:
        assert prefill_status(d, L=65536, ws=None, ws_bytes=0) == 6
        assert prefill_status(d, L=65536, ws=P, ws_bytes=sizes[0] - 1) == 6
    bad = binding.make_desc(1, 32, 96, 5, 128, L=65536)
    assert lib.linattn_workspace_bytes(ctypes.byref(bad), 65536) == 0


def grouped_status(desc, L=256, alpha=1.0, **over):
    lib = binding.load()
    a = dict(q=P, k=P, v=P, conv_w=P, S_in=None, z_in=None, hist_in=None, out=P, S_out=P, z_out=P, hist_out=P,
             ws=P, ws_bytes=1 << 40)
    a.update(over)
    return lib.linattn_prefill_grouped(ctypes.byref(desc) if desc is not None else None, L, alpha, a["q"], a["k"], a["v"],
                                       a["conv_w"], a["S_in"], a["z_in"], a["hist_in"], a["out"], a["S_out"], a["z_out"],
                                       a["hist_out"], a["ws"], a["ws_bytes"], None)


def test_prefill_grouped_rejects_bad_arguments():
    d = good_desc()
    assert grouped_status(None) == 1
    assert grouped_status(d, L=-1) == 2
    assert grouped_status(d, alpha=float("nan")) == 2
    assert grouped_status(d, alpha=float("inf")) == 2
    assert grouped_status(d, k=None) == 1
    assert grouped_status(d, out=P + 8) == 4
    assert grouped_status(d, S_in=P) == 1
    assert grouped_status(good_desc(chunk=128)) == 5                        # the group is part of the result: 64 or 256
    assert grouped_status(good_desc(chunk=256, io_dtype=binding.LINATTN_F32)) == 5   # fp32 rows of 128 in groups of 256: no kernel
    assert grouped_status(good_desc(conv_k=64)) == 2
    assert grouped_status(good_desc(chunk=32)) == 2
    few = binding.make_desc(1, 2, 128, 3, 64, L=4096)                       # segmented: needs the workspace
    assert binding.linattn_workspace_bytes(few, 4096) > 0
    assert grouped_status(few, L=4096, ws=None, ws_bytes=0) == 6


def backward_status(desc, L=256, alpha=1.0, **over):
    lib = binding.load()
    a = dict(q=P, k=P, v=P, conv_w=P, dout=P, dq=P, dk=P, dv=P, dw=P, ws=P, ws_bytes=1 << 40)
    a.update(over)
    return lib.linattn_prefill_grouped_backward(ctypes.byref(desc) if desc is not None else None, L, alpha, a["q"], a["k"],
                                                a["v"], a["conv_w"], a["dout"], a["dq"], a["dk"], a["dv"], a["dw"], a["ws"],
                                                a["ws_bytes"], None)


def test_prefill_grouped_backward_rejects_bad_arguments():
    d = good_desc(chunk=256)
    assert backward_status(None) == 1
    assert backward_status(d, L=-1) == 2
    assert backward_status(d, alpha=float("nan")) == 2
    assert backward_status(d, dout=None) == 1
    assert backward_status(d, dk=None) == 1
    assert backward_status(d, conv_w=None) == 1
    assert backward_status(d, dq=P + 8) == 4
    assert backward_status(d, dw=P + 4) == 4
    assert backward_status(good_desc(chunk=128)) == 5                       # groups of 64 or 256
    assert backward_status(good_desc(io_dtype=binding.LINATTN_F32)) == 5    # bf16 rows only
    assert backward_status(binding.make_desc(2, 4, 64, 3, 64, L=256, d_v=128)) == 5   # d_v = d only
    assert backward_status(good_desc(conv_k=64)) == 2
    need = binding.linattn_backward_workspace_bytes(d, 256)
    assert need > 2 * 2 * 4 * (128 * 128 + 128) * 4                         # two slots per group and head, and more
    assert backward_status(d, ws=None, ws_bytes=0) == 6
    assert backward_status(d, ws_bytes=need - 1) == 6
    assert binding.linattn_backward_workspace_bytes(good_desc(io_dtype=binding.LINATTN_F32), 256) == 0
    # the size grows with the number of groups, not faster
    assert binding.linattn_backward_workspace_bytes(d, 2560) < 11 * need


def vgrouped_status(desc, kk=4, alpha=1.0, **over):
    lib = binding.load()
    a = dict(q=P, k=P, v=P, conv_w=P, S=P, z=P, hist=P, kwin=P, vwin=P, fill=P, n_commit=None, out=P)
    a.update(over)
    return lib.linattn_verify_grouped(ctypes.byref(desc) if desc is not None else None, kk, alpha, a["q"], a["k"], a["v"],
                                      a["conv_w"], a["S"], a["z"], a["hist"], a["kwin"], a["vwin"], a["fill"],
                                      a["n_commit"], a["out"], None)


def test_verify_grouped_rejects_bad_arguments():
    d = good_desc()
    assert vgrouped_status(None) == 1
    assert vgrouped_status(d, kk=0) == 2
    assert vgrouped_status(d, kk=17) == 2
    assert vgrouped_status(d, alpha=float("nan")) == 2
    assert vgrouped_status(d, kwin=None) == 1
    assert vgrouped_status(d, fill=None) == 1
    assert vgrouped_status(d, hist=None) == 1
    assert vgrouped_status(d, vwin=P + 8) == 4
    assert vgrouped_status(d, fill=P + 2) == 4
    assert vgrouped_status(d, n_commit=P + 1) == 4
    assert vgrouped_status(good_desc(chunk=128)) == 5           # the window is one group of 64 rows
    assert vgrouped_status(good_desc(d=96)) == 2
    assert vgrouped_status(good_desc(conv_k=9)) == 2


def verify_status(desc, kk=4, **over):
    lib = binding.load()
    a = dict(q=P, k=P, v=P, conv_w=P, S=P, z=P, hist=P, n_commit=None, out=P)
    a.update(over)
    return lib.linattn_verify(ctypes.byref(desc) if desc is not None else None, kk, a["q"], a["k"], a["v"],
                              a["conv_w"], a["S"], a["z"], a["hist"], a["n_commit"], a["out"], None)


def test_verify_rejects_bad_arguments():
    d = good_desc()
    assert verify_status(None) == 1
    assert verify_status(d, kk=0) == 2
    assert verify_status(d, kk=17) == 2
    assert verify_status(d, S=None) == 1
    assert verify_status(d, hist=None) == 1
    assert verify_status(d, z=P + 4) == 4
    assert verify_status(d, n_commit=P + 2) == 4
    assert verify_status(good_desc(d=32)) == 2
    assert verify_status(good_desc(conv_k=9)) == 2              # kernels of more than 8 taps: prefill entry points only
    lib = binding.load()
    assert lib.linattn_decode(ctypes.byref(d), P, None, P, P, P, P, P, P, None) == 1


def tree_status(desc, n=8, **over):
    lib = binding.load()
    a = dict(q=P, k=P, v=P, parent=P, conv_w=P, S=P, z=P, hist=P, accept=None, out=P)
    a.update(over)
    return lib.linattn_verify_tree(ctypes.byref(desc) if desc is not None else None, n, a["q"], a["k"], a["v"],
                                   a["parent"], a["conv_w"], a["S"], a["z"], a["hist"], a["accept"], a["out"], None)


def test_verify_tree_rejects_bad_arguments():
    d = good_desc()
    assert tree_status(None) == 1
    assert tree_status(d, n=0) == 2
    assert tree_status(d, n=65) == 2
    assert tree_status(d, parent=None) == 1
    assert tree_status(d, hist=None) == 1
    assert tree_status(d, S=P + 8) == 4
    assert tree_status(d, parent=P + 2) == 4
    assert tree_status(d, accept=P + 1) == 4
    assert tree_status(binding.make_desc(2, 4, 64, 3, 64, L=8, d_v=128)) == 5   # d_v = d only
    assert tree_status(good_desc(d=96)) == 2
    assert tree_status(good_desc(conv_k=63)) == 2


def test_binding_raises_on_refusal():
    with pytest.raises(binding.LinattnError) as ei:
        binding.linattn_verify(good_desc(), 0, P, P, P, P, P, P, P, None, P, stream=0)
    assert ei.value.status == 2
