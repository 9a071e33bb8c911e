"""ctypes binding of liblinattn.so: argument marshalling only.

Every call has the name and argument order of its declaration in ``include/linattn.h``.
Tensors are torch tensors on the GPU (torch is used for device memory and
streams, nothing else); every arithmetic step runs inside the library's
kernels.  If the library is missing or a call is refused, this module raises;
there is no other code path.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblinattn.so")
_lib = None

LINATTN_F32, LINATTN_BF16 = 0, 1
LINATTN_PHI_ELU1, LINATTN_PHI_RELU = 0, 1
PHI = {"elu1": LINATTN_PHI_ELU1, "relu": LINATTN_PHI_RELU}
MAX_CONV_K, MAX_CONV_K_PREFILL, MAX_DRAFT, MAX_TREE = 8, 63, 16, 64
SYMBOLS = ("linattn_workspace_bytes", "linattn_prefill", "linattn_prefill_noalloc", "linattn_noalloc_scratch_bytes", "linattn_prefill_grouped", "linattn_backward_workspace_bytes", "linattn_prefill_grouped_backward", "linattn_verify", "linattn_verify_grouped", "linattn_verify_tree", "linattn_decode",
           "linattn_set_wait_limit", "linattn_status_string", "linattn_version")


class LinattnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class Desc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("d", ctypes.c_int32),
                ("conv_k", ctypes.c_int32), ("chunk", ctypes.c_int32), ("io_dtype", ctypes.c_int32),
                ("phi", ctypes.c_int32), ("eps", ctypes.c_float),
                ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_t", ctypes.c_int64),
                ("d_v", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("stride_b_v", ctypes.c_int64), ("stride_h_v", ctypes.c_int64), ("stride_t_v", ctypes.c_int64)]


def load():
    """Load the built library (build it first if it has never been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    dp = ctypes.POINTER(Desc)
    lib.linattn_workspace_bytes.restype = sz
    lib.linattn_workspace_bytes.argtypes = [dp, i32]
    lib.linattn_prefill.restype = ctypes.c_int
    lib.linattn_prefill.argtypes = [dp, i32] + [vp] * 11 + [vp, sz, vp]
    lib.linattn_prefill_noalloc.restype = ctypes.c_int
    lib.linattn_prefill_noalloc.argtypes = [dp, i32] + [vp] * 11 + [vp]
    lib.linattn_noalloc_scratch_bytes.restype = sz
    lib.linattn_noalloc_scratch_bytes.argtypes = []
    lib.linattn_prefill_grouped.restype = ctypes.c_int
    lib.linattn_prefill_grouped.argtypes = [dp, i32, ctypes.c_float] + [vp] * 11 + [vp, sz, vp]
    lib.linattn_backward_workspace_bytes.restype = sz
    lib.linattn_backward_workspace_bytes.argtypes = [dp, i32]
    lib.linattn_prefill_grouped_backward.restype = ctypes.c_int
    lib.linattn_prefill_grouped_backward.argtypes = [dp, i32, ctypes.c_float] + [vp] * 9 + [vp, sz, vp]
    lib.linattn_verify.restype = ctypes.c_int
    lib.linattn_verify.argtypes = [dp, i32] + [vp] * 9 + [vp]
    lib.linattn_verify_grouped.restype = ctypes.c_int
    lib.linattn_verify_grouped.argtypes = [dp, i32, ctypes.c_float] + [vp] * 12 + [vp]
    lib.linattn_verify_tree.restype = ctypes.c_int
    lib.linattn_verify_tree.argtypes = [dp, i32] + [vp] * 10 + [vp]
    lib.linattn_decode.restype = ctypes.c_int
    lib.linattn_decode.argtypes = [dp] + [vp] * 8 + [vp]
    lib.linattn_status_string.restype = ctypes.c_char_p
    lib.linattn_status_string.argtypes = [ctypes.c_int]
    lib.linattn_version.restype = i32
    lib.linattn_set_wait_limit.restype = i32
    lib.linattn_set_wait_limit.argtypes = [i32]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().linattn_status_string(int(status)).decode()


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(status: int, where: str):
    if status != 0:
        raise LinattnError(status, where)


def make_desc(B, H, d, conv_k, chunk=64, io_dtype=torch.bfloat16, eps=0.0, strides=None, L=None, phi="elu1",
              d_v=None, strides_v=None) -> Desc:
    """Descriptor for dense [B,H,L,d] tensors unless ``strides`` (b, h, t) is given.  phi: "elu1" or "relu".
    d_v: width of the value rows when it differs from d (a multiple of d); v and out are then dense [B,H,L,d_v]
    unless ``strides_v`` is given."""
    code = {torch.float32: LINATTN_F32, torch.bfloat16: LINATTN_BF16}[io_dtype]
    Lx = 0 if L is None else int(L)
    if strides is None:
        strides = (H * Lx * d, Lx * d, d)
    if d_v is None or d_v == d:
        return Desc(B, H, d, conv_k, chunk, code, PHI[phi], float(eps), *[int(s) for s in strides], 0, 0, 0, 0, 0)
    if strides_v is None:
        strides_v = (H * Lx * d_v, Lx * d_v, d_v)
    return Desc(B, H, d, conv_k, chunk, code, PHI[phi], float(eps), *[int(s) for s in strides], int(d_v), 0,
                *[int(s) for s in strides_v])


def linattn_set_wait_limit(spins: int) -> int:
    return int(load().linattn_set_wait_limit(int(spins)))


def linattn_workspace_bytes(desc: Desc, L: int) -> int:
    return int(load().linattn_workspace_bytes(ctypes.byref(desc), int(L)))


def linattn_prefill(desc: Desc, L, q, k, v, conv_w, S_in, z_in, hist_in, out, S_out, z_out, hist_out,
                    workspace=None, workspace_bytes=None, stream=None) -> None:
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = load().linattn_prefill(ctypes.byref(desc), int(L), _ptr(q), _ptr(k), _ptr(v), _ptr(conv_w),
                                _ptr(S_in), _ptr(z_in), _ptr(hist_in), _ptr(out), _ptr(S_out), _ptr(z_out),
                                _ptr(hist_out), _ptr(workspace), int(workspace_bytes), _stream(stream))
    _check(st, "linattn_prefill")


def linattn_prefill_noalloc(desc: Desc, L, q, k, v, conv_w, S_in, z_in, hist_in, out, S_out, z_out, hist_out, stream=None) -> None:
    st = load().linattn_prefill_noalloc(ctypes.byref(desc), int(L), _ptr(q), _ptr(k), _ptr(v), _ptr(conv_w),
                                        _ptr(S_in), _ptr(z_in), _ptr(hist_in), _ptr(out), _ptr(S_out), _ptr(z_out),
                                        _ptr(hist_out), _stream(stream))
    _check(st, "linattn_prefill_noalloc")


def linattn_noalloc_scratch_bytes() -> int:
    return int(load().linattn_noalloc_scratch_bytes())


def linattn_prefill_grouped(desc: Desc, L, alpha, q, k, v, conv_w, S_in, z_in, hist_in, out, S_out, z_out, hist_out,
                            workspace=None, workspace_bytes=None, stream=None) -> None:
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = load().linattn_prefill_grouped(ctypes.byref(desc), int(L), float(alpha), _ptr(q), _ptr(k), _ptr(v), _ptr(conv_w),
                                        _ptr(S_in), _ptr(z_in), _ptr(hist_in), _ptr(out), _ptr(S_out), _ptr(z_out),
                                        _ptr(hist_out), _ptr(workspace), int(workspace_bytes), _stream(stream))
    _check(st, "linattn_prefill_grouped")


def linattn_backward_workspace_bytes(desc: Desc, L) -> int:
    return int(load().linattn_backward_workspace_bytes(ctypes.byref(desc), int(L)))


def linattn_prefill_grouped_backward(desc: Desc, L, alpha, q, k, v, conv_w, dout, dq, dk, dv, dconv_w, workspace,
                                     workspace_bytes=None, stream=None) -> None:
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = load().linattn_prefill_grouped_backward(ctypes.byref(desc), int(L), float(alpha), _ptr(q), _ptr(k), _ptr(v),
                                                 _ptr(conv_w), _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dconv_w),
                                                 _ptr(workspace), int(workspace_bytes), _stream(stream))
    _check(st, "linattn_prefill_grouped_backward")


def linattn_verify(desc: Desc, kk, q, k, v, conv_w, S, z, hist, n_commit, out, stream=None) -> None:
    st = load().linattn_verify(ctypes.byref(desc), int(kk), _ptr(q), _ptr(k), _ptr(v), _ptr(conv_w),
                               _ptr(S), _ptr(z), _ptr(hist), _ptr(n_commit), _ptr(out), _stream(stream))
    _check(st, "linattn_verify")


def linattn_verify_grouped(desc: Desc, kk, alpha, q, k, v, conv_w, S, z, hist, kwin, vwin, fill, n_commit, out, stream=None) -> None:
    st = load().linattn_verify_grouped(ctypes.byref(desc), int(kk), float(alpha), _ptr(q), _ptr(k), _ptr(v), _ptr(conv_w),
                                       _ptr(S), _ptr(z), _ptr(hist), _ptr(kwin), _ptr(vwin), _ptr(fill), _ptr(n_commit),
                                       _ptr(out), _stream(stream))
    _check(st, "linattn_verify_grouped")


def linattn_verify_tree(desc: Desc, n, q, k, v, parent, conv_w, S, z, hist, accept, out, stream=None) -> None:
    st = load().linattn_verify_tree(ctypes.byref(desc), int(n), _ptr(q), _ptr(k), _ptr(v), _ptr(parent), _ptr(conv_w),
                                    _ptr(S), _ptr(z), _ptr(hist), _ptr(accept), _ptr(out), _stream(stream))
    _check(st, "linattn_verify_tree")


def linattn_decode(desc: Desc, q, k, v, conv_w, S, z, hist, out, stream=None) -> None:
    st = load().linattn_decode(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(conv_w),
                               _ptr(S), _ptr(z), _ptr(hist), _ptr(out), _stream(stream))
    _check(st, "linattn_decode")


# ---- conveniences that only allocate with torch and forward to the calls above ---------------
def prefill(q, k, v, conv_w, state=None, chunk=64, eps=0.0, want_state=True, stream=None, phi="elu1", grouped_alpha=None):
    """q, k: [B,H,L,d], v: [B,H,L,d_v] CUDA tensors (fp32 or bf16; d_v = d or a multiple of d), dense or any view
    with unit stride along the last axis (e.g. ``x.transpose(1, 2)`` of a token-major [B,L,H,d] tensor); q and k
    share their strides, and so does v when d_v = d; ``out`` gets v's shape and strides.  Returns out, (S, z, hist).
    grouped_alpha: None, or the weight of the grouped branch of the three-branch form (``linattn_prefill_grouped``)."""
    B, H, L, d = q.shape
    d_v = v.shape[3]
    Kc = conv_w.shape[2]
    dense = q.is_contiguous() and k.is_contiguous() and v.is_contiguous()
    if not dense and (q.stride(3) != 1 or v.stride(3) != 1 or k.stride() != q.stride() or (d_v == d and v.stride() != q.stride())):
        raise ValueError("q, k (and v, when it has their width) must share their strides and be contiguous along d")
    sq = None if dense else q.stride()[:3]
    sv = None if dense else v.stride()[:3]
    if d_v == d:
        desc = make_desc(B, H, d, Kc, chunk, q.dtype, eps, strides=sq, L=L, phi=phi)
    else:
        desc = make_desc(B, H, d, Kc, chunk, q.dtype, eps, strides=sq, L=L, phi=phi, d_v=d_v, strides_v=sv)
    out = torch.empty_like(v) if dense else torch.empty_strided(v.shape, v.stride(), dtype=v.dtype, device=v.device)
    S_in, z_in, h_in = state if state is not None else (None, None, None)
    S = z = h = None
    if want_state:
        S = torch.empty((B, H, d, d_v), dtype=torch.float32, device=q.device)
        z = torch.empty((B, H, d), dtype=torch.float32, device=q.device)
        h = torch.empty((B, H, max(Kc - 1, 0), d_v), dtype=q.dtype, device=q.device)
    nbytes = linattn_workspace_bytes(desc, L)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=q.device) if nbytes else None
    if ws is not None and stream is not None and not isinstance(stream, int):
        ws.record_stream(stream)     # the allocator must not hand this memory out again before the launch stream is done with it
    if grouped_alpha is None:
        linattn_prefill(desc, L, q, k, v, conv_w, S_in, z_in, h_in, out, S, z, h, ws, nbytes, stream)
    else:
        linattn_prefill_grouped(desc, L, grouped_alpha, q, k, v, conv_w, S_in, z_in, h_in, out, S, z, h, ws, nbytes, stream)
    return out, (S, z, h)


def prefill_grouped(q, k, v, conv_w, alpha=1.0, state=None, eps=0.0, want_state=True, stream=None, phi="elu1", group=64):
    """The three-branch form (grouped linear attention, weight alpha + local softmax attention + masked conv)
    with groups of 64 or 256 tokens; arguments as for ``prefill``."""
    return prefill(q, k, v, conv_w, state, group, eps, want_state, stream, phi, grouped_alpha=alpha)


def prefill_grouped_backward(q, k, v, conv_w, dout, alpha=1.0, eps=0.0, stream=None, phi="elu1", group=256,
                             want_dw=True):
    """Gradient of ``prefill_grouped`` for a sequence that starts from nothing: q, k, v, dout bf16 [B,H,L,d] CUDA
    tensors, dense or views that share their strides and are contiguous along d.  Returns dq, dk, dv (same layout)
    and the gradient of the conv weights (fp32 [H,d,Kc], summed over the batch; None if not wanted)."""
    B, H, L, d = q.shape
    Kc = conv_w.shape[2]
    dense = all(t.is_contiguous() for t in (q, k, v, dout))
    if not dense and (q.stride(3) != 1 or any(t.stride() != q.stride() for t in (k, v, dout))):
        raise ValueError("q, k, v and dout must share their strides and be contiguous along d")
    desc = make_desc(B, H, d, Kc, group, q.dtype, eps, strides=None if dense else q.stride()[:3], L=L, phi=phi)
    new = (lambda: torch.empty_like(q)) if dense else (lambda: torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device))
    dq, dk, dv = new(), new(), new()
    dw = torch.empty((H, d, Kc), dtype=torch.float32, device=q.device) if want_dw else None
    nbytes = linattn_backward_workspace_bytes(desc, L)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=q.device)
    if stream is not None and not isinstance(stream, int):
        ws.record_stream(stream)
    linattn_prefill_grouped_backward(desc, L, alpha, q, k, v, conv_w, dout, dq, dk, dv, dw, ws, nbytes, stream)
    return dq, dk, dv, dw


def verify(q, k, v, conv_w, state, n_commit=None, eps=0.0, stream=None, phi="elu1"):
    """q, k: dense [B,H,kk,d]; v: dense [B,H,kk,d_v].  ``state`` = (S, z, hist) is updated in place.  Returns out."""
    B, H, kk, d = q.shape
    desc = make_desc(B, H, d, conv_w.shape[2], 64, q.dtype, eps, L=kk, phi=phi, d_v=v.shape[-1])
    out = torch.empty_like(v)
    S, z, h = state
    linattn_verify(desc, kk, q, k, v, conv_w, S, z, h, n_commit, out, stream)
    return out


def grouped_state(B, H, d, conv_k, dtype=torch.bfloat16, device="cuda", prefill_state=None):
    """State of the three-branch form for ``verify_grouped``: (S, z, hist, kwin, vwin, fill).  Zeros (start of a
    sequence), or the (S, z, hist) that ``prefill_grouped`` returned for a multiple of 64 tokens, with an empty
    open group."""
    if prefill_state is None:
        S = torch.zeros((B, H, d, d), dtype=torch.float32, device=device)
        z = torch.zeros((B, H, d), dtype=torch.float32, device=device)
        h = torch.zeros((B, H, max(conv_k - 1, 0), d), dtype=dtype, device=device)
    else:
        S, z, h = prefill_state
    kwin = torch.zeros((B, H, 64, d), dtype=dtype, device=device)
    vwin = torch.zeros((B, H, 64, d), dtype=dtype, device=device)
    fill = torch.zeros((B, H), dtype=torch.int32, device=device)
    return S, z, h, kwin, vwin, fill


def verify_grouped(q, k, v, conv_w, state, alpha=1.0, n_commit=None, eps=0.0, stream=None, phi="elu1"):
    """q, k, v: dense [B,H,kk,d].  ``state`` = (S, z, hist, kwin, vwin, fill) is updated in place.  Returns out."""
    B, H, kk, d = q.shape
    desc = make_desc(B, H, d, conv_w.shape[2], 64, q.dtype, eps, L=kk, phi=phi)
    out = torch.empty_like(q)
    S, z, h, kwin, vwin, fill = state
    linattn_verify_grouped(desc, kk, alpha, q, k, v, conv_w, S, z, h, kwin, vwin, fill, n_commit, out, stream)
    return out


def verify_tree(q, k, v, parent, conv_w, state, accept=None, eps=0.0, stream=None, phi="elu1"):
    """q, k, v: dense [B,H,n,d], bf16 or fp32; parent: int32 [n] on the GPU.  ``state`` is updated in place along the
    root path of candidate ``accept[b]`` (int32 [B] on the GPU; None accepts nothing).  Returns out."""
    B, H, n, d = q.shape
    desc = make_desc(B, H, d, conv_w.shape[2], 64, q.dtype, eps, L=n, phi=phi)
    out = torch.empty_like(q)
    S, z, h = state
    linattn_verify_tree(desc, n, q, k, v, parent, conv_w, S, z, h, accept, out, stream)
    return out


def decode(q, k, v, conv_w, state, eps=0.0, stream=None, phi="elu1"):
    """q, k: dense [B,H,d] (or [B,H,1,d]); v: dense [B,H,d_v].  ``state`` is updated in place.  Returns out."""
    B, H, d = q.shape[0], q.shape[1], q.shape[-1]
    desc = make_desc(B, H, d, conv_w.shape[2], 64, q.dtype, eps, L=1, phi=phi, d_v=v.shape[-1])
    out = torch.empty_like(v)
    S, z, h = state
    linattn_decode(desc, q, k, v, conv_w, S, z, h, out, stream)
    return out
