"""Thin ctypes binding of libla2.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; there is no CPU or
PyTorch fallback.  torch is used for device memory and streams.  If the shared
library is missing the first call raises (build it with
`python -m paper_2401_04658_amd.build` or `__graft_entry__.build()`).
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libla2.so")
_lib = None

LA2_F32, LA2_BF16, LA2_F16 = 0, 1, 2
LA2_OP_FWD, LA2_OP_BWD, LA2_OP_FWD_STATE, LA2_OP_BWD_STATE = 0, 1, 2, 3


class LA2Error(RuntimeError):
    def __init__(self, code, message):
        super().__init__("la2 status %d: %s" % (code, message))
        self.code = code


class la2_desc(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("heads", ctypes.c_int32), ("seqlen", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32), ("reserved", ctypes.c_int32),
        ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_n", ctypes.c_int64),
    ]


def lib_path():
    return _LIB_PATH


def load():
    """Loads libla2.so (no fallback: raises if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            "%s not found: the HIP library has not been built (python -m paper_2401_04658_amd.build)" % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32
    dp = ctypes.POINTER(la2_desc)
    lib.la2_desc_dense.argtypes = [dp, i32, i32, i32, i32, i32]
    lib.la2_desc_dense.restype = None
    lib.la2_workspace_bytes.argtypes = [dp, i32]
    lib.la2_workspace_bytes.restype = sz
    lib.la2_chunk_plan.argtypes = [dp, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.la2_chunk_plan.restype = ctypes.c_int
    lib.la2_block_size.argtypes = [dp]
    lib.la2_block_size.restype = i32
    lib.la2_set_chunk_tokens.argtypes = [i32]
    lib.la2_set_chunk_tokens.restype = None
    lib.la2_set_scan_variant.argtypes = [i32]
    lib.la2_set_scan_variant.restype = None
    lib.la2_fwd_state_norm.argtypes = [dp, vp, vp, vp, vp, vp, ctypes.c_float, vp, vp, vp, vp, sz, vp]
    lib.la2_fwd_state_norm.restype = ctypes.c_int
    lib.la2_bwd_state_norm.argtypes = [dp] + [vp] * 15 + [sz, vp]
    lib.la2_bwd_state_norm.restype = ctypes.c_int
    lib.la2_decode_step_norm.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, vp, ctypes.c_float, vp, vp]
    lib.la2_decode_step_norm.restype = ctypes.c_int
    lib.la2_fwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.la2_fwd.restype = ctypes.c_int
    lib.la2_fwd_noalloc.argtypes = [dp, vp, vp, vp, vp, vp, vp]
    lib.la2_fwd_noalloc.restype = ctypes.c_int
    lib.la2_bwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.la2_bwd.restype = ctypes.c_int
    lib.la2_fwd_state.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.la2_fwd_state.restype = ctypes.c_int
    lib.la2_bwd_state.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.la2_bwd_state.restype = ctypes.c_int
    lib.la2_bwd_saved.argtypes = [dp] + [vp] * 12 + [sz, i32, vp, sz, vp]
    lib.la2_bwd_saved.restype = ctypes.c_int
    lib.la2_fwd_norm.argtypes = [dp, vp, vp, vp, vp, ctypes.c_float, vp, vp, vp, sz, vp]
    lib.la2_fwd_norm.restype = ctypes.c_int
    lib.la2_bwd_norm.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.la2_bwd_norm.restype = ctypes.c_int
    lib.la2_varlen_workspace_bytes.argtypes = [dp, ctypes.c_int64, i32]
    lib.la2_varlen_workspace_bytes.restype = sz
    lib.la2_fwd_varlen.argtypes = [dp, vp, ctypes.c_int64, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.la2_fwd_varlen.restype = ctypes.c_int
    lib.la2_bwd_varlen.argtypes = [dp, vp, ctypes.c_int64, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.la2_bwd_varlen.restype = ctypes.c_int
    lib.la2_fwd_varlen_state.argtypes = [dp, vp, ctypes.c_int64, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.la2_fwd_varlen_state.restype = ctypes.c_int
    lib.la2_bwd_varlen_state.argtypes = [dp, vp, ctypes.c_int64] + [vp] * 11 + [vp, sz, vp]
    lib.la2_bwd_varlen_state.restype = ctypes.c_int
    lib.la2_fwd_varlen_norm.argtypes = [dp, vp, ctypes.c_int64, vp, vp, vp, vp, ctypes.c_float, vp, vp, vp, sz, vp]
    lib.la2_fwd_varlen_norm.restype = ctypes.c_int
    lib.la2_bwd_varlen_norm.argtypes = [dp, vp, ctypes.c_int64] + [vp] * 11 + [vp, sz, vp]
    lib.la2_bwd_varlen_norm.restype = ctypes.c_int
    lib.la2_decode_multi_norm.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, ctypes.c_float, vp, vp, vp]
    lib.la2_decode_multi_norm.restype = ctypes.c_int
    lib.la2_left_product_fwd.argtypes = [dp, vp, vp, vp, vp, vp, vp]
    lib.la2_left_product_fwd.restype = ctypes.c_int
    lib.la2_left_product_bwd.argtypes = [dp] + [vp] * 9
    lib.la2_left_product_bwd.restype = ctypes.c_int
    lib.la2_decode_multi.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.la2_decode_multi.restype = ctypes.c_int
    lib.la2_decode_step.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.la2_decode_step.restype = ctypes.c_int
    lib.la2_status_string.argtypes = [ctypes.c_int]
    lib.la2_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check(code):
    if code != 0:
        raise LA2Error(code, load().la2_status_string(code).decode())


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return LA2_BF16
    if t.dtype == torch.float16:
        return LA2_F16
    if t.dtype == torch.float32:
        return LA2_F32
    raise TypeError("la2: dtype must be torch.bfloat16, torch.float16 or torch.float32, got %s" % t.dtype)


def make_desc(t):
    """Descriptor of a [batch, heads, seqlen, head_dim] tensor (feature stride must be 1)."""
    if t.dim() != 4:
        raise ValueError("la2: expected a [batch, heads, seqlen, head_dim] tensor")
    if t.shape[3] > 1 and t.stride(3) != 1:
        raise ValueError("la2: the feature dimension must be contiguous")
    b, h, n, d = t.shape
    return la2_desc(b, h, n, d, _dtype_code(t), 0, t.stride(0), t.stride(1), t.stride(2))


def _same_layout(ref, *others):
    for o in others:
        if o.shape != ref.shape or o.stride() != ref.stride() or o.dtype != ref.dtype or o.device != ref.device:
            raise ValueError("la2: all sequence tensors must share shape, strides, dtype and device")


def _stream(t):
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def la2_workspace_bytes(t, op=LA2_OP_FWD):
    desc = make_desc(t)
    return int(load().la2_workspace_bytes(ctypes.byref(desc), op))


def la2_chunk_plan(t):
    """(nchunks, chunk_tokens) of the sequence chunks la2_fwd / la2_bwd run in parallel for this tensor."""
    desc = make_desc(t)
    n, c = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(load().la2_chunk_plan(ctypes.byref(desc), ctypes.byref(n), ctypes.byref(c)))
    return int(n.value), int(c.value)


def la2_block_size(t):
    desc = make_desc(t)
    return int(load().la2_block_size(ctypes.byref(desc)))


def la2_set_chunk_tokens(tokens):
    load().la2_set_chunk_tokens(int(tokens))


def la2_set_scan_variant(variant):
    load().la2_set_scan_variant(int(variant))


def _workspace(t, op, workspace):
    need = la2_workspace_bytes(t, op)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=t.device)
    if workspace is None:
        return None, 0, None
    return ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(), workspace


def la2_fwd(q, k, v, lam, out=None, workspace=None):
    """o = LA2(q, k, v; lam) on the GPU.  q, k, v: [b, H, n, d] bf16/fp32; lam: fp32 [H] (device)."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_fwd: tensors must live on the GPU")
    _same_layout(q, k, v)
    if out is None:
        out = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    _same_layout(q, out)
    desc = make_desc(q)
    ws_ptr, ws_bytes, _keep = _workspace(q, LA2_OP_FWD, workspace)
    with torch.cuda.device(q.device):
        _check(lib.la2_fwd(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(), lam.data_ptr(),
                           out.data_ptr(), ws_ptr, ws_bytes, _stream(q)))
    return out


def la2_fwd_noalloc(q, k, v, lam, out):
    """la2_fwd into `out` with the library's built-in scratch instead of a workspace; the call itself allocates
    nothing (so `out` is required)."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_fwd_noalloc: tensors must live on the GPU")
    _same_layout(q, k, v, out)
    desc = make_desc(q)
    with torch.cuda.device(q.device):
        _check(lib.la2_fwd_noalloc(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(), lam.data_ptr(),
                                   out.data_ptr(), _stream(q)))
    return out


def la2_bwd(q, k, v, d_o, lam, out=None, workspace=None):
    """(dq, dk, dv) of sum(o * d_o) on the GPU."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_bwd: tensors must live on the GPU")
    _same_layout(q, k, v, d_o)
    if out is None:
        out = tuple(torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device) for _ in range(3))
    dq, dk, dv = out
    _same_layout(q, dq, dk, dv)
    desc = make_desc(q)
    ws_ptr, ws_bytes, _keep = _workspace(q, LA2_OP_BWD, workspace)
    with torch.cuda.device(q.device):
        _check(lib.la2_bwd(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(), d_o.data_ptr(),
                           lam.data_ptr(), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), ws_ptr, ws_bytes,
                           _stream(q)))
    return dq, dk, dv


def la2_fwd_norm(q, k, v, lam, eps=1e-6, out=None, rstd=None, workspace=None):
    """(o, rstd) = Norm(LA2(q, k, v; lam)): every output row scaled by rstd = 1 / sqrt(mean(row^2) + eps)."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_fwd_norm: tensors must live on the GPU")
    _same_layout(q, k, v)
    if out is None:
        out = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    _same_layout(q, out)
    if rstd is None:
        rstd = torch.empty(q.shape[:3], dtype=torch.float32, device=q.device)
    if rstd.dtype != torch.float32 or tuple(rstd.shape) != tuple(q.shape[:3]) or not rstd.is_contiguous():
        raise ValueError("la2_fwd_norm: rstd must be a contiguous fp32 [batch, heads, seqlen] tensor")
    desc = make_desc(q)
    ws_ptr, ws_bytes, _keep = _workspace(q, LA2_OP_FWD, workspace)
    with torch.cuda.device(q.device):
        _check(lib.la2_fwd_norm(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(), lam.data_ptr(),
                                float(eps), out.data_ptr(), rstd.data_ptr(), ws_ptr, ws_bytes, _stream(q)))
    return out, rstd


def la2_bwd_norm(q, k, v, o, rstd, d_o, lam, out=None, d_u=None, workspace=None):
    """(dq, dk, dv) of sum(la2_fwd_norm(q, k, v)[0] * d_o); o, rstd are la2_fwd_norm's results.  d_u (same
    layout as d_o) receives the gradient with respect to the un-normalised output."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_bwd_norm: tensors must live on the GPU")
    _same_layout(q, k, v, o, d_o)
    if out is None:
        out = tuple(torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device) for _ in range(3))
    if d_u is None:
        d_u = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    dq, dk, dv = out
    _same_layout(q, dq, dk, dv, d_u)
    if rstd.dtype != torch.float32 or tuple(rstd.shape) != tuple(q.shape[:3]) or not rstd.is_contiguous():
        raise ValueError("la2_bwd_norm: rstd must be a contiguous fp32 [batch, heads, seqlen] tensor")
    desc = make_desc(q)
    ws_ptr, ws_bytes, _keep = _workspace(q, LA2_OP_BWD, workspace)
    with torch.cuda.device(q.device):
        _check(lib.la2_bwd_norm(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
                                rstd.data_ptr(), d_o.data_ptr(), lam.data_ptr(), d_u.data_ptr(), dq.data_ptr(),
                                dk.data_ptr(), dv.data_ptr(), ws_ptr, ws_bytes, _stream(q)))
    return dq, dk, dv


def _varlen_desc(q, cu_seqlens, max_seqlen):
    """Descriptor of packed sequences: q is [total_positions, heads, head_dim], cu_seqlens int32 [batch + 1]."""
    if q.dim() != 3 or q.stride(2) != 1:
        raise ValueError("la2: packed tensors are [total_positions, heads, head_dim] with unit feature stride")
    if cu_seqlens.dtype != torch.int32 or cu_seqlens.dim() != 1 or not cu_seqlens.is_contiguous() or not cu_seqlens.is_cuda:
        raise ValueError("la2: cu_seqlens must be a contiguous int32 vector on the GPU")
    return la2_desc(cu_seqlens.numel() - 1, q.shape[1], int(max_seqlen), q.shape[2], _dtype_code(q), 0,
                    0, q.stride(1), q.stride(0))


def _varlen_workspace(q, desc, op, workspace):
    need = int(load().la2_varlen_workspace_bytes(ctypes.byref(desc), q.shape[0], op))
    if need == 0:
        return None, 0, None
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    if workspace.numel() * workspace.element_size() < need:
        raise ValueError("la2: workspace too small (%d < %d bytes)" % (workspace.numel() * workspace.element_size(), need))
    return workspace.data_ptr(), workspace.numel() * workspace.element_size(), workspace


def la2_fwd_varlen(q, k, v, lam, cu_seqlens, max_seqlen, out=None, workspace=None):
    """o for packed sequences of different lengths: q, k, v [total_positions, heads, head_dim]; sequence b is
    positions cu_seqlens[b] .. cu_seqlens[b + 1] - 1; max_seqlen bounds the lengths."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_fwd_varlen: tensors must live on the GPU")
    _same_layout(q, k, v)
    if out is None:
        out = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    _same_layout(q, out)
    desc = _varlen_desc(q, cu_seqlens, max_seqlen)
    ws_ptr, ws_bytes, _keep = _varlen_workspace(q, desc, LA2_OP_FWD, workspace)
    with torch.cuda.device(q.device):
        _check(lib.la2_fwd_varlen(ctypes.byref(desc), cu_seqlens.data_ptr(), q.shape[0], q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                  lam.data_ptr(), out.data_ptr(), ws_ptr, ws_bytes, _stream(q)))
    return out


def la2_bwd_varlen(q, k, v, d_o, lam, cu_seqlens, max_seqlen, out=None, workspace=None):
    """(dq, dk, dv) for packed sequences of different lengths (see la2_fwd_varlen)."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_bwd_varlen: tensors must live on the GPU")
    _same_layout(q, k, v, d_o)
    if out is None:
        out = tuple(torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device) for _ in range(3))
    dq, dk, dv = out
    _same_layout(q, dq, dk, dv)
    desc = _varlen_desc(q, cu_seqlens, max_seqlen)
    ws_ptr, ws_bytes, _keep = _varlen_workspace(q, desc, LA2_OP_BWD, workspace)
    with torch.cuda.device(q.device):
        _check(lib.la2_bwd_varlen(ctypes.byref(desc), cu_seqlens.data_ptr(), q.shape[0], q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                  d_o.data_ptr(), lam.data_ptr(), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), ws_ptr,
                                  ws_bytes, _stream(q)))
    return dq, dk, dv


def _packed_state(t, q, cu_seqlens, name):
    """A dense fp32 [sequences, H, d, d] state tensor (or None) -> pointer argument."""
    if t is None:
        return None
    nseq, h, d = cu_seqlens.numel() - 1, q.shape[1], q.shape[2]
    if t.dtype != torch.float32 or tuple(t.shape) != (nseq, h, d, d) or not t.is_contiguous() or t.device != q.device:
        raise ValueError("%s must be dense fp32 [sequences, H, d, d] on the tensors' device" % name)
    return ctypes.c_void_p(t.data_ptr()) if t.numel() else None


def la2_fwd_varlen_state(q, k, v, lam, cu_seqlens, max_seqlen, kv_init=None, want_final=True, out=None, kv_final=None,
                         workspace=None):
    """Packed sequences as segments: o and every sequence's state after its last position, each started from its
    kv_init (fp32 [sequences, H, d, d], None = zero).  Returns (o, kv_final or None)."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_fwd_varlen_state: tensors must live on the GPU")
    _same_layout(q, k, v)
    if out is None:
        out = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    _same_layout(q, out)
    desc = _varlen_desc(q, cu_seqlens, max_seqlen)
    if want_final and kv_final is None:
        kv_final = torch.empty((cu_seqlens.numel() - 1, q.shape[1], q.shape[2], q.shape[2]), dtype=torch.float32,
                               device=q.device)
    ws_ptr, ws_bytes, _keep = _varlen_workspace(q, desc, LA2_OP_FWD, workspace)
    with torch.cuda.device(q.device):
        _check(lib.la2_fwd_varlen_state(ctypes.byref(desc), cu_seqlens.data_ptr(), q.shape[0], q.data_ptr(), k.data_ptr(),
                                        v.data_ptr(), lam.data_ptr(), _packed_state(kv_init, q, cu_seqlens, "kv_init"),
                                        out.data_ptr(),
                                        _packed_state(kv_final, q, cu_seqlens, "kv_final") if want_final else None,
                                        ws_ptr, ws_bytes, _stream(q)))
    return out, (kv_final if want_final else None)


def la2_bwd_varlen_state(q, k, v, d_o, lam, cu_seqlens, max_seqlen, kv_init=None, d_kv_final=None, want_d_kv_init=True,
                         out=None, d_kv_init=None, workspace=None):
    """Backward of la2_fwd_varlen_state.  Returns (dq, dk, dv, d_kv_init or None)."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_bwd_varlen_state: tensors must live on the GPU")
    _same_layout(q, k, v, d_o)
    if out is None:
        out = tuple(torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device) for _ in range(3))
    dq, dk, dv = out
    _same_layout(q, dq, dk, dv)
    desc = _varlen_desc(q, cu_seqlens, max_seqlen)
    if want_d_kv_init and d_kv_init is None:
        d_kv_init = torch.empty((cu_seqlens.numel() - 1, q.shape[1], q.shape[2], q.shape[2]), dtype=torch.float32,
                                device=q.device)
    ws_ptr, ws_bytes, _keep = _varlen_workspace(q, desc, LA2_OP_BWD, workspace)
    with torch.cuda.device(q.device):
        _check(lib.la2_bwd_varlen_state(ctypes.byref(desc), cu_seqlens.data_ptr(), q.shape[0], q.data_ptr(), k.data_ptr(),
                                        v.data_ptr(), d_o.data_ptr(), lam.data_ptr(),
                                        _packed_state(kv_init, q, cu_seqlens, "kv_init"),
                                        _packed_state(d_kv_final, q, cu_seqlens, "d_kv_final"), dq.data_ptr(),
                                        dk.data_ptr(), dv.data_ptr(),
                                        _packed_state(d_kv_init, q, cu_seqlens, "d_kv_init") if want_d_kv_init else None,
                                        ws_ptr, ws_bytes, _stream(q)))
    return dq, dk, dv, (d_kv_init if want_d_kv_init else None)


def la2_fwd_varlen_norm(q, k, v, lam, cu_seqlens, max_seqlen, eps=1e-6, out=None, rstd=None, workspace=None):
    """(o, rstd) of the normalised operator over packed sequences; rstd is fp32 [heads, total_positions]."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_fwd_varlen_norm: tensors must live on the GPU")
    _same_layout(q, k, v)
    if out is None:
        out = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    _same_layout(q, out)
    if rstd is None:
        rstd = torch.empty((q.shape[1], q.shape[0]), dtype=torch.float32, device=q.device)
    if rstd.dtype != torch.float32 or tuple(rstd.shape) != (q.shape[1], q.shape[0]) or not rstd.is_contiguous():
        raise ValueError("la2_fwd_varlen_norm: rstd must be a contiguous fp32 [heads, total_positions] tensor")
    desc = _varlen_desc(q, cu_seqlens, max_seqlen)
    ws_ptr, ws_bytes, _keep = _varlen_workspace(q, desc, LA2_OP_FWD, workspace)
    with torch.cuda.device(q.device):
        _check(lib.la2_fwd_varlen_norm(ctypes.byref(desc), cu_seqlens.data_ptr(), q.shape[0], q.data_ptr(), k.data_ptr(),
                                       v.data_ptr(), lam.data_ptr(), float(eps), out.data_ptr(), rstd.data_ptr(), ws_ptr,
                                       ws_bytes, _stream(q)))
    return out, rstd


def la2_bwd_varlen_norm(q, k, v, o, rstd, d_o, lam, cu_seqlens, max_seqlen, out=None, d_u=None, workspace=None):
    """(dq, dk, dv) of the normalised operator over packed sequences (o, rstd from la2_fwd_varlen_norm)."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_bwd_varlen_norm: tensors must live on the GPU")
    _same_layout(q, k, v, o, d_o)
    if out is None:
        out = tuple(torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device) for _ in range(3))
    if d_u is None:
        d_u = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    dq, dk, dv = out
    _same_layout(q, dq, dk, dv, d_u)
    if rstd.dtype != torch.float32 or tuple(rstd.shape) != (q.shape[1], q.shape[0]) or not rstd.is_contiguous():
        raise ValueError("la2_bwd_varlen_norm: rstd must be a contiguous fp32 [heads, total_positions] tensor")
    desc = _varlen_desc(q, cu_seqlens, max_seqlen)
    ws_ptr, ws_bytes, _keep = _varlen_workspace(q, desc, LA2_OP_BWD, workspace)
    with torch.cuda.device(q.device):
        _check(lib.la2_bwd_varlen_norm(ctypes.byref(desc), cu_seqlens.data_ptr(), q.shape[0], q.data_ptr(), k.data_ptr(),
                                       v.data_ptr(), o.data_ptr(), rstd.data_ptr(), d_o.data_ptr(), lam.data_ptr(),
                                       d_u.data_ptr(), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), ws_ptr, ws_bytes,
                                       _stream(q)))
    return dq, dk, dv


def la2_decode_multi_norm(q, k, v, lam, kv_state, eps=1e-6, out=None, rstd=None):
    """ntokens consecutive steps of the normalised operator in one launch; returns (o, rstd [b, H, T])."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_decode_multi_norm: tensors must live on the GPU")
    b, h, t, d = q.shape
    for x in (q, k, v):
        if x.shape != q.shape or x.dtype != q.dtype or not x.is_contiguous():
            raise ValueError("la2_decode_multi_norm: q, k, v must be dense [b, H, T, d] of one dtype")
    if kv_state.dtype != torch.float32 or tuple(kv_state.shape) != (b, h, d, d) or not kv_state.is_contiguous():
        raise ValueError("la2_decode_multi_norm: kv_state must be dense fp32 [b, H, d, d]")
    if out is None:
        out = torch.empty_like(q)
    if rstd is None:
        rstd = torch.empty((b, h, t), dtype=torch.float32, device=q.device)
    with torch.cuda.device(q.device):
        _check(lib.la2_decode_multi_norm(b, h, d, t, _dtype_code(q), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                         lam.data_ptr(), kv_state.data_ptr(), float(eps), out.data_ptr(), rstd.data_ptr(),
                                         _stream(q)))
    return out, rstd


def _state(t, q, name):
    """A dense fp32 [b, H, d, d] state tensor (or None) -> pointer argument."""
    if t is None:
        return None
    b, h, _, d = q.shape
    if t.dtype != torch.float32 or tuple(t.shape) != (b, h, d, d) or not t.is_contiguous() or t.device != q.device:
        raise ValueError("%s must be dense fp32 [b, H, d, d] on the tensors' device" % name)
    return ctypes.c_void_p(t.data_ptr()) if t.numel() else None


def la2_fwd_state(q, k, v, lam, kv_init=None, want_final=True, out=None, kv_final=None, workspace=None):
    """One segment of a sequence: o and the state after its last position, started from kv_init
    (fp32 [b, H, d, d], None = zero).  Returns (o, kv_final or None)."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_fwd_state: tensors must live on the GPU")
    _same_layout(q, k, v)
    if out is None:
        out = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    _same_layout(q, out)
    b, h, _, d = q.shape
    if want_final and kv_final is None:
        kv_final = torch.empty((b, h, d, d), dtype=torch.float32, device=q.device)
    desc = make_desc(q)
    ws_ptr, ws_bytes, _keep = _workspace(q, LA2_OP_FWD_STATE, workspace)
    with torch.cuda.device(q.device):
        _check(lib.la2_fwd_state(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(), lam.data_ptr(),
                                 _state(kv_init, q, "kv_init"), out.data_ptr(),
                                 _state(kv_final, q, "kv_final") if want_final else None,
                                 ws_ptr, ws_bytes, _stream(q)))
    return out, (kv_final if want_final else None)


def la2_bwd_state(q, k, v, d_o, lam, kv_init=None, d_kv_final=None, want_d_kv_init=True, out=None,
                  d_kv_init=None, workspace=None, fwd_workspace=None, fwd_wrote_kv_final=False):
    """Backward of one segment.  Returns (dq, dk, dv, d_kv_init or None).  fwd_workspace: the workspace
    tensor the forward call used (contents untouched since), to reuse its chunk states; fwd_wrote_kv_final:
    whether that call handed out kv_final."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_bwd_state: tensors must live on the GPU")
    _same_layout(q, k, v, d_o)
    if out is None:
        out = tuple(torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device) for _ in range(3))
    dq, dk, dv = out
    _same_layout(q, dq, dk, dv)
    b, h, _, d = q.shape
    if want_d_kv_init and d_kv_init is None:
        d_kv_init = torch.empty((b, h, d, d), dtype=torch.float32, device=q.device)
    desc = make_desc(q)
    ws_ptr, ws_bytes, _keep = _workspace(q, LA2_OP_BWD_STATE, workspace)
    with torch.cuda.device(q.device):
        fwd_ws = ctypes.c_void_p(fwd_workspace.data_ptr()) if fwd_workspace is not None else None
        _check(lib.la2_bwd_saved(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(), d_o.data_ptr(),
                                 lam.data_ptr(), _state(kv_init, q, "kv_init"),
                                 _state(d_kv_final, q, "d_kv_final"), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(),
                                 _state(d_kv_init, q, "d_kv_init") if want_d_kv_init else None,
                                 fwd_ws, fwd_workspace.numel() * fwd_workspace.element_size() if fwd_workspace is not None else 0,
                                 1 if fwd_wrote_kv_final else 0, ws_ptr, ws_bytes, _stream(q)))
    return dq, dk, dv, (d_kv_init if want_d_kv_init else None)


def la2_decode_step(q, k, v, lam, kv_state, out=None):
    """One recurrent step; kv_state (fp32 [b, H, d, d]) is updated in place, returns o [b, H, d]."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_decode_step: tensors must live on the GPU")
    b, h, d = q.shape
    for t in (q, k, v):
        if t.shape != q.shape or t.dtype != q.dtype or not t.is_contiguous():
            raise ValueError("la2_decode_step: q, k, v must be dense [b, H, d] of one dtype")
    if kv_state.dtype != torch.float32 or tuple(kv_state.shape) != (b, h, d, d) or not kv_state.is_contiguous():
        raise ValueError("la2_decode_step: kv_state must be dense fp32 [b, H, d, d]")
    if out is None:
        out = torch.empty_like(q)
    with torch.cuda.device(q.device):
        _check(lib.la2_decode_step(b, h, d, _dtype_code(q), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                   lam.data_ptr(), kv_state.data_ptr(), out.data_ptr(), _stream(q)))
    return out


def la2_decode_multi(q, k, v, lam, kv_state, out=None):
    """ntokens consecutive recurrent steps in one launch.  q, k, v: dense [b, H, T, d]; kv_state (fp32
    [b, H, d, d]) is updated in place; returns o [b, H, T, d]."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_decode_multi: tensors must live on the GPU")
    b, h, t, d = q.shape
    for x in (q, k, v):
        if x.shape != q.shape or x.dtype != q.dtype or not x.is_contiguous():
            raise ValueError("la2_decode_multi: q, k, v must be dense [b, H, T, d] of one dtype")
    if kv_state.dtype != torch.float32 or tuple(kv_state.shape) != (b, h, d, d) or not kv_state.is_contiguous():
        raise ValueError("la2_decode_multi: kv_state must be dense fp32 [b, H, d, d]")
    if out is None:
        out = torch.empty_like(q)
    with torch.cuda.device(q.device):
        _check(lib.la2_decode_multi(b, h, d, t, _dtype_code(q), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                    lam.data_ptr(), kv_state.data_ptr(), out.data_ptr(), _stream(q)))
    return out


def la2_left_product_fwd(q, k, v, lam, out=None):
    """The forward pass as the O(n^2 d) masked left product (comparison kernel, bf16)."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_left_product_fwd: tensors must live on the GPU")
    _same_layout(q, k, v)
    if out is None:
        out = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    _same_layout(q, out)
    desc = make_desc(q)
    with torch.cuda.device(q.device):
        _check(lib.la2_left_product_fwd(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(), lam.data_ptr(),
                                        out.data_ptr(), _stream(q)))
    return out


def la2_left_product_bwd(q, k, v, d_o, lam, out=None):
    """(dq, dk, dv) as O(n^2 d) masked products (comparison kernel, bf16)."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_left_product_bwd: tensors must live on the GPU")
    _same_layout(q, k, v, d_o)
    if out is None:
        out = tuple(torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device) for _ in range(3))
    dq, dk, dv = out
    _same_layout(q, dq, dk, dv)
    desc = make_desc(q)
    with torch.cuda.device(q.device):
        _check(lib.la2_left_product_bwd(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(), d_o.data_ptr(),
                                        lam.data_ptr(), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), _stream(q)))
    return dq, dk, dv


def la2_fwd_state_norm(q, k, v, lam, eps=1e-6, kv_init=None, want_final=True, out=None, rstd=None, kv_final=None,
                       workspace=None):
    """la2_fwd_norm on one segment of a sequence, started from kv_init.  Returns (o, rstd, kv_final or None)."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_fwd_state_norm: tensors must live on the GPU")
    _same_layout(q, k, v)
    if out is None:
        out = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    _same_layout(q, out)
    b, h, n, d = q.shape
    if rstd is None:
        rstd = torch.empty((b, h, n), dtype=torch.float32, device=q.device)
    if rstd.dtype != torch.float32 or tuple(rstd.shape) != (b, h, n) or not rstd.is_contiguous():
        raise ValueError("la2_fwd_state_norm: rstd must be a contiguous fp32 [batch, heads, seqlen] tensor")
    if want_final and kv_final is None:
        kv_final = torch.empty((b, h, d, d), dtype=torch.float32, device=q.device)
    desc = make_desc(q)
    ws_ptr, ws_bytes, _keep = _workspace(q, LA2_OP_FWD_STATE, workspace)
    with torch.cuda.device(q.device):
        _check(lib.la2_fwd_state_norm(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(), lam.data_ptr(),
                                      _state(kv_init, q, "kv_init"), float(eps), out.data_ptr(), rstd.data_ptr(),
                                      _state(kv_final, q, "kv_final") if want_final else None,
                                      ws_ptr, ws_bytes, _stream(q)))
    return out, rstd, (kv_final if want_final else None)


def la2_bwd_state_norm(q, k, v, o, rstd, d_o, lam, kv_init=None, d_kv_final=None, want_d_kv_init=True, out=None,
                       d_u=None, d_kv_init=None, workspace=None):
    """Backward of la2_fwd_state_norm.  Returns (dq, dk, dv, d_kv_init or None)."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_bwd_state_norm: tensors must live on the GPU")
    _same_layout(q, k, v, o, d_o)
    if out is None:
        out = tuple(torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device) for _ in range(3))
    if d_u is None:
        d_u = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    _same_layout(q, d_u, *out)
    b, h, n, d = q.shape
    if rstd.dtype != torch.float32 or tuple(rstd.shape) != (b, h, n) or not rstd.is_contiguous():
        raise ValueError("la2_bwd_state_norm: rstd must be a contiguous fp32 [batch, heads, seqlen] tensor")
    if want_d_kv_init and d_kv_init is None:
        d_kv_init = torch.empty((b, h, d, d), dtype=torch.float32, device=q.device)
    desc = make_desc(q)
    ws_ptr, ws_bytes, _keep = _workspace(q, LA2_OP_BWD_STATE, workspace)
    with torch.cuda.device(q.device):
        _check(lib.la2_bwd_state_norm(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
                                      rstd.data_ptr(), d_o.data_ptr(), lam.data_ptr(), _state(kv_init, q, "kv_init"),
                                      _state(d_kv_final, q, "d_kv_final"), d_u.data_ptr(), out[0].data_ptr(),
                                      out[1].data_ptr(), out[2].data_ptr(),
                                      _state(d_kv_init, q, "d_kv_init") if want_d_kv_init else None,
                                      ws_ptr, ws_bytes, _stream(q)))
    return out[0], out[1], out[2], (d_kv_init if want_d_kv_init else None)


def la2_decode_step_norm(q, k, v, lam, kv_state, eps=1e-6, out=None):
    """One recurrent step of the normalised operator; kv_state (fp32 [b, H, d, d]) is updated in place, returns
    the normalised o [b, H, d]."""
    lib = load()
    if not q.is_cuda:
        raise ValueError("la2_decode_step_norm: tensors must live on the GPU")
    b, h, d = q.shape
    for t in (q, k, v):
        if t.shape != q.shape or t.dtype != q.dtype or not t.is_contiguous():
            raise ValueError("la2_decode_step_norm: q, k, v must be dense [b, H, d] of one dtype")
    if kv_state.dtype != torch.float32 or tuple(kv_state.shape) != (b, h, d, d) or not kv_state.is_contiguous():
        raise ValueError("la2_decode_step_norm: kv_state must be dense fp32 [b, H, d, d]")
    if out is None:
        out = torch.empty_like(q)
    with torch.cuda.device(q.device):
        _check(lib.la2_decode_step_norm(b, h, d, _dtype_code(q), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                        lam.data_ptr(), kv_state.data_ptr(), float(eps), out.data_ptr(), _stream(q)))
    return out
