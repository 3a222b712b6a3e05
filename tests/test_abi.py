"""Host-only checks of the C-ABI library: it loads, exports every declared symbol, and rejects
bad arguments with a status code before anything is launched (no GPU needed)."""
import ctypes
import os
import re

import pytest

from paper_2401_04658_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "la2.h")

OK, E_NULL, E_SHAPE, E_DTYPE, E_ALIGN, E_WS, E_LAUNCH, E_VALUE = range(8)


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.lib_path()):
        from paper_2401_04658_amd.build import build
        build()
    return binding.load()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(la2_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_entry_points():
    names = declared_functions()
    for must in ("la2_fwd", "la2_bwd", "la2_decode_step", "la2_workspace_bytes", "la2_status_string"):
        assert must in names


def test_every_declared_symbol_is_exported(lib):
    for name in declared_functions():
        assert hasattr(lib, name), "libla2.so does not export %s" % name


def dense(lib, b, h, n, d, dtype):
    desc = binding.la2_desc()
    lib.la2_desc_dense(ctypes.byref(desc), b, h, n, d, dtype)
    return desc


def test_desc_dense(lib):
    d = dense(lib, 2, 3, 100, 64, binding.LA2_BF16)
    assert (d.stride_n, d.stride_h, d.stride_b) == (64, 6400, 19200)
    assert (d.batch, d.heads, d.seqlen, d.head_dim, d.dtype, d.reserved) == (2, 3, 100, 64, 1, 0)


P = 0x10000  # a fake, suitably aligned "device pointer"; validation failures return before any use


def fwd(lib, desc, q=P, k=P, v=P, lam=P, o=P, ws=None, ws_bytes=0):
    return lib.la2_fwd(ctypes.byref(desc) if desc is not None else None, q, k, v, lam, o, ws, ws_bytes, None)


def bwd(lib, desc, ptrs=None, ws=None, ws_bytes=0):
    ptrs = ptrs or [P] * 8
    return lib.la2_bwd(ctypes.byref(desc), *ptrs, ws, ws_bytes, None)


def test_null_arguments(lib):
    d = dense(lib, 1, 1, 128, 64, binding.LA2_BF16)
    assert fwd(lib, None) == E_NULL
    for name in ("q", "k", "v", "lam", "o"):
        assert fwd(lib, d, **{name: None}) == E_NULL
    for i in range(8):
        ptrs = [P] * 8
        ptrs[i] = None
        assert bwd(lib, d, ptrs) == E_NULL
    assert lib.la2_decode_step(1, 1, 64, 1, None, P, P, P, P, P, None) == E_NULL
    assert lib.la2_decode_step(1, 1, 64, 1, P, P, P, P, None, P, None) == E_NULL


def test_shape_errors(lib):
    for bad in (dict(batch=-1), dict(heads=-2), dict(seqlen=-5), dict(head_dim=80), dict(head_dim=192), dict(head_dim=0),
                dict(reserved=1)):
        d = dense(lib, 1, 1, 128, 64, binding.LA2_BF16)
        for kk, vv in bad.items():
            setattr(d, kk, vv)
        assert fwd(lib, d) == E_SHAPE, bad
        assert bwd(lib, d) == E_SHAPE, bad
        assert lib.la2_workspace_bytes(ctypes.byref(d), 0) == 0
        assert lib.la2_block_size(ctypes.byref(d)) == 0
    assert lib.la2_decode_step(1, 1, 100, 1, P, P, P, P, P, P, None) == E_SHAPE
    assert lib.la2_decode_step(-1, 1, 64, 1, P, P, P, P, P, P, None) == E_SHAPE


def test_dtype_errors(lib):
    d = dense(lib, 1, 1, 128, 64, binding.LA2_BF16)
    d.dtype = 7
    assert fwd(lib, d) == E_DTYPE
    assert bwd(lib, d) == E_DTYPE
    assert lib.la2_decode_step(1, 1, 64, 5, P, P, P, P, P, P, None) == E_DTYPE


def test_alignment_errors(lib):
    d = dense(lib, 1, 1, 128, 64, binding.LA2_BF16)
    assert fwd(lib, d, q=P + 2) == E_ALIGN
    assert fwd(lib, d, o=P + 8) == E_ALIGN
    d.stride_n = 68  # 136 bytes: not a multiple of 16
    assert fwd(lib, d) == E_ALIGN
    d = dense(lib, 1, 1, 128, 64, binding.LA2_F32)
    d.stride_n = 32  # rows would overlap
    assert fwd(lib, d) == E_ALIGN
    d = dense(lib, 1, 2, 128, 64, binding.LA2_F32)
    d.stride_h = 128 * 64 + 2
    assert bwd(lib, d) == E_ALIGN
    assert lib.la2_decode_step(1, 1, 64, 1, P + 4, P, P, P, P, P, None) == E_ALIGN


def test_workspace_rules(lib):
    try:
        lib.la2_set_chunk_tokens(256)
        d = dense(lib, 1, 2, 1024, 128, binding.LA2_BF16)
        need = lib.la2_workspace_bytes(ctypes.byref(d), 0)
        assert need == 2 * 4 * 128 * 128 * 4  # chains x chunks x d x d fp32
        # backward, 16-bit head_dim 128: the dQ scan's chunk states and the dK / dV scan's, side by side
        assert lib.la2_workspace_bytes(ctypes.byref(d), 1) == 2 * need
        d32 = dense(lib, 1, 2, 1024, 128, binding.LA2_F32)
        assert lib.la2_workspace_bytes(ctypes.byref(d32), 1) == lib.la2_workspace_bytes(ctypes.byref(d32), 0) > 0
        assert lib.la2_workspace_bytes(ctypes.byref(d), 9) == 0
        assert fwd(lib, d) == E_WS
        assert fwd(lib, d, ws=P, ws_bytes=need - 1) == E_WS
        assert fwd(lib, d, ws=P + 16, ws_bytes=need) == E_WS
        assert bwd(lib, d, ws=None, ws_bytes=2 * need) == E_WS
        assert bwd(lib, d, ws=P * 16, ws_bytes=2 * need - 1) == E_WS
        # a chunk as long as the sequence needs no workspace
        lib.la2_set_chunk_tokens(1024)
        assert lib.la2_workspace_bytes(ctypes.byref(d), 0) == 0
    finally:
        lib.la2_set_chunk_tokens(0)


def test_automatic_chunking_is_sized_for_the_device(lib):
    # 16 chains on a 256-CU device: the sequence is cut so that about 256 workgroups exist
    d = dense(lib, 1, 16, 65536, 128, binding.LA2_BF16)
    need = lib.la2_workspace_bytes(ctypes.byref(d), 0)
    chunks = need // (16 * 128 * 128 * 4)
    assert 8 <= chunks <= 64
    # enough chains already: no chunking, no workspace
    d = dense(lib, 64, 16, 1024, 128, binding.LA2_BF16)
    assert lib.la2_workspace_bytes(ctypes.byref(d), 0) == 0


def test_empty_problem_is_ok_without_a_device(lib):
    d = dense(lib, 0, 4, 128, 64, binding.LA2_BF16)
    assert fwd(lib, d) == OK
    d = dense(lib, 2, 4, 0, 64, binding.LA2_F32)
    assert fwd(lib, d) == OK
    assert bwd(lib, d) == OK


def test_block_size_and_status_strings(lib):
    for dt in (binding.LA2_BF16, binding.LA2_F32):
        for hd in (64, 128):
            d = dense(lib, 1, 1, 128, hd, dt)
            assert lib.la2_block_size(ctypes.byref(d)) in (32, 64, 128)
    seen = set()
    for code in range(8):
        s = lib.la2_status_string(code)
        assert s and s not in seen
        seen.add(s)
    assert lib.la2_status_string(99) == b"unknown status"


def test_binding_refuses_cpu_tensors(lib):
    import torch
    x = torch.zeros(1, 1, 8, 64, dtype=torch.bfloat16)
    lam = torch.ones(1)
    with pytest.raises(ValueError):
        binding.la2_fwd(x, x, x, lam)
    with pytest.raises(ValueError):
        binding.la2_bwd(x, x, x, x, lam)


def fwd_state(lib, desc, kv_init=None, kv_final=None, q=P, ws=None, ws_bytes=0):
    return lib.la2_fwd_state(ctypes.byref(desc), q, P, P, P, kv_init, P, kv_final, ws, ws_bytes, None)


def bwd_state(lib, desc, kv_init=None, d_kv_final=None, d_kv_init=None, q=P):
    return lib.la2_bwd_state(ctypes.byref(desc), q, P, P, P, P, kv_init, d_kv_final, P, P, P, d_kv_init, None, 0,
                             None)


def test_state_entry_points_validate_before_any_launch(lib):
    # fp32 data: a gradient entering at the end of a sequence that does not end on a block boundary needs workspace
    # (the hand-over of dKV from the token-by-token tail to the block kernels)
    d = dense(lib, 300, 2, 100, 64, binding.LA2_F32)
    assert lib.la2_workspace_bytes(ctypes.byref(d), 1) == 0
    assert lib.la2_workspace_bytes(ctypes.byref(d), 3) == 300 * 2 * 64 * 64 * 4
    assert lib.la2_workspace_bytes(ctypes.byref(d), 2) == 0
    assert bwd_state(lib, d, d_kv_final=P) == E_WS
    d = dense(lib, 300, 2, 128, 64, binding.LA2_F32)
    assert lib.la2_workspace_bytes(ctypes.byref(d), 3) == 0
    # the 16-bit kernels form the state at a ragged end themselves: no tail, no hand-over
    d = dense(lib, 300, 2, 100, 64, binding.LA2_BF16)
    assert lib.la2_workspace_bytes(ctypes.byref(d), 3) == 0
    # misaligned state pointers
    d = dense(lib, 300, 1, 128, 64, binding.LA2_BF16)
    assert fwd_state(lib, d, kv_init=P + 4) == E_ALIGN
    assert fwd_state(lib, d, kv_final=P + 8) == E_ALIGN
    assert bwd_state(lib, d, d_kv_final=P + 4) == E_ALIGN
    assert bwd_state(lib, d, d_kv_init=P + 4) == E_ALIGN
    # the other checks are those of la2_fwd / la2_bwd
    assert fwd_state(lib, d, kv_init=P, q=None) == E_NULL
    assert bwd_state(lib, d, kv_init=P, q=None) == E_NULL
    d.head_dim = 80
    assert fwd_state(lib, d, kv_init=P) == E_SHAPE
    # nothing to do: no chains; an empty sequence with no state wanted
    assert fwd_state(lib, dense(lib, 0, 4, 128, 64, binding.LA2_BF16), kv_init=P, kv_final=P) == OK
    assert fwd_state(lib, dense(lib, 2, 4, 0, 64, binding.LA2_BF16), kv_init=P) == OK
    assert bwd_state(lib, dense(lib, 2, 4, 0, 64, binding.LA2_BF16), kv_init=P) == OK


def test_decode_multi_validation(lib):
    dm = lambda b=1, h=1, d=64, t=4, dt=1, q=P, kv=P: lib.la2_decode_multi(b, h, d, t, dt, q, P, P, P, kv, P, None)
    assert dm(q=None) == E_NULL and dm(kv=None) == E_NULL
    assert dm(d=100) == E_SHAPE and dm(t=-1) == E_SHAPE and dm(b=-1) == E_SHAPE
    assert dm(dt=5) == E_DTYPE
    assert dm(q=P + 4) == E_ALIGN
    assert dm(t=0, q=None) == OK and dm(b=0, q=None) == OK


def test_norm_entry_points_validate_before_any_launch(lib):
    d = dense(lib, 300, 2, 128, 64, binding.LA2_BF16)
    ref = ctypes.byref(d)
    fn = lambda eps=1e-6, q=P, o=P, rstd=P: lib.la2_fwd_norm(ref, q, P, P, P, eps, o, rstd, None, 0, None)
    assert fn(eps=-1.0) == E_VALUE and fn(eps=float("nan")) == E_VALUE and fn(eps=float("inf")) == E_VALUE
    assert fn(q=None) == E_NULL and fn(rstd=None) == E_NULL
    assert fn(o=P + 8) == E_ALIGN and fn(rstd=P + 2) == E_ALIGN
    bn = lambda o=P, rstd=P, d_u=P, dq=P: lib.la2_bwd_norm(ref, P, P, P, o, rstd, P, P, d_u, dq, P, P, None, 0, None)
    assert bn(o=None) == E_NULL and bn(rstd=None) == E_NULL and bn(d_u=None) == E_NULL and bn(dq=None) == E_NULL
    assert bn(d_u=P + 4) == E_ALIGN and bn(rstd=P + 1) == E_ALIGN
    d.head_dim = 100
    assert fn() == E_SHAPE and bn() == E_SHAPE
    # chunked problems need the workspace of la2_fwd / la2_bwd
    try:
        lib.la2_set_chunk_tokens(256)
        d = dense(lib, 1, 2, 1024, 128, binding.LA2_F32)
        ref = ctypes.byref(d)
        assert fn() == E_WS and bn() == E_WS
    finally:
        lib.la2_set_chunk_tokens(0)
    # nothing to do
    d = dense(lib, 0, 2, 128, 64, binding.LA2_BF16)
    ref = ctypes.byref(d)
    assert fn(q=None, rstd=None) == OK and bn(o=None) == OK


def test_header_is_plain_c_and_cxx():
    """The boundary is a C ABI: the header compiles as C99 and as C++ without any HIP or torch header."""
    import subprocess
    for cmd in (["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-x", "c", HEADER],
                ["g++", "-std=c++11", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c++", HEADER]):
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert res.returncode == 0, res.stdout


def test_chain_span_limit(lib):
    """One chain must stay addressable with 32-bit byte offsets, ragged last block included."""
    d = dense(lib, 1, 1, (1 << 24) - 127, 128, binding.LA2_BF16)     # one position too many
    assert fwd(lib, d) == E_SHAPE and bwd(lib, d) == E_SHAPE
    assert lib.la2_workspace_bytes(ctypes.byref(d), 0) == 0
    d = dense(lib, 1, 1, (1 << 23) - 127, 128, binding.LA2_F32)
    assert fwd(lib, d) == E_SHAPE
    d = dense(lib, 4, 1, 200000, 64, binding.LA2_BF16)               # [b, n, H, d] storage with a large row pitch
    d.stride_n = 16384
    assert fwd(lib, d) == E_SHAPE


def test_fp16_is_accepted_except_by_the_comparison_kernel(lib):
    d = dense(lib, 0, 2, 128, 64, binding.LA2_F16)          # an empty problem passes validation without a launch
    assert fwd(lib, d) == OK and bwd(lib, d) == OK
    d = dense(lib, 300, 2, 128, 64, binding.LA2_F16)
    assert fwd(lib, d, q=None) == E_NULL and fwd(lib, d, o=P + 8) == E_ALIGN
    assert lib.la2_block_size(ctypes.byref(d)) == 32
    d = dense(lib, 300, 2, 128, 128, binding.LA2_F16)
    assert lib.la2_block_size(ctypes.byref(d)) == 32
    assert lib.la2_left_product_fwd(ctypes.byref(d), P, P, P, P, P, None) == E_DTYPE
    assert lib.la2_left_product_bwd(ctypes.byref(d), P, P, P, P, P, P, P, P, None) == E_DTYPE
    db = dense(lib, 2, 2, 128, 128, binding.LA2_BF16)
    assert lib.la2_left_product_bwd(ctypes.byref(db), P, P, P, None, P, P, P, P, None) == E_NULL
    assert lib.la2_left_product_bwd(ctypes.byref(db), P, P, P, P, P, P, P + 8, P, None) == E_ALIGN
    db.head_dim = 96
    db.stride_n = 96
    assert lib.la2_left_product_bwd(ctypes.byref(db), P, P, P, P, P, P, P, P, None) == E_SHAPE
    assert lib.la2_decode_step(0, 1, 64, binding.LA2_F16, None, None, None, None, None, None, None) == OK


def test_a_c_program_links_and_calls_the_library(lib, tmp_path):
    """include/la2.h + libla2.so from plain C (gcc), host-side calls only."""
    import subprocess
    exe = tmp_path / "abi_client"
    libdir = os.path.dirname(binding.lib_path())
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "abi_client.c"), "-o", str(exe),
                           "-L", libdir, "-l:libla2.so", "-Wl,-rpath," + libdir])
    res = subprocess.run([str(exe)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert res.returncode == 0 and "abi client ok" in res.stdout, (res.returncode, res.stdout)


def test_varlen_entry_points_validate_before_any_launch(lib):
    d = dense(lib, 5, 2, 300, 64, binding.LA2_BF16)      # 5 sequences of at most 300 positions, [total, H, d] packing
    d.stride_b, d.stride_h, d.stride_n = 0, 64, 128
    ref = ctypes.byref(d)
    fv = lambda cu=P, q=P, o=P, total=0: lib.la2_fwd_varlen(ref, cu, total, q, P, P, P, o, None, 0, None)
    bv = lambda cu=P, dq=P, total=0: lib.la2_bwd_varlen(ref, cu, total, P, P, P, P, P, dq, P, P, None, 0, None)
    assert fv(total=-1) == E_SHAPE and bv(total=-1) == E_SHAPE
    assert fv(cu=None) == E_NULL and fv(q=None) == E_NULL and bv(cu=None) == E_NULL and bv(dq=None) == E_NULL
    assert fv(cu=P + 2) == E_ALIGN and fv(o=P + 8) == E_ALIGN and bv(dq=P + 4) == E_ALIGN
    d.head_dim = 80
    assert fv() == E_SHAPE and bv() == E_SHAPE
    d.head_dim = 64
    d.batch = 0
    assert fv(cu=None, q=None) == OK and bv(cu=None) == OK
    # few long sequences: the workspace of the dense plan for (batch, max_seqlen)
    try:
        lib.la2_set_chunk_tokens(256)
        d = dense(lib, 2, 2, 1024, 128, binding.LA2_BF16)
        d.stride_b, d.stride_h, d.stride_n = 0, 128, 256
        ref = ctypes.byref(d)
        assert lib.la2_workspace_bytes(ref, 0) == 4 * 4 * 128 * 128 * 4
        assert fv() == E_WS and bv() == E_WS
    finally:
        lib.la2_set_chunk_tokens(0)


def test_packed_state_entry_points_validate_before_any_launch(lib):
    vp = ctypes.c_void_p
    lib.la2_fwd_varlen_state.argtypes = [vp, vp, ctypes.c_int64] + [vp] * 8 + [ctypes.c_size_t, vp]
    lib.la2_fwd_varlen_state.restype = ctypes.c_int
    lib.la2_bwd_varlen_state.argtypes = [vp, vp, ctypes.c_int64] + [vp] * 12 + [ctypes.c_size_t, vp]
    lib.la2_bwd_varlen_state.restype = ctypes.c_int
    d = dense(lib, 5, 2, 300, 64, binding.LA2_BF16)
    d.stride_b, d.stride_h, d.stride_n = 0, 64, 128
    ref = ctypes.byref(d)
    fs = lambda cu=P, q=P, init=P, fin=P, total=0: lib.la2_fwd_varlen_state(ref, cu, total, q, P, P, P, init, P, fin, None, 0, None)
    bs = lambda cu=P, dq=P, init=P, dfin=P, dinit=P, total=0: lib.la2_bwd_varlen_state(
        ref, cu, total, P, P, P, P, P, init, dfin, dq, P, P, dinit, None, 0, None)
    assert fs(total=-1) == E_SHAPE and bs(total=-1) == E_SHAPE
    assert fs(cu=None) == E_NULL and fs(q=None) == E_NULL and bs(cu=None) == E_NULL and bs(dq=None) == E_NULL
    assert fs(init=P + 4) == E_ALIGN and fs(fin=P + 8) == E_ALIGN
    assert bs(init=P + 4) == E_ALIGN and bs(dfin=P + 8) == E_ALIGN and bs(dinit=P + 4) == E_ALIGN
    # state hand-over over packed batches: the 16-bit types at head_dim 64 and 128
    d.dtype = binding.LA2_F32
    assert fs() == E_DTYPE and bs() == E_DTYPE
    assert fs(init=None, fin=None, cu=None) == E_NULL      # without states: la2_fwd_varlen, which takes fp32
    d.dtype = binding.LA2_F16
    assert fs(cu=None) == E_NULL
    for hd in (96, 256):
        w = dense(lib, 5, 2, 300, hd, binding.LA2_BF16)
        w.stride_b, w.stride_h, w.stride_n = 0, hd, 2 * hd
        wr = ctypes.byref(w)
        assert lib.la2_fwd_varlen_state(wr, P, 0, P, P, P, P, P, P, P, None, 0, None) == E_SHAPE
        assert lib.la2_bwd_varlen_state(wr, P, 0, P, P, P, P, P, P, P, P, P, P, P, None, 0, None) == E_SHAPE
        assert lib.la2_fwd_varlen_state(wr, None, 0, P, P, P, P, None, P, None, None, 0, None) == E_NULL
    d.dtype = binding.LA2_BF16
    d.batch = 0
    assert fs(cu=None, q=None) == OK and bs(cu=None) == OK


def test_head_dim_96_and_256_are_accepted_where_they_have_kernels(lib):
    for hd in (96, 256):
        for dt in (binding.LA2_BF16, binding.LA2_F16, binding.LA2_F32):
            d = dense(lib, 2, 2, 100, hd, dt)
            ref = ctypes.byref(d)
            # validation passes the shape check and goes on to the pointer checks
            assert fwd(lib, d, q=None) == E_NULL and bwd(lib, d, [None] + [P] * 7) == E_NULL
            assert fwd_state(lib, d, kv_init=P, q=None) == E_NULL
            assert lib.la2_block_size(ref) == (32 if dt != binding.LA2_F32 else 1)
            assert lib.la2_decode_step(1, 1, hd, dt, None, P, P, P, P, P, None) == E_NULL
            assert lib.la2_decode_multi(1, 1, hd, 4, dt, None, P, P, P, P, P, None) == E_NULL
            assert lib.la2_fwd_norm(ref, None, P, P, P, 1e-6, P, P, None, 0, None) == E_NULL
            assert lib.la2_bwd_norm(ref, None, P, P, P, P, P, P, P, P, P, P, None, 0, None) == E_NULL
            # no left-product comparison at these head dimensions
            if dt == binding.LA2_BF16:
                assert lib.la2_left_product_fwd(ref, P, P, P, P, P, None) == E_SHAPE
            # packed batches: the 16-bit types only
            d.stride_b, d.stride_h, d.stride_n = 0, hd, 2 * hd
            want = E_NULL if dt != binding.LA2_F32 else E_DTYPE
            assert lib.la2_fwd_varlen(ref, None, 0, P, P, P, P, P, None, 0, None) == want
            assert lib.la2_bwd_varlen(ref, None, 0, P, P, P, P, P, P, P, P, None, 0, None) == want
        # fp32 runs the token recurrence: never a workspace; the 16-bit kernel is exact at ragged ends: no
        # hand-over state in the workspace
        try:
            lib.la2_set_chunk_tokens(64)
            assert lib.la2_workspace_bytes(ctypes.byref(dense(lib, 1, 2, 1000, hd, binding.LA2_F32)), 1) == 0
            d = dense(lib, 1, 2, 1000, hd, binding.LA2_BF16)
            nchunks = (1000 + 63) // 64
            assert lib.la2_workspace_bytes(ctypes.byref(d), 0) == 2 * nchunks * hd * hd * 4
            assert lib.la2_workspace_bytes(ctypes.byref(d), 3) == 2 * nchunks * hd * hd * 4
        finally:
            lib.la2_set_chunk_tokens(0)


def test_bench_helpers_are_a_library_of_their_own(lib):
    """The measurement kernels live in libla2_bench.so; the C-ABI library does not export them."""
    from paper_2401_04658_amd import bench_probe
    assert not hasattr(lib, "la2_stream_probe") and not hasattr(lib, "la2_bench_stream_probe")
    bl = bench_probe.load()
    sp = lambda r=3, w=1, i=P, o=P, n=1024: bl.la2_bench_stream_probe(r, w, 0, i, o, n, None)
    assert sp(r=5) == E_SHAPE and sp(w=3) == E_SHAPE and sp(r=-1) == E_SHAPE and sp(r=0, w=0) == E_SHAPE
    assert sp(n=24) == E_ALIGN and sp(i=P + 8) == E_ALIGN and sp(o=P + 4) == E_ALIGN
    assert sp(i=None) == E_NULL and sp(o=None) == E_NULL
    assert sp(n=0, i=None, o=None) == OK
    assert bl.la2_bench_mfma_peak(0, 10, P, None) == E_SHAPE and bl.la2_bench_mfma_peak(4, 10, None, None) == E_NULL


def test_noalloc_entry_validates_on_the_host(lib):
    fn = lambda d, q=P, k=P, v=P, lam=P, o=P: lib.la2_fwd_noalloc(ctypes.byref(d) if d is not None else None,
                                                                  q, k, v, lam, o, None)
    d = dense(lib, 1, 8, 8192, 128, binding.LA2_BF16)
    assert lib.la2_workspace_bytes(ctypes.byref(d), 0) == 16 << 20      # exactly what the built-in scratch holds
    assert fn(None) == E_NULL
    for name in ("q", "k", "v", "lam", "o"):
        assert fn(d, **{name: None}) == E_NULL
    assert fn(d, q=P + 2) == E_ALIGN
    d.head_dim = 80
    assert fn(d) == E_SHAPE
    big = dense(lib, 1, 64, 1 << 16, 256, binding.LA2_BF16)             # 64 MiB of chunk states (four chunks, head_dim 256)
    assert lib.la2_workspace_bytes(ctypes.byref(big), 0) > 16 << 20
    assert fn(big) == E_WS
    empty = dense(lib, 0, 8, 8192, 128, binding.LA2_BF16)
    assert fn(empty, q=None, k=None, v=None, lam=None, o=None) == OK


def test_packed_batches_of_unequal_lengths_are_cut_into_chunks(lib):
    """191 sequences of 128 .. 8192 positions (65,536 in all) x 16 heads fill the device many times over, yet the
    longest sequence's block loop would outlast the rest: with the total known the plan cuts at an eighth of the
    longest length; with equal lengths, or the total unknown, it does not."""
    lib.la2_varlen_workspace_bytes.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32]
    lib.la2_varlen_workspace_bytes.restype = ctypes.c_size_t
    d = dense(lib, 191, 16, 8192, 128, binding.LA2_BF16)
    d.stride_b, d.stride_h, d.stride_n = 0, 128, 16 * 128
    ref = ctypes.byref(d)
    # chunks of 2048 positions (a quarter of the longest): at most 65536 / 2048 + 191 (sequence, chunk) pairs, 16
    # bytes of map each, plus 4 bytes for each of the at most 32 sequences longer than a chunk; at most
    # 2 * 65536 / 2048 state slots (only those sequences have them), times 16 heads
    map_bytes, states = 3840, 64 * 16 * 128 * 128 * 4
    assert lib.la2_varlen_workspace_bytes(ref, 65536, 0) == map_bytes + states
    assert lib.la2_varlen_workspace_bytes(ref, 65536, 1) == map_bytes + 2 * states
    assert lib.la2_varlen_workspace_bytes(ref, 0, 0) == 0 == lib.la2_workspace_bytes(ref, 0)
    assert lib.la2_varlen_workspace_bytes(ref, 191 * 8192, 0) == 0          # all sequences as long as the longest
    assert lib.la2_varlen_workspace_bytes(ref, 191 * 5000, 0) == 0          # about equal
    assert lib.la2_varlen_workspace_bytes(ref, -1, 0) == 0
    assert lib.la2_fwd_varlen(ref, P, 65536, P, P, P, P, P, None, 0, None) == E_WS
    assert lib.la2_bwd_varlen(ref, P, 65536, P, P, P, P, P, P, P, P, P * 16, map_bytes + states, None) == E_WS
    short = dense(lib, 4000, 16, 256, 128, binding.LA2_BF16)                 # nothing long enough to matter
    short.stride_b, short.stride_h, short.stride_n = 0, 128, 16 * 128
    assert lib.la2_varlen_workspace_bytes(ctypes.byref(short), 4000 * 40, 0) == 0


def test_packed_norm_and_multi_token_norm_validate_before_any_launch(lib):
    vp, i64, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_float
    lib.la2_fwd_varlen_norm.argtypes = [vp, vp, i64, vp, vp, vp, vp, f32, vp, vp, vp, ctypes.c_size_t, vp]
    lib.la2_fwd_varlen_norm.restype = ctypes.c_int
    lib.la2_bwd_varlen_norm.argtypes = [vp, vp, i64] + [vp] * 11 + [vp, ctypes.c_size_t, vp]
    lib.la2_bwd_varlen_norm.restype = ctypes.c_int
    lib.la2_decode_multi_norm.argtypes = [ctypes.c_int32] * 5 + [vp] * 5 + [f32, vp, vp, vp]
    lib.la2_decode_multi_norm.restype = ctypes.c_int
    d = dense(lib, 5, 2, 300, 64, binding.LA2_BF16)
    d.stride_b, d.stride_h, d.stride_n = 0, 64, 128
    ref = ctypes.byref(d)
    fn = lambda total=900, eps=1e-6, cu=P, rstd=P, q=P: lib.la2_fwd_varlen_norm(ref, cu, total, q, P, P, P, eps, P, rstd, None, 0, None)
    assert fn(eps=-1.0) == E_VALUE and fn(total=0) == E_SHAPE and fn(total=1 << 31) == E_SHAPE
    assert fn(rstd=None) == E_NULL and fn(cu=None) == E_NULL and fn(q=None) == E_NULL and fn(rstd=P + 2) == E_ALIGN
    bn = lambda total=900, o=P, rstd=P, d_u=P: lib.la2_bwd_varlen_norm(ref, P, total, P, P, P, o, rstd, P, P, d_u, P, P, P, None, 0, None)
    assert bn(total=0) == E_SHAPE and bn(o=None) == E_NULL and bn(rstd=None) == E_NULL and bn(d_u=None) == E_NULL
    assert bn(d_u=P + 8) == E_ALIGN
    dm = lambda eps=1e-6, rstd=P, q=P, T=8, hd=128: lib.la2_decode_multi_norm(2, 2, hd, T, 1, q, P, P, P, P, eps, P, rstd, None)
    assert dm(eps=float("nan")) == E_VALUE and dm(rstd=None) == E_NULL and dm(q=None) == E_NULL and dm(hd=100) == E_SHAPE
    assert dm(T=0, rstd=None, q=None) == OK and dm(rstd=P + 2) == E_ALIGN


def test_bwd_saved_checks_the_forward_workspace(lib):
    vp = ctypes.c_void_p
    lib.la2_bwd_saved.argtypes = [vp] * 13 + [ctypes.c_size_t, ctypes.c_int32, vp, ctypes.c_size_t, vp]
    lib.la2_bwd_saved.restype = ctypes.c_int
    try:
        lib.la2_set_chunk_tokens(256)
        d = dense(lib, 1, 2, 1024, 128, binding.LA2_BF16)
        need = lib.la2_workspace_bytes(ctypes.byref(d), 3)
        fneed = lib.la2_workspace_bytes(ctypes.byref(d), 2)
        assert need > 0 and fneed > 0
        call = lambda fws, fbytes, ws=P * 16, wsb=need: lib.la2_bwd_saved(
            ctypes.byref(d), P, P, P, P, P, None, None, P, P, P, None, fws, fbytes, 0, ws, wsb, None)
        assert call(P * 16 + 8, fneed) == E_WS        # misaligned
        assert call(P * 16, fneed - 1) == E_WS        # smaller than what the forward call needed
        # with the forward call's chunk states at hand the backward pass needs room for the dK / dV scan's only
        assert call(P * 16, fneed, wsb=fneed - 1) == E_WS
    finally:
        lib.la2_set_chunk_tokens(0)


def test_launch_grids_are_checked_before_any_launch(lib):
    """Chains x chunks beyond what a grid can index is a shape error of the descriptor, whatever the entry point."""
    try:
        lib.la2_set_chunk_tokens(64)
        d = dense(lib, 1 << 12, 1 << 12, 8192, 64, binding.LA2_BF16)    # 2^24 chains x 128 chunks x 2 scans = 2^32
        d.stride_b = d.stride_h = 0                                      # (overlapping chains: never launched)
        assert fwd(lib, d) == E_SHAPE and bwd(lib, d) == E_SHAPE
        assert lib.la2_workspace_bytes(ctypes.byref(d), 0) == 0
        d = dense(lib, 1 << 8, 1 << 8, 8192, 64, binding.LA2_BF16)      # 2^16 chains x 128 chunks: fine for a grid
        assert fwd(lib, d, ws=None, ws_bytes=0) == E_WS                 # (and then the workspace is asked for)
    finally:
        lib.la2_set_chunk_tokens(0)
    d = dense(lib, 1 << 12, 1 << 12, 512, 64, binding.LA2_BF16)         # 2^33 rows
    d.stride_b = d.stride_h = 0
    assert fwd(lib, d) == E_SHAPE


def test_state_norm_entry_points_validate_before_any_launch(lib):
    vp = ctypes.c_void_p
    lib.la2_fwd_state_norm.argtypes = [ctypes.c_void_p] * 6 + [ctypes.c_float] + [vp] * 4 + [ctypes.c_size_t, vp]
    lib.la2_fwd_state_norm.restype = ctypes.c_int
    lib.la2_bwd_state_norm.argtypes = [vp] * 16 + [ctypes.c_size_t, vp]
    lib.la2_bwd_state_norm.restype = ctypes.c_int
    d = dense(lib, 2, 2, 100, 128, binding.LA2_BF16)      # ragged: 100 = 3 * 32 + 4
    ref = ctypes.byref(d)
    fn = lambda eps=1e-6, q=P, rstd=P, kv0=None, kvn=None, ws=None, wsb=0: \
        lib.la2_fwd_state_norm(ref, q, P, P, P, kv0, eps, P, rstd, kvn, ws, wsb, None)
    assert fn(eps=-1.0) == E_VALUE and fn(eps=float("nan")) == E_VALUE
    assert fn(q=None) == E_NULL and fn(rstd=None) == E_NULL
    assert fn(rstd=P + 2) == E_ALIGN and fn(kv0=P + 4) == E_ALIGN and fn(kvn=P + 8) == E_ALIGN
    bn = lambda o=P, rstd=P, d_u=P, dkvn=None, dkv0=None, ws=None, wsb=0: \
        lib.la2_bwd_state_norm(ref, P, P, P, o, rstd, P, P, None, dkvn, d_u, P, P, P, dkv0, ws, wsb, None)
    assert bn(o=None) == E_NULL and bn(rstd=None) == E_NULL and bn(d_u=None) == E_NULL
    assert bn(d_u=P + 4) == E_ALIGN and bn(dkvn=P + 4) == E_ALIGN and bn(dkv0=P + 8) == E_ALIGN
    # fp32 data: a gradient coming in at a ragged end needs the hand-over state in the workspace: checked before
    # the row pass (the 16-bit kernels form the state at a ragged end themselves)
    assert lib.la2_workspace_bytes(ref, 3) == 0
    d.dtype = binding.LA2_F32
    d.stride_b, d.stride_h, d.stride_n = 2 * 100 * 128, 100 * 128, 128
    assert bn(dkvn=P) == E_WS
    assert lib.la2_workspace_bytes(ref, 3) == 2 * 2 * 128 * 128 * 4
    # an empty segment: nothing to check but the descriptor
    e = dense(lib, 2, 2, 0, 128, binding.LA2_BF16)
    assert lib.la2_fwd_state_norm(ctypes.byref(e), None, None, None, None, None, 1e-6, None, None, None, None, 0, None) == OK


def test_decode_step_norm_validation(lib):
    vp = ctypes.c_void_p
    lib.la2_decode_step_norm.argtypes = [ctypes.c_int32] * 4 + [vp] * 5 + [ctypes.c_float, vp, vp]
    lib.la2_decode_step_norm.restype = ctypes.c_int
    dn = lambda b=1, h=1, d=64, dt=1, q=P, kv=P, eps=1e-6, o=P: lib.la2_decode_step_norm(b, h, d, dt, q, P, P, P, kv, eps, o, None)
    assert dn(eps=-1.0) == E_VALUE and dn(eps=float("inf")) == E_VALUE
    assert dn(d=100) == E_SHAPE and dn(b=-1) == E_SHAPE and dn(dt=9) == E_DTYPE
    assert dn(q=None) == E_NULL and dn(kv=None) == E_NULL and dn(o=P + 8) == E_ALIGN
    assert dn(b=0, q=None, kv=None, o=None) == OK


def plan(lib, b, h, n, d, dtype):
    desc = dense(lib, b, h, n, d, dtype)
    nch, ct = ctypes.c_int32(0), ctypes.c_int32(0)
    assert lib.la2_chunk_plan(ctypes.byref(desc), ctypes.byref(nch), ctypes.byref(ct)) == OK
    return nch.value, ct.value


def test_the_chunk_planner_keeps_its_measured_rules(lib):
    """The rules of the sequence-chunk planner, each taken from a measurement (256 compute units, which is also what
    the library assumes when it sees no device)."""
    lib.la2_set_chunk_tokens(0)
    BF, F32 = binding.LA2_BF16, binding.LA2_F32
    # enough chains for every compute unit: no cut
    assert plan(lib, 16, 16, 4096, 128, BF) == (1, 4096)
    assert plan(lib, 64, 16, 1024, 128, BF)[0] == 1
    # few chains: as many chunks as keep the workgroups at or below one per compute unit, never more
    assert plan(lib, 4, 16, 16384, 128, BF) == (4, 4096)
    assert plan(lib, 1, 16, 65536, 128, BF) == (16, 4096)
    assert plan(lib, 4, 16, 2048, 64, BF) == (4, 512)
    for b, h, n, d in ((3, 16, 4096, 128), (5, 16, 4096, 128), (6, 16, 8192, 128), (7, 16, 4096, 128), (3, 16, 4096, 64),
                       (5, 16, 4096, 64), (7, 8, 4096, 256), (5, 8, 16384, 256)):
        nch, _ = plan(lib, b, h, n, d, BF)
        assert nch > 1 and b * h * nch <= 256 < b * h * (nch + 1), (b, h, n, d, nch)
    # more chains than half the compute units: no cut (two chunks would move 1.4 times the bytes for little)
    for d in (64, 96, 128, 256):
        assert plan(lib, 12, 16, 4096, d, BF)[0] == 1, d
        assert plan(lib, 9, 16, 4096, d, BF)[0] == 1, d
    # head_dim 96 also at exactly half, and two workgroups per unit while the chunks stay 640 positions or longer
    assert plan(lib, 8, 16, 4096, 96, BF)[0] == 1
    assert plan(lib, 4, 16, 8192, 96, BF) == (8, 1024)
    assert plan(lib, 1, 8, 32768, 96, BF) == (32, 1024)
    # head_dim 256: half-idle compute units run a block faster than busy ones, so 128 chains stay whole
    assert plan(lib, 16, 8, 4096, 256, BF)[0] == 1
    assert plan(lib, 8, 8, 8192, 256, BF) == (4, 2048)
    # fp32 at head_dim 64: three workgroups per compute unit
    assert plan(lib, 4, 16, 4096, 64, F32)[0] == 12 or plan(lib, 4, 16, 4096, 64, F32)[0] == 11
    assert plan(lib, 12, 16, 4096, 64, F32)[0] == 4
    # short sequences are not worth a pre-pass
    assert plan(lib, 8, 16, 256, 128, BF)[0] == 1


def test_batches_a_little_above_the_unit_count_take_the_workspace_of_their_remaining_rows(lib):
    """Every dense entry point runs a batch with a few more chains than one (or two) per compute unit as two calls:
    the rows that make whole rounds, un-chunked, and the remaining rows by their own plan.  The workspace query answers for
    exactly that (256 units assumed without a device); la2_chunk_plan still describes one call over the whole batch.
    Which shapes: those where two calls measured at least 5 % faster than one."""
    lib.la2_set_chunk_tokens(0)
    BF, F16, F32 = binding.LA2_BF16, binding.LA2_F16, binding.LA2_F32
    ws = lambda desc, op: lib.la2_workspace_bytes(ctypes.byref(desc), op)
    split = [(20, 16, 4096, 128, BF), (18, 16, 2048, 64, F16), (11, 32, 4096, 128, BF), (22, 16, 4096, 128, F16),
             (20, 16, 2048, 128, BF), (40, 8, 3072, 64, BF), (22, 12, 4096, 128, BF),      # up to 1.25 / 1.375 per unit
             (36, 16, 4096, 128, BF), (34, 16, 8192, 64, F16),                             # a little above two per unit
             (52, 16, 4096, 128, BF), (50, 16, 8192, 64, F16), (66, 16, 4096, 64, BF),     # ... three and four
             (34, 8, 2048, 256, BF), (36, 8, 4096, 256, F16),                              # head_dim 256: up to 1.125
             (18, 16, 2048, 96, BF), (20, 16, 4096, 96, BF), (34, 16, 4096, 96, F16),      # head_dim 96
             (20, 16, 4096, 128, F32), (24, 16, 1024, 64, F32), (34, 16, 4096, 128, F32)]  # fp32: up to 1.5
    for b, h, n, d, dt in split:
        first = (b * h // 256) * 256 // h
        whole, rest = dense(lib, b, h, n, d, dt), dense(lib, b - first, h, n, d, dt)
        assert plan(lib, b, h, n, d, dt)[0] == 1
        assert plan(lib, first, h, n, d, dt)[0] == 1
        assert plan(lib, b - first, h, n, d, dt)[0] > 1
        for op in (0, 1, 2, 3):           # plain and state entry points alike
            assert ws(whole, op) == ws(rest, op) > 0, (b, h, n, d, dt, op)
    # heads that do not divide the unit count: the first part has 21 x 12 = 252 chains, which the fp32 head_dim 64 plan
    # cuts in three; both parts then use the workspace, one after the other, and the query answers for the larger
    parts = [dense(lib, 21, 12, 1024, 64, F32), dense(lib, 1, 12, 1024, 64, F32)]
    assert plan(lib, 21, 12, 1024, 64, F32)[0] == 3 and plan(lib, 1, 12, 1024, 64, F32)[0] > 1
    for op in (0, 1, 2, 3):
        assert ws(dense(lib, 22, 12, 1024, 64, F32), op) == max(ws(p_, op) for p_ in parts) > 0
    # not split: too many chains for the shape, a whole number of rounds, sequences too short, five rounds, three
    # rounds of the kernels whose rule stops at two
    for b, h, n, d, dt in ((23, 16, 4096, 128, BF), (21, 16, 2048, 128, BF), (16, 16, 4096, 128, BF),
                           (20, 16, 1024, 128, BF), (20, 16, 2047, 64, F16), (36, 16, 2048, 128, BF),
                           (38, 8, 2048, 256, BF), (34, 8, 1024, 256, BF), (68, 8, 4096, 256, BF),
                           (20, 16, 2048, 96, BF), (36, 16, 4096, 96, BF), (25, 16, 4096, 64, F32),
                           (24, 16, 512, 64, F32), (34, 16, 4096, 64, F32), (48, 16, 4096, 128, BF),
                           (32, 16, 4096, 128, BF), (54, 16, 4096, 128, BF), (68, 16, 4096, 128, BF),
                           (82, 16, 4096, 128, BF), (50, 16, 2048, 128, BF), (50, 16, 4096, 96, BF),
                           (50, 16, 4096, 128, F32)):
        assert ws(dense(lib, b, h, n, d, dt), 0) == 0, (b, h, n, d, dt)
    lib.la2_set_chunk_tokens(1024)       # a caller's chunk size: one call, cut as asked
    try:
        d = dense(lib, 20, 16, 4096, 128, BF)
        assert ws(d, 0) == 20 * 16 * 4 * 128 * 128 * 4
    finally:
        lib.la2_set_chunk_tokens(0)


def test_two_call_batches_are_validated_before_the_first_launch(lib):
    """Everything either of the two calls would refuse is refused before the first one launches anything (fake
    pointers: a launch would fault)."""
    lib.la2_set_chunk_tokens(0)
    d = dense(lib, 20, 16, 4096, 128, binding.LA2_BF16)
    ref = ctypes.byref(d)
    need_f, need_b = lib.la2_workspace_bytes(ref, 0), lib.la2_workspace_bytes(ref, 1)
    assert 0 < need_f < need_b
    assert fwd(lib, d) == E_WS and fwd(lib, d, ws=P, ws_bytes=need_f - 1) == E_WS
    assert fwd(lib, d, ws=P + 16, ws_bytes=need_f) == E_WS
    assert fwd(lib, d, q=None, ws=P, ws_bytes=need_f) == E_NULL and fwd(lib, d, o=None, ws=P, ws_bytes=need_f) == E_NULL
    assert fwd(lib, d, v=P + 8, ws=P, ws_bytes=need_f) == E_ALIGN
    assert bwd(lib, d) == E_WS and bwd(lib, d, ws=P, ws_bytes=need_b - 1) == E_WS
    for i in range(8):
        ptrs = [P] * 8
        ptrs[i] = None
        assert bwd(lib, d, ptrs, ws=P, ws_bytes=need_b) == E_NULL
    fn = lambda eps=1e-6, q=P, o=P, rstd=P, ws=P, wb=need_f: lib.la2_fwd_norm(ref, q, P, P, P, eps, o, rstd, ws, wb, None)
    assert fn(eps=-1.0) == E_VALUE and fn(q=None) == E_NULL and fn(rstd=None) == E_NULL
    assert fn(o=P + 8) == E_ALIGN and fn(rstd=P + 2) == E_ALIGN
    assert fn(ws=None, wb=0) == E_WS and fn(wb=need_f - 1) == E_WS
    bn = lambda o=P, rstd=P, d_u=P, dq=P, ws=P, wb=need_b: lib.la2_bwd_norm(ref, P, P, P, o, rstd, P, P, d_u, dq, P, P, ws,
                                                                          wb, None)
    assert bn(o=None) == E_NULL and bn(rstd=None) == E_NULL and bn(d_u=None) == E_NULL and bn(dq=None) == E_NULL
    assert bn(d_u=P + 4) == E_ALIGN and bn(rstd=P + 1) == E_ALIGN
    assert bn(ws=None, wb=0) == E_WS and bn(wb=need_b - 1) == E_WS

