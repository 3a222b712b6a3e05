"""la2_fwd_noalloc (the entry point that allocates nothing) against la2_fwd, through the C ABI.

Two calls in a row on the same GPU share the library's built-in scratch; the second is smaller, so whatever the
first left behind in the scratch must not leak into it.  Same kernels, same chunk plan: the results are
bit-identical to la2_fwd's, which the other GPU tests hold to the oracle (and the first case is checked
against the oracle here as well)."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2401_04658_amd import binding, workloads
from parity import assert_close, to64

pytestmark = pytest.mark.gpu

CASES = [
    # (batch, heads, seqlen, head_dim, dtype): sequence-chunked launches (few chains), larger then smaller
    (1, 8, 8192, 128, torch.bfloat16),
    (1, 4, 4096, 128, torch.bfloat16),
    (2, 3, 2500, 64, torch.bfloat16),
    (1, 2, 3000, 128, torch.float32),
    (64, 4, 512, 128, torch.bfloat16),   # chains fill the device: no scratch needed at all
    # a few more chains than compute units: the first rows whole, the other rows in chunks whose states take the
    # scratch (all 16 MiB of it on a device of 256 units)
    (20, 16, 2048, 128, torch.bfloat16),
    # the same kind at head_dim 256: the other rows' chunk states (64 MiB) do not fit the scratch, so the batch runs
    # as one un-chunked call here, which needs none
    (34, 8, 2048, 256, torch.bfloat16),
]


def test_noalloc_matches_la2_fwd_two_calls_in_a_row():
    dev = torch.device("cuda:0")
    for i, (b, h, n, d, dt) in enumerate(CASES):
        wl = workloads.Workload("noalloc%d" % i, b, h, n, d, dt, seed=70 + i)
        t = wl.tensors()
        g = {k_: v_.to(dev) for k_, v_ in t.items()}
        print("case", i, (b, h, n, d, dt), "workspace bytes", binding.la2_workspace_bytes(g["q"]), flush=True)
        if i < 4:
            assert binding.la2_workspace_bytes(g["q"]) > 0, "case is meant to use the scratch"
        if i == 6 and binding.la2_workspace_bytes(g["q"]) > (16 << 20):   # la2_fwd as one call as well
            binding.la2_set_chunk_tokens(n)
        ref = binding.la2_fwd(g["q"], g["k"], g["v"], g["lam"])
        binding.la2_set_chunk_tokens(0)
        out = torch.full_like(g["q"], float("nan"))
        binding.la2_fwd_noalloc(g["q"], g["k"], g["v"], g["lam"], out)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.uint8), ref.view(torch.uint8)), "case %d differs from la2_fwd" % i
        if i == 0:
            q, k, v, lam = (to64(t[x]) for x in ("q", "k", "v", "lam"))
            assert_close("o", out, oracle.fwd_recurrent(q, k, v, lam), dt)


def test_noalloc_refuses_what_the_scratch_cannot_hold():
    lib = binding.load()
    desc = binding.la2_desc()
    lib.la2_desc_dense(ctypes.byref(desc), 1, 64, 1 << 16, 256, binding.LA2_BF16)   # four chunks at head_dim 256: 64 MiB of states
    assert lib.la2_workspace_bytes(ctypes.byref(desc), 0) > (16 << 20)
    P = ctypes.c_void_p(0x10000)   # never dereferenced: the call is refused on the host
    assert lib.la2_fwd_noalloc(ctypes.byref(desc), P, P, P, P, P, None) == 5   # LA2_ERR_WORKSPACE
