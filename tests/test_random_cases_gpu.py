"""Seeded random sweep over the library's options, each case against the fp64 oracle: data type, head_dim,
batch, heads, sequence length (ragged more often than not), sequence-chunk size, storage layout, decay,
start / final states and their gradients, the Norm epilogue, multi-token decode and packed variable-length batches.  The fixed cases elsewhere pick the corners
by hand; this one looks for combinations nobody thought of."""
import numpy as np
import pytest
import torch

import oracle
from paper_2401_04658_amd import binding, workloads
from parity import assert_close, to64

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
DTYPES = (torch.bfloat16, torch.float16, torch.float32)


@pytest.fixture(autouse=True)
def _defaults():
    binding.la2_set_chunk_tokens(0)
    binding.la2_set_scan_variant(0)
    yield
    binding.la2_set_chunk_tokens(0)
    binding.la2_set_scan_variant(0)


def draw_case(i, dims=(64, 128), modes=("plain", "state", "state_nofinal", "norm", "decode_multi", "varlen"), salt=90210):
    rng = np.random.default_rng(salt + i)
    dtype = DTYPES[int(rng.integers(0, 3))]
    d = int(rng.choice(list(dims)))
    b, H = int(rng.integers(1, 4)), int(rng.integers(1, 5))
    n = int(rng.choice([rng.integers(1, 70), rng.integers(70, 400), 32 * rng.integers(1, 12), rng.integers(400, 900)]))
    chunk = int(rng.choice([0, 0, 64, 128, 192, 320]))
    layout = str(rng.choice(["bhnd", "bnhd", "padded"]))
    lam = rng.choice([1.0, 0.999, 0.97, 0.8, 0.3, 1e-3], size=H).astype(np.float32)
    mode = str(rng.choice(list(modes)))
    variant = int(rng.choice([0, 1, 2]))
    return dict(dtype=dtype, d=d, b=b, H=H, n=n, chunk=chunk, layout=layout, lam=lam, mode=mode, variant=variant,
                seed=int(rng.integers(0, 1 << 30)))


def place(x, layout):
    """The tensor x [b, H, n, d] stored in the given layout on the GPU, viewed as [b, H, n, d]."""
    if layout == "bhnd":
        return x.to(DEV)
    if layout == "bnhd":
        return x.permute(0, 2, 1, 3).contiguous().to(DEV).permute(0, 2, 1, 3)
    b, H, n, d = x.shape                      # rows padded to d + 8 elements
    store = torch.zeros((b, H, n, d + 8), dtype=x.dtype, device=DEV)
    store[..., :d] = x.to(DEV)
    return store[..., :d]


@pytest.mark.parametrize("i", range(200))
def test_random_case(i):
    run_case(i, draw_case(i))


@pytest.mark.parametrize("i", range(80))
def test_random_case_head_dim_96_256(i):
    """The same sweep over the head dimensions with the plain block kernel (packed batches in the 16-bit
    types only)."""
    c = draw_case(i, dims=(96, 256), salt=41000)
    if c["mode"] == "varlen" and c["dtype"] == torch.float32:
        c["dtype"] = torch.bfloat16
    run_case(i, c)


@pytest.mark.parametrize("i", range(80))
def test_random_case_norm_with_state(i):
    """The normalised operator with state hand-over, all four head dimensions."""
    run_case(i, draw_case(i, dims=(64, 96, 128, 256), modes=("norm_state", "norm_state_nofinal"), salt=52000))


@pytest.mark.parametrize("i", range(60))
def test_random_case_packed_with_states(i):
    """Packed batches with a start state, a final state and their gradients per sequence (16-bit types, head_dim 64
    and 128), random lengths on and off the block boundaries, chunked and not."""
    c = draw_case(i, modes=("varlen_state", "varlen_state_nofinal"), salt=63000)
    if c["dtype"] == torch.float32:
        c["dtype"] = torch.bfloat16 if i % 2 else torch.float16
    run_case(i, c)


def run_case(i, c):
    dtype, d, b, H, n = c["dtype"], c["d"], c["b"], c["H"], c["n"]
    tag = "case %d %s" % (i, {k: (v if k != "lam" else v.tolist()) for k, v in c.items()})
    t = workloads.Workload("random", b, H, n, d, dtype, seed=c["seed"], backward=True).tensors()
    t["lam"] = torch.as_tensor(c["lam"])
    gen = torch.Generator(device="cpu")
    gen.manual_seed(c["seed"] + 1)
    t["kv_init"] = torch.randn((b, H, d, d), generator=gen, dtype=torch.float32) * 0.3
    t["d_kv_final"] = torch.randn((b, H, d, d), generator=gen, dtype=torch.float32) * 0.3
    g = {name: place(t[name], c["layout"]) for name in ("q", "k", "v", "d_o")}
    for name in ("lam", "kv_init", "d_kv_final"):
        g[name] = t[name].to(DEV)
    binding.la2_set_chunk_tokens(c["chunk"])
    binding.la2_set_scan_variant(c["variant"])
    q, k, v, do, lam = (to64(t[x]) for x in ("q", "k", "v", "d_o", "lam"))

    if c["mode"] in ("varlen_state", "varlen_state_nofinal"):   # packed sequences, each with states of its own
        final = c["mode"] == "varlen_state"
        rng = np.random.default_rng(c["seed"])
        lengths = [int(x) for x in rng.integers(0, n + 1, size=b + 3)]
        lengths[int(rng.integers(0, len(lengths)))] = n           # one of them reaches the stated maximum
        total = sum(lengths)
        tt = workloads.Workload("random", 1, H, max(total, 1), d, dtype, seed=c["seed"], backward=True).tensors()
        pk = {name: tt[name][0, :, :total].permute(1, 0, 2).contiguous() for name in ("q", "k", "v", "d_o")}
        gp = {name: pk[name].to(DEV) for name in pk}
        cu = torch.tensor(np.concatenate([[0], np.cumsum(lengths)]), dtype=torch.int32, device=DEV)
        init = torch.randn((len(lengths), H, d, d), generator=gen, dtype=torch.float32) * 0.3
        dfin = torch.randn((len(lengths), H, d, d), generator=gen, dtype=torch.float32) * 0.3
        o, kvf = binding.la2_fwd_varlen_state(gp["q"], gp["k"], gp["v"], g["lam"], cu, n, kv_init=init.to(DEV),
                                              want_final=final)
        dq, dk, dv, dkv0 = binding.la2_bwd_varlen_state(gp["q"], gp["k"], gp["v"], gp["d_o"], g["lam"], cu, n,
                                                        kv_init=init.to(DEV), d_kv_final=dfin.to(DEV) if final else None)
        torch.cuda.synchronize()
        lo = 0
        for s_, m in enumerate(lengths):
            i64, f64 = to64(init[s_:s_ + 1]), (to64(dfin[s_:s_ + 1]) if final else None)
            if m == 0:
                if final:
                    assert torch.equal(kvf[s_].cpu(), init[s_]), tag
                assert torch.equal(dkv0[s_].cpu(), dfin[s_] if final else torch.zeros_like(dfin[s_])), tag
                continue
            sq = {name: to64(pk[name][lo:lo + m]).transpose(1, 0, 2)[None] for name in pk}
            ro, rkvf = oracle.fwd_recurrent(sq["q"], sq["k"], sq["v"], lam, kv_init=i64, return_state=True)
            refs = oracle.bwd_recurrent_state(sq["q"], sq["k"], sq["v"], sq["d_o"], lam, kv_init=i64, d_kv_final=f64)
            assert_close(tag + " seq %d o" % s_, o[lo:lo + m].permute(1, 0, 2)[None], ro, dtype)
            if final:
                assert_close(tag + " seq %d kv_final" % s_, kvf[s_:s_ + 1], rkvf, dtype)
            for name, got, ref in zip(("dq", "dk", "dv"), (dq, dk, dv), refs[:3]):
                assert_close(tag + " seq %d %s" % (s_, name), got[lo:lo + m].permute(1, 0, 2)[None], ref, dtype)
            assert_close(tag + " seq %d d_kv_init" % s_, dkv0[s_:s_ + 1], refs[3], dtype)
            lo += m
        return
    if c["mode"] == "varlen":   # the batch rows become packed sequences of random lengths <= n
        rng = np.random.default_rng(c["seed"])
        lengths = [int(x) for x in rng.integers(0, n + 1, size=b + 2)]
        lengths[int(rng.integers(0, len(lengths)))] = n           # one of them reaches the stated maximum
        total = sum(lengths)
        tt = workloads.Workload("random", 1, H, max(total, 1), d, dtype, seed=c["seed"], backward=True).tensors()
        pk = {name: tt[name][0, :, :total].permute(1, 0, 2).contiguous() for name in ("q", "k", "v", "d_o")}
        gp = {name: pk[name].to(DEV) for name in pk}
        cu = torch.tensor(np.concatenate([[0], np.cumsum(lengths)]), dtype=torch.int32, device=DEV)
        o = binding.la2_fwd_varlen(gp["q"], gp["k"], gp["v"], g["lam"], cu, n)
        grads = binding.la2_bwd_varlen(gp["q"], gp["k"], gp["v"], gp["d_o"], g["lam"], cu, n)
        torch.cuda.synchronize()
        lo = 0
        for m in lengths:
            if m > 0:
                sq = {name: to64(pk[name][lo:lo + m]).transpose(1, 0, 2)[None] for name in pk}
                assert_close(tag + " o", o[lo:lo + m].permute(1, 0, 2)[None], oracle.fwd_direct(sq["q"], sq["k"], sq["v"], lam), dtype)
                for name, got, ref in zip(("dq", "dk", "dv"), grads, oracle.bwd_direct(sq["q"], sq["k"], sq["v"], sq["d_o"], lam)):
                    assert_close(tag + " " + name, got[lo:lo + m].permute(1, 0, 2)[None], ref, dtype)
            lo += m
        return
    if c["mode"] == "plain":
        o = binding.la2_fwd(g["q"], g["k"], g["v"], g["lam"])
        grads = binding.la2_bwd(g["q"], g["k"], g["v"], g["d_o"], g["lam"])
        torch.cuda.synchronize()
        assert_close(tag + " o", o, oracle.fwd_direct(q, k, v, lam), dtype)
        for name, got, ref in zip(("dq", "dk", "dv"), grads, oracle.bwd_direct(q, k, v, do, lam)):
            assert_close(tag + " " + name, got, ref, dtype)
    elif c["mode"] == "decode_multi":   # dense tensors only; the state is updated in place
        state = g["kv_init"].clone()
        o = binding.la2_decode_multi(g["q"].contiguous(), g["k"].contiguous(), g["v"].contiguous(), g["lam"], state)
        torch.cuda.synchronize()
        ro, rs = oracle.fwd_recurrent(q, k, v, lam, kv_init=to64(t["kv_init"]), return_state=True)
        assert_close(tag + " o", o, ro, dtype)
        assert_close(tag + " state", state, rs, dtype)
        return
    elif c["mode"] in ("norm_state", "norm_state_nofinal"):
        final = c["mode"] == "norm_state"
        eps = 1e-3
        o, rstd, kvf = binding.la2_fwd_state_norm(g["q"], g["k"], g["v"], g["lam"], eps, kv_init=g["kv_init"],
                                                  want_final=final)
        got = binding.la2_bwd_state_norm(g["q"], g["k"], g["v"], o, rstd, g["d_o"], g["lam"], kv_init=g["kv_init"],
                                         d_kv_final=g["d_kv_final"] if final else None)
        torch.cuda.synchronize()
        init64 = to64(t["kv_init"])
        ro, rr, rkvf = oracle.fwd_norm_state(q, k, v, lam, eps, init64)
        refs = oracle.bwd_norm_state(q, k, v, do, lam, eps, init64, to64(t["d_kv_final"]) if final else None)
        assert_close(tag + " o", o, ro, dtype)
        assert_close(tag + " rstd", rstd, rr, dtype)
        if final:
            assert_close(tag + " kv_final", kvf, rkvf, dtype)
        for name, x, ref in zip(("dq", "dk", "dv", "d_kv_init"), got, refs):
            assert_close(tag + " " + name, x, ref, dtype)
    elif c["mode"] == "norm":
        eps = 1e-3
        o, rstd = binding.la2_fwd_norm(g["q"], g["k"], g["v"], g["lam"], eps)
        grads = binding.la2_bwd_norm(g["q"], g["k"], g["v"], o, rstd, g["d_o"], g["lam"])
        torch.cuda.synchronize()
        ref_o, ref_r = oracle.fwd_norm(q, k, v, lam, eps)
        assert_close(tag + " o", o, ref_o, dtype)
        assert_close(tag + " rstd", rstd, ref_r, dtype)
        if n > 1:   # a single position leaves dq, dk as pure cancellation (see test_norm_gpu)
            for name, got, ref in zip(("dq", "dk", "dv"), grads, oracle.bwd_norm(q, k, v, do, lam, eps)):
                assert_close(tag + " " + name, got, ref, dtype)
    else:
        final = c["mode"] == "state"
        o, kvf = binding.la2_fwd_state(g["q"], g["k"], g["v"], g["lam"], kv_init=g["kv_init"], want_final=final)
        dq, dk, dv, dkv0 = binding.la2_bwd_state(g["q"], g["k"], g["v"], g["d_o"], g["lam"], kv_init=g["kv_init"],
                                                 d_kv_final=g["d_kv_final"] if final else None)
        torch.cuda.synchronize()
        init64 = to64(t["kv_init"])
        ro, rkvf = oracle.fwd_recurrent(q, k, v, lam, kv_init=init64, return_state=True)
        refs = oracle.bwd_recurrent_state(q, k, v, do, lam, kv_init=init64,
                                          d_kv_final=to64(t["d_kv_final"]) if final else None)
        assert_close(tag + " o", o, ro, dtype)
        if final:
            assert_close(tag + " kv_final", kvf, rkvf, dtype)
        for name, got, ref in zip(("dq", "dk", "dv", "d_kv_init"), (dq, dk, dv, dkv0), refs):
            assert_close(tag + " " + name, got, ref, dtype)
    for x in (g["q"], o):
        assert x.stride() == g["q"].stride()


def rel_diff(a, b):
    a, b = a.double(), b.double()
    return float((a - b).abs().max() / b.abs().max().clamp_min(1e-30))


@pytest.mark.parametrize("i", range(10))
def test_random_batch_above_whole_rounds_two_calls_against_one(i):
    """Batches with a few more chains than one or two per compute unit, which the library runs as two calls, against
    the same entry points run as one call (the caller's chunk size set to the whole sequence): heads that do and do
    not divide the unit count, both storage layouts, states and their gradients, the Norm pair.  The two differ by
    the rounding of the second part's chunk states only; each way is held to the oracle by the fixed cases."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    rng = np.random.default_rng(4711 + i)
    dtype = DTYPES[int(rng.integers(0, 3))]
    d = int(rng.choice([64, 128])) if dtype == torch.float32 else int(rng.choice([64, 128, 128, 96, 256]))
    H = int(rng.choice([4, 8, 12, 16, 20, 24, 32]))
    rounds = int(rng.choice([1, 1, 1, 2]))
    b = max(2, int(np.ceil(cus * (rounds + rng.uniform(0.02, 0.3)) / H)))
    n = int(rng.integers(1024, 2500)) if dtype == torch.float32 or rounds == 2 else int(rng.integers(2048, 4200))
    if rounds == 2 and dtype != torch.float32:
        n = int(rng.integers(4096, 4300))
    layout = str(rng.choice(["bhnd", "bnhd"]))
    t = workloads.Workload("case", b, H, n, d, dtype, seed=int(rng.integers(0, 1 << 30)), backward=True).tensors()
    g = {name: place(t[name], layout) for name in ("q", "k", "v", "d_o")}
    lam = t["lam"].to(DEV)
    gen = torch.Generator(device="cpu")
    gen.manual_seed(i)
    kv0 = (torch.randn((b, H, d, d), generator=gen) * 0.3).to(DEV)
    dkvf = (torch.randn((b, H, d, d), generator=gen) * 0.3).to(DEV)

    def run():
        o, kvf = binding.la2_fwd_state(g["q"], g["k"], g["v"], lam, kv_init=kv0, want_final=True)
        dq, dk, dv, dkv0 = binding.la2_bwd_state(g["q"], g["k"], g["v"], g["d_o"], lam, kv_init=kv0, d_kv_final=dkvf)
        on, rstd = binding.la2_fwd_norm(g["q"], g["k"], g["v"], lam, 1e-6)
        du = torch.empty_like(g["d_o"])
        nq, nk, nv = binding.la2_bwd_norm(g["q"], g["k"], g["v"], on, rstd, g["d_o"], lam, d_u=du)
        torch.cuda.synchronize()
        return dict(o=o, kv_final=kvf, dq=dq, dk=dk, dv=dv, d_kv_init=dkv0, o_norm=on, rstd=rstd, d_u=du, dq_norm=nq,
                    dk_norm=nk, dv_norm=nv)

    two_calls = binding.la2_chunk_plan(g["q"])[0] == 1 and binding.la2_workspace_bytes(g["q"], binding.LA2_OP_FWD) > 0
    print("case", i, dtype, (b, H, n, d), layout, "two calls" if two_calls else "one call", flush=True)
    got = run()
    binding.la2_set_chunk_tokens(n)
    assert binding.la2_workspace_bytes(g["q"], binding.LA2_OP_FWD) == 0 or n % 64 != 0
    ref = run()
    tol = {torch.float32: 2e-5, torch.bfloat16: 2e-2, torch.float16: 3e-3}[dtype]
    for name in got:
        assert torch.isfinite(got[name].float()).all(), name
        assert rel_diff(got[name], ref[name]) <= tol, (name, rel_diff(got[name], ref[name]))
