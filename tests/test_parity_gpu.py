"""GPU parity: la2_fwd / la2_bwd / la2_decode_step (through the C ABI) against the fp64 oracle,
element by element on the same seeded inputs."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2401_04658_amd import binding, workloads
from parity import TOL, assert_close, max_rel, to64

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(autouse=True)
def _auto_chunking():
    binding.la2_set_chunk_tokens(0)
    binding.la2_set_scan_variant(0)
    yield
    binding.la2_set_chunk_tokens(0)
    binding.la2_set_scan_variant(0)


def make_inputs(b, H, n, d, dtype, seed, lam=None, backward=True):
    wl = workloads.Workload("case", b, H, n, d, dtype, seed=seed, backward=backward)
    t = wl.tensors()
    if lam is not None:
        t["lam"] = torch.as_tensor(lam, dtype=torch.float32).reshape(-1).expand(H).contiguous()
    return t


def gpu(t):
    return {k: v.to(DEV) for k, v in t.items()}


def check_fwd_bwd(t, dtype, tag, backward=True):
    g = gpu(t)
    o = binding.la2_fwd(g["q"], g["k"], g["v"], g["lam"])
    torch.cuda.synchronize()
    q, k, v, lam = to64(t["q"]), to64(t["k"]), to64(t["v"]), to64(t["lam"])
    res = {"o": assert_close(tag + " o", o, oracle.fwd_direct(q, k, v, lam), dtype)}
    if backward:
        dq, dk, dv = binding.la2_bwd(g["q"], g["k"], g["v"], g["d_o"], g["lam"])
        torch.cuda.synchronize()
        rq, rk, rv = oracle.bwd_direct(q, k, v, to64(t["d_o"]), lam)
        res["dq"] = assert_close(tag + " dq", dq, rq, dtype)
        res["dk"] = assert_close(tag + " dk", dk, rk, dtype)
        res["dv"] = assert_close(tag + " dv", dv, rv, dtype)
    return res


# ---- configuration 1: forward, fp32 -------------------------------------------------------------------------
def test_config1_fwd_fp32():
    wl = workloads.CONFIG1
    check_fwd_bwd(wl.tensors(), wl.dtype, wl.name, backward=False)


# ---- configuration 2: 400M-model layer, bf16, full tensors against the O(n^2) oracle -----------------------------
def test_config2_fwd_bwd_bf16_full():
    wl = workloads.CONFIG2
    check_fwd_bwd(wl.tensors(), wl.dtype, wl.name)


# ---- small shapes spanning several tiles and ragged tails, both dtypes, both head dims ------------------------------
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16, torch.float32])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("n", [1, 31, 128, 129, 200, 384, 517])
def test_small_shapes(dtype, d, n):
    t = make_inputs(2, 3, n, d, dtype, seed=100 + n + d, lam=[0.5, 0.93, 1.0])
    check_fwd_bwd(t, dtype, "n%d d%d %s" % (n, d, dtype))


# ---- both bf16 head_dim-128 scan kernels (full-block B = 64, half-block B = 32), forced explicitly: the
# automatic choice depends on the launch size and would pick the full-block kernel for all small cases
@pytest.mark.parametrize("variant", [1, 2])
@pytest.mark.parametrize("n", [1, 31, 32, 33, 64, 95, 129, 200, 517])
def test_scan_variants_small_shapes(variant, n):
    binding.la2_set_scan_variant(variant)
    t = make_inputs(2, 3, n, 128, torch.bfloat16, seed=300 + n, lam=[0.5, 0.93, 1.0])
    check_fwd_bwd(t, torch.bfloat16, "variant%d n%d" % (variant, n))


@pytest.mark.parametrize("variant", [1, 2])
@pytest.mark.parametrize("chunk,n", [(128, 1000), (192, 1024), (256, 700)])
def test_scan_variants_chunked(variant, chunk, n):
    binding.la2_set_scan_variant(variant)
    binding.la2_set_chunk_tokens(chunk)
    t = make_inputs(1, 4, n, 128, torch.bfloat16, seed=17 * n + chunk)
    assert binding.la2_workspace_bytes(t["q"].to(DEV)) > 0
    check_fwd_bwd(t, torch.bfloat16, "variant%d chunk%d n%d" % (variant, chunk, n))


@pytest.mark.parametrize("variant", [1, 2])
def test_scan_variants_extreme_decays_and_strides(variant):
    binding.la2_set_scan_variant(variant)
    t = make_inputs(1, 3, 300, 128, torch.bfloat16, seed=23, lam=[1.0, 1e-6, 0.43])
    check_fwd_bwd(t, torch.bfloat16, "variant%d extreme decays" % variant)
    b, H, n, d = 2, 4, 260, 128
    t = make_inputs(b, H, n, d, torch.bfloat16, seed=33)
    g = {}
    for name in ("q", "k", "v", "d_o"):
        g[name] = t[name].permute(0, 2, 1, 3).contiguous().to(DEV).permute(0, 2, 1, 3)   # [b, n, H, d] storage
    lam = t["lam"].to(DEV)
    o = binding.la2_fwd(g["q"], g["k"], g["v"], lam)
    dq, dk, dv = binding.la2_bwd(g["q"], g["k"], g["v"], g["d_o"], lam)
    torch.cuda.synchronize()
    q, k, v, do, lam64 = (to64(t[x]) for x in ("q", "k", "v", "d_o", "lam"))
    assert_close("variant%d strided o" % variant, o, oracle.fwd_direct(q, k, v, lam64), torch.bfloat16)
    for name, got, ref in zip(("dq", "dk", "dv"), (dq, dk, dv), oracle.bwd_direct(q, k, v, do, lam64)):
        assert_close("variant%d strided %s" % (variant, name), got, ref, torch.bfloat16)


def test_scan_variants_agree():
    """The two kernels compute the same function: outputs differ by bf16 rounding only."""
    t = gpu(make_inputs(2, 4, 1500, 128, torch.bfloat16, seed=55))
    out = {}
    for variant in (1, 2):
        binding.la2_set_scan_variant(variant)
        out[variant] = (binding.la2_fwd(t["q"], t["k"], t["v"], t["lam"]),) + tuple(
            binding.la2_bwd(t["q"], t["k"], t["v"], t["d_o"], t["lam"]))
    torch.cuda.synchronize()
    for a, b in zip(out[1], out[2]):
        assert max_rel(to64(a), to64(b)) <= 1e-2


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16, torch.float32])
@pytest.mark.parametrize("chunk", [128, 256, 384])
@pytest.mark.parametrize("d,n", [(64, 1000), (128, 1000), (128, 1024), (64, 257)])
def test_chunked_path(dtype, chunk, d, n):
    """Forces the sequence-chunk path (state pre-pass + scan) incl. a ragged last chunk."""
    binding.la2_set_chunk_tokens(chunk)
    t = make_inputs(1, 4, n, d, dtype, seed=7 * n + d + chunk)
    if chunk < n - 128:
        assert binding.la2_workspace_bytes(t["q"].to(DEV)) > 0
    check_fwd_bwd(t, dtype, "chunk%d n%d d%d %s" % (chunk, n, d, dtype))


def test_chunking_changes_results_only_by_rounding():
    t = gpu(make_inputs(1, 2, 2048, 128, torch.bfloat16, seed=11))
    base = binding.la2_fwd(t["q"], t["k"], t["v"], t["lam"])
    binding.la2_set_chunk_tokens(512)
    chunked = binding.la2_fwd(t["q"], t["k"], t["v"], t["lam"])
    torch.cuda.synchronize()
    assert max_rel(to64(chunked), to64(base)) <= 1e-2


def test_empty_and_degenerate():
    for n in (0,):
        t = gpu(make_inputs(2, 2, n, 64, torch.bfloat16, seed=1))
        o = binding.la2_fwd(t["q"], t["k"], t["v"], t["lam"])
        g = binding.la2_bwd(t["q"], t["k"], t["v"], t["d_o"], t["lam"])
        torch.cuda.synchronize()
        assert o.shape == (2, 2, 0, 64) and all(x.shape == (2, 2, 0, 64) for x in g)
    # batch of zero
    t = gpu(make_inputs(0, 2, 64, 64, torch.bfloat16, seed=1))
    assert binding.la2_fwd(t["q"], t["k"], t["v"], t["lam"]).numel() == 0


def test_longest_sequence_one_chain_spans_4_gib():
    """Close to the longest sequence the descriptor allows for head_dim 128 in bf16: one chain of 16,777,087
    positions, just short of 4 GiB (the kernels address a chain with 32-bit byte offsets), cut into about 256
    chunks, ragged at the end.  Constant inputs and lambda = 1/2: contributions from more than 160 positions away are
    below 2^-160, so every row equals a row of the oracle's result on a 160-position window."""
    n, d, win = (1 << 24) - 129, 128, 160
    c = 0.25
    x = torch.full((1, 1, n, d), c, dtype=torch.bfloat16, device=DEV)
    lam = torch.tensor([0.5], dtype=torch.float32, device=DEV)
    w64 = np.full((1, 1, win, d), c)
    ref_o = oracle.fwd_direct(w64, w64, w64, 0.5)[0, 0]
    ref_dq, ref_dk, ref_dv = (r[0, 0] for r in oracle.bwd_direct(w64, w64, w64, w64, 0.5))
    tol = TOL[torch.bfloat16]

    def check(name, got, ref, forward):
        got = got[0, 0]
        scale = float(np.max(np.abs(ref)))
        if forward:   # the first rows, then the steady state
            head, steady, rest = got[:win], ref[win - 1], got[win - 1:]
            edge_ref = ref
        else:         # the last rows (aligned at the end), and the steady state before them
            head, steady, rest = got[n - win:], ref[0], got[:n - win + 1]
            edge_ref = ref
        assert np.max(np.abs(to64(head) - edge_ref)) <= tol * scale, name + " edge rows"
        steady_t = torch.as_tensor(steady, dtype=torch.float32, device=DEV)
        err = (rest.float() - steady_t).abs().max().item()
        assert err <= tol * scale, "%s steady state: %.3e" % (name, err / scale)

    o = binding.la2_fwd(x, x, x, lam)
    torch.cuda.synchronize()
    check("o", o, ref_o, True)
    del o
    dq, dk, dv = binding.la2_bwd(x, x, x, x, lam)
    torch.cuda.synchronize()
    check("dq", dq, ref_dq, True)
    check("dk", dk, ref_dk, False)
    check("dv", dv, ref_dv, False)
    # two more positions do not fit the 32-bit chain offsets: refused on the host
    y = torch.empty((1, 1, n + 2, d), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(binding.LA2Error):
        binding.la2_fwd(y, y, y, lam)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
def test_unscaled_values_and_slow_decay(dtype):
    """V and dO of unit variance (configuration 4's value scale) with decays close to 1 over a long sequence: the
    running state grows to its largest, which is what the 16-bit state operand (fp16: range 65504) has to hold."""
    wl = workloads.Workload("unscaled", 1, 3, 3000, 128, dtype, seed=71, v_scale=1.0)
    t = wl.tensors()
    t["lam"] = torch.tensor([1.0, 0.9999, 0.99], dtype=torch.float32)
    check_fwd_bwd(t, dtype, "unscaled %s" % dtype)


def test_extreme_decays():
    """lambda = 1 (pure causal prefix sum) and a very small lambda (only the diagonal survives)."""
    for dtype in (torch.bfloat16, torch.float16, torch.float32):
        t = make_inputs(1, 3, 300, 64, dtype, seed=21, lam=[1.0, 1e-6, 0.43])
        check_fwd_bwd(t, dtype, "extreme decays %s" % dtype)


def test_strided_layout():
    """[b, n, H, d] storage viewed as [b, H, n, d]: strides go through the descriptor."""
    b, H, n, d = 2, 4, 260, 128
    for dtype in (torch.bfloat16, torch.float16, torch.float32):
        t = make_inputs(b, H, n, d, dtype, seed=31)
        g = {}
        for name in ("q", "k", "v", "d_o"):
            store = t[name].permute(0, 2, 1, 3).contiguous().to(DEV)  # [b, n, H, d]
            g[name] = store.permute(0, 2, 1, 3)                       # view [b, H, n, d]
            assert not g[name].is_contiguous()
        lam = t["lam"].to(DEV)
        o = binding.la2_fwd(g["q"], g["k"], g["v"], lam)
        dq, dk, dv = binding.la2_bwd(g["q"], g["k"], g["v"], g["d_o"], lam)
        torch.cuda.synchronize()
        q, k, v, do, lam64 = (to64(t[x]) for x in ("q", "k", "v", "d_o", "lam"))
        assert_close("strided o", o, oracle.fwd_direct(q, k, v, lam64), dtype)
        for name, got, ref in zip(("dq", "dk", "dv"), (dq, dk, dv), oracle.bwd_direct(q, k, v, do, lam64)):
            assert_close("strided " + name, got, ref, dtype)


SPLIT_CASES = [(b, H, n, d, st, dt) for dt in (torch.bfloat16, torch.float16)
               for b, H, n, d, st in ((20, 16, 2048, 128, False), (18, 16, 2100, 64, True), (11, 32, 4096, 128, False))]
SPLIT_CASES += [(36, 16, 4096, 128, False, torch.float16), (34, 16, 4100, 64, True, torch.bfloat16),   # two rounds
                (50, 16, 4096, 64, False, torch.bfloat16),                                           # three
                (34, 8, 2048, 256, False, torch.bfloat16), (36, 8, 2100, 256, True, torch.float16),
                (18, 16, 2048, 96, False, torch.float16), (34, 16, 4096, 96, False, torch.bfloat16),
                (24, 16, 1024, 64, False, torch.float32), (20, 16, 1100, 128, True, torch.float32),
                (34, 16, 2048, 128, False, torch.float32)]


@pytest.mark.parametrize("b,H,n,d,strided,dtype", SPLIT_CASES)
def test_batches_a_little_above_the_compute_unit_count(b, H, n, d, strided, dtype):
    """A few more chains than one (or two) per compute unit: la2_fwd / la2_bwd run the rows that make whole rounds
    un-chunked and the remaining rows in chunks, as two calls on the same stream.  Chains on both sides of that cut,
    at sampled positions (block and chunk borders among them) against the O(n^2) oracle, and the Euler identity over
    everything."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    t = make_inputs(b, H, n, d, dtype, seed=53)
    g = {}
    for name in ("q", "k", "v", "d_o"):
        if strided:
            g[name] = t[name].permute(0, 2, 1, 3).contiguous().to(DEV).permute(0, 2, 1, 3)
        else:
            g[name] = t[name].to(DEV)
    lam = t["lam"].to(DEV)
    cut = min(max((b * H // cus) * cus // H, 1), b - 1)
    nch, chunk = binding.la2_chunk_plan(g["q"][cut:])
    if cus == 256:     # the split is what runs: its workspace is that of the remaining rows' plan
        assert nch > 1
        assert binding.la2_workspace_bytes(g["q"]) == binding.la2_workspace_bytes(g["q"][cut:]) > 0
    o = binding.la2_fwd(g["q"], g["k"], g["v"], lam)
    dq, dk, dv = binding.la2_bwd(g["q"], g["k"], g["v"], g["d_o"], lam)
    torch.cuda.synchronize()
    rng = np.random.default_rng(53)
    tol = TOL[dtype]
    borders = [c * chunk + e for c in range(1, nch) for e in (-1, 0, 1)]
    for row in sorted({0, cut - 1, cut, b - 1}):
        for h in (0, H // 2, H - 1):
            rows = np.array(sorted(set(sampled_rows(n, rng).tolist() + [r for r in borders if 0 <= r < n])), dtype=np.int64)
            q, k, v, do = (to64(t[x][row, h]) for x in ("q", "k", "v", "d_o"))
            lam_h = float(t["lam"][h].double())
            ref_o = oracle.fwd_rows(q, k, v, lam_h, rows)
            ref_dq, ref_dk, ref_dv = oracle.bwd_rows(q, k, v, do, lam_h, rows)
            for name, got, ref in (("o", o, ref_o), ("dq", dq, ref_dq), ("dk", dk, ref_dk), ("dv", dv, ref_dv)):
                x = to64(got[row, h])[rows]
                assert np.all(np.isfinite(x))
                err = float(np.max(np.abs(x - ref))) / float(np.max(np.abs(ref)))
                assert err <= tol, "%s (b%d h%d): %.3e" % (name, row, h, err)
    f64 = lambda x: x.to(torch.float64)
    L = torch.sum(f64(o) * f64(g["d_o"])).item()
    scale = torch.sum(torch.abs(f64(o) * f64(g["d_o"]))).item()
    for name, grad, x in (("dq", dq, g["q"]), ("dk", dk, g["k"]), ("dv", dv, g["v"])):
        assert abs(torch.sum(f64(grad) * f64(x)).item() - L) <= 2e-3 * scale, name
    for x in (o, dq, dk, dv):
        assert torch.isfinite(x.float()).all()


def test_deterministic_and_causal():
    t = gpu(make_inputs(2, 2, 700, 128, torch.bfloat16, seed=41))
    o1 = binding.la2_fwd(t["q"], t["k"], t["v"], t["lam"])
    o2 = binding.la2_fwd(t["q"], t["k"], t["v"], t["lam"])
    g1 = binding.la2_bwd(t["q"], t["k"], t["v"], t["d_o"], t["lam"])
    g2 = binding.la2_bwd(t["q"], t["k"], t["v"], t["d_o"], t["lam"])
    torch.cuda.synchronize()
    assert torch.equal(o1, o2)
    assert all(torch.equal(a, b) for a, b in zip(g1, g2))
    # changing tokens after position `cut` must leave earlier outputs bit-identical
    cut = 300
    q2, k2, v2 = t["q"].clone(), t["k"].clone(), t["v"].clone()
    for x in (q2, k2, v2):
        x[:, :, cut:] += 1.0
    o3 = binding.la2_fwd(q2, k2, v2, t["lam"])
    torch.cuda.synchronize()
    assert torch.equal(o1[:, :, :cut], o3[:, :, :cut])
    # changing dO before `cut` must leave dK, dV from `cut` on bit-identical
    do2 = t["d_o"].clone()
    do2[:, :, :cut] -= 2.0
    g3 = binding.la2_bwd(t["q"], t["k"], t["v"], do2, t["lam"])
    torch.cuda.synchronize()
    assert torch.equal(g1[1][:, :, cut:], g3[1][:, :, cut:])
    assert torch.equal(g1[2][:, :, cut:], g3[2][:, :, cut:])


# ---- full-size configurations 3 and 4: sampled rows against the O(n^2) oracle + Euler identity ----------------------
def sampled_rows(n, rng, count=24):
    fixed = [0, 1, 127, 128, 129, n // 2 - 1, n // 2, n - 129, n - 128, n - 2, n - 1]
    rnd = rng.integers(0, n, size=count - len(fixed)).tolist()
    return np.array(sorted(set(int(r) for r in fixed + rnd if 0 <= r < n)), dtype=np.int64)


def check_sampled(wl):
    t = wl.tensors()
    g = gpu(t)
    o = binding.la2_fwd(g["q"], g["k"], g["v"], g["lam"])
    dq, dk, dv = binding.la2_bwd(g["q"], g["k"], g["v"], g["d_o"], g["lam"])
    torch.cuda.synchronize()
    rng = np.random.default_rng(wl.seed)
    H = wl.heads
    tol = TOL[wl.dtype]
    for b, h in ((0, 0), (wl.batch - 1, H // 2), (0, H - 1)):
        rows = sampled_rows(wl.seqlen, rng)
        q, k, v, do = (to64(t[x][b, h]) for x in ("q", "k", "v", "d_o"))
        lam = float(t["lam"][h].double())
        ref_o = oracle.fwd_rows(q, k, v, lam, rows)
        ref_dq, ref_dk, ref_dv = oracle.bwd_rows(q, k, v, do, lam, rows)
        for name, got, ref in (("o", o, ref_o), ("dq", dq, ref_dq), ("dk", dk, ref_dk), ("dv", dv, ref_dv)):
            x = to64(got[b, h])[rows]
            # normalise by the largest magnitude of the sampled oracle rows of this chain
            err = float(np.max(np.abs(x - ref))) / float(np.max(np.abs(ref)))
            assert np.all(np.isfinite(x))
            assert err <= tol, "%s %s (b%d h%d): %.3e" % (wl.name, name, b, h, err)
    # Euler identity on the full GPU outputs: <dQ,Q> = <dK,K> = <dV,V> = <dO,O>
    f64 = lambda x: x.to(torch.float64)
    L = torch.sum(f64(o) * f64(g["d_o"])).item()
    scale = torch.sum(torch.abs(f64(o) * f64(g["d_o"]))).item()
    for name, grad, x in (("dq", dq, g["q"]), ("dk", dk, g["k"]), ("dv", dv, g["v"])):
        val = torch.sum(f64(grad) * f64(x)).item()
        assert abs(val - L) <= 2e-3 * scale, "%s Euler identity: %g vs %g" % (name, val, L)
    for x in (o, dq, dk, dv):
        assert torch.isfinite(x.float()).all()


@pytest.mark.parametrize("idx", range(4))
def test_config3_sweep_sampled(idx):
    check_sampled(workloads.CONFIG3[idx])


def test_config4_3b_layer_sampled():
    check_sampled(workloads.CONFIG4)


# ---- configuration 5: decode ------------------------------------------------------------------------------------
def run_decode(wl, batch, steps):
    g = wl.generator()
    H, d = wl.heads, wl.head_dim
    state0 = wl.initial_state(g)[:batch].contiguous()
    lam = wl.decay()
    kv_gpu = state0.to(DEV)
    kv_ref = state0.double().numpy().copy()
    lam_gpu, lam64 = lam.to(DEV), lam.double().numpy()
    worst = 0.0
    for step in range(steps):
        q, k, v = (x[:batch].contiguous() for x in wl.token(g))
        o = binding.la2_decode_step(q.to(DEV), k.to(DEV), v.to(DEV), lam_gpu, kv_gpu)
        ref = oracle.decode_step(to64(q), to64(k), to64(v), lam64, kv_ref)
        if step < 4 or step % 97 == 0 or step == steps - 1:
            worst = max(worst, max_rel(to64(o), ref))
            assert worst <= TOL[torch.bfloat16], "decode o at step %d: %.3e" % (step, worst)
    torch.cuda.synchronize()
    m = max_rel(to64(kv_gpu), kv_ref)
    assert m <= 1e-5, "decode state after %d steps: %.3e" % (steps, m)


def test_config5_decode_full_batch_few_steps():
    run_decode(workloads.CONFIG5, workloads.CONFIG5.batch, 3)


def test_config5_decode_1024_steps_one_batch_row():
    run_decode(workloads.CONFIG5, 1, workloads.CONFIG5.steps)


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16, torch.float32])
def test_decode_matches_forward(d, dtype):
    """n decode steps from a zero state reproduce the forward output row by row."""
    b, H, n = 2, 3, 40
    t = make_inputs(b, H, n, d, dtype, seed=51, backward=False)
    g = gpu(t)
    kv = torch.zeros(b, H, d, d, dtype=torch.float32, device=DEV)
    rows = []
    for s in range(n):
        rows.append(binding.la2_decode_step(g["q"][:, :, s].contiguous(), g["k"][:, :, s].contiguous(),
                                            g["v"][:, :, s].contiguous(), g["lam"], kv))
    torch.cuda.synchronize()
    o = torch.stack(rows, dim=2)
    q, k, v, lam = (to64(t[x]) for x in ("q", "k", "v", "lam"))
    assert_close("decode-as-forward", o, oracle.fwd_direct(q, k, v, lam), dtype)
    _, kvf = oracle.fwd_recurrent(q, k, v, lam, return_state=True)
    assert max_rel(to64(kv), kvf) <= 1e-5


def test_hip_graph_capture_and_replay():
    """The library allocates nothing and never synchronises, so a forward + backward (incl. the chunked
    path with its workspace) can be captured into a HIP graph.  Replays, with eager work and
    synchronisations between them, must reproduce the eager results bit for bit."""
    # the last shape runs as two calls (288 chains on 256 units): an un-chunked part and a chunked one per pass
    for (b, H, n, d) in ((2, 4, 700, 128), (1, 2, 2048, 128), (1, 4, 900, 64), (18, 16, 2048, 64)):
        t = gpu(make_inputs(b, H, n, d, torch.bfloat16, seed=61 + n))
        ws = torch.empty(max(256, binding.la2_workspace_bytes(t["q"], binding.LA2_OP_BWD)), dtype=torch.uint8,
                         device=DEV)
        o = torch.empty_like(t["q"])
        grads = tuple(torch.empty_like(t["q"]) for _ in range(3))
        eager_o = binding.la2_fwd(t["q"], t["k"], t["v"], t["lam"], workspace=ws).clone()
        eager_g = [x.clone() for x in binding.la2_bwd(t["q"], t["k"], t["v"], t["d_o"], t["lam"], workspace=ws)]
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            # warm-up on the capture stream, then capture
            binding.la2_fwd(t["q"], t["k"], t["v"], t["lam"], out=o, workspace=ws)
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                binding.la2_fwd(t["q"], t["k"], t["v"], t["lam"], out=o, workspace=ws)
                binding.la2_bwd(t["q"], t["k"], t["v"], t["d_o"], t["lam"], out=grads, workspace=ws)
        torch.cuda.current_stream().wait_stream(side)
        for replay in range(3):
            o.fill_(float("nan"))
            for x in grads:
                x.fill_(float("nan"))
            ws.random_(0, 255)                      # the workspace carries nothing between calls
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(o, eager_o), (n, d, replay)
            for got, ref in zip(grads, eager_g):
                assert torch.equal(got, ref), (n, d, replay)
            # eager work between replays
            assert torch.equal(binding.la2_fwd(t["q"], t["k"], t["v"], t["lam"], workspace=ws), eager_o)
            torch.cuda.synchronize()


def test_hip_graph_capture_of_the_other_entry_points():
    """Segments with state hand-over (ragged: block kernels + short-run kernels), the normalised operator,
    multi-token decode and a decode step in one captured graph; replays reproduce the eager results bit for bit."""
    b, H, n, d = 2, 3, 300, 128
    t = gpu(make_inputs(b, H, n, d, torch.bfloat16, seed=77))
    gen = torch.Generator(device="cpu")
    gen.manual_seed(78)
    kv0 = (torch.randn((b, H, d, d), generator=gen) * 0.3).to(DEV)
    dkvn = (torch.randn((b, H, d, d), generator=gen) * 0.3).to(DEV)
    ws = torch.empty(max(256, binding.la2_workspace_bytes(t["q"], binding.LA2_OP_BWD_STATE)), dtype=torch.uint8, device=DEV)
    T = 8
    qm, km, vm = (t[x][:, :, :T].contiguous() for x in ("q", "k", "v"))

    def run(out):
        o, kvf = binding.la2_fwd_state(t["q"], t["k"], t["v"], t["lam"], kv_init=kv0, out=out["o"], kv_final=out["kvf"],
                                       workspace=ws)
        binding.la2_bwd_state(t["q"], t["k"], t["v"], t["d_o"], t["lam"], kv_init=kv0, d_kv_final=dkvn,
                              out=out["grads"], d_kv_init=out["dkv0"], workspace=ws)
        binding.la2_fwd_norm(t["q"], t["k"], t["v"], t["lam"], 1e-5, out=out["on"], rstd=out["rstd"], workspace=ws)
        binding.la2_bwd_norm(t["q"], t["k"], t["v"], out["on"], out["rstd"], t["d_o"], t["lam"], out=out["gn"],
                             d_u=out["du"], workspace=ws)
        out["state"].copy_(kv0)
        binding.la2_decode_multi(qm, km, vm, t["lam"], out["state"], out=out["om"])
        binding.la2_decode_step(qm[:, :, 0].contiguous(), km[:, :, 0].contiguous(), vm[:, :, 0].contiguous(), t["lam"],
                                out["state"], out=out["o1"])

    def buffers():
        like = lambda: torch.empty_like(t["q"])
        return {"o": like(), "kvf": torch.empty_like(kv0), "grads": (like(), like(), like()), "dkv0": torch.empty_like(kv0),
                "on": like(), "rstd": torch.empty((b, H, n), device=DEV), "gn": (like(), like(), like()), "du": like(),
                "state": torch.empty_like(kv0), "om": torch.empty_like(qm), "o1": torch.empty_like(qm[:, :, 0])}

    def flat(out):
        return [out["o"], out["kvf"], *out["grads"], out["dkv0"], out["on"], out["rstd"], *out["gn"], out["du"],
                out["state"], out["om"], out["o1"]]

    # .contiguous() inside run() allocates: do those once outside the capture by warming up first
    eager = buffers()
    run(eager)
    torch.cuda.synchronize()
    captured = buffers()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(captured)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run(captured)
    torch.cuda.current_stream().wait_stream(side)
    for replay in range(3):
        for x in flat(captured):
            x.fill_(float("nan"))
        ws.random_(0, 255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (got, ref) in enumerate(zip(flat(captured), flat(eager))):
            assert torch.equal(got, ref), (replay, i)
        scratch = buffers()            # eager work between the replays
        run(scratch)
        torch.cuda.synchronize()


# ---- the O(n^2 d) left-product comparison kernel computes the same forward pass ---------------------------------------
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("n", [1, 31, 64, 128, 129, 200, 517, 1000])
def test_left_product_kernel_small_shapes(d, n):
    t = make_inputs(2, 3, n, d, torch.bfloat16, seed=400 + n + d, lam=[0.5, 0.93, 1.0])
    g = gpu(t)
    o = binding.la2_left_product_fwd(g["q"], g["k"], g["v"], g["lam"])
    torch.cuda.synchronize()
    ref = oracle.fwd_direct(to64(t["q"]), to64(t["k"]), to64(t["v"]), to64(t["lam"]))
    assert_close("left product n%d d%d" % (n, d), o, ref, torch.bfloat16)


def test_left_product_kernel_config2_and_extreme_decays():
    wl = workloads.CONFIG2
    t = wl.tensors()
    g = gpu(t)
    o = binding.la2_left_product_fwd(g["q"], g["k"], g["v"], g["lam"])
    torch.cuda.synchronize()
    assert_close("left product config2", o, oracle.fwd_direct(to64(t["q"]), to64(t["k"]), to64(t["v"]), to64(t["lam"])),
                 torch.bfloat16)
    t = make_inputs(1, 3, 300, 128, torch.bfloat16, seed=24, lam=[1.0, 1e-6, 0.43])
    g = gpu(t)
    o = binding.la2_left_product_fwd(g["q"], g["k"], g["v"], g["lam"])
    torch.cuda.synchronize()
    assert_close("left product extreme decays", o,
                 oracle.fwd_direct(to64(t["q"]), to64(t["k"]), to64(t["v"]), to64(t["lam"])), torch.bfloat16)
    with pytest.raises(binding.LA2Error):
        f = gpu(make_inputs(1, 1, 64, 64, torch.float32, seed=1))
        binding.la2_left_product_fwd(f["q"], f["k"], f["v"], f["lam"])


# ---- ... and its backward form the same gradients ------------------------------------------------------------------
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("n", [1, 31, 64, 128, 129, 200, 517, 1000])
def test_left_product_backward_small_shapes(d, n):
    t = make_inputs(2, 3, n, d, torch.bfloat16, seed=450 + n + d, lam=[0.5, 0.93, 1.0])
    g = gpu(t)
    dq, dk, dv = binding.la2_left_product_bwd(g["q"], g["k"], g["v"], g["d_o"], g["lam"])
    torch.cuda.synchronize()
    refs = oracle.bwd_direct(to64(t["q"]), to64(t["k"]), to64(t["v"]), to64(t["d_o"]), to64(t["lam"]))
    for name, got, ref in zip(("dq", "dk", "dv"), (dq, dk, dv), refs):
        assert_close("left product %s n%d d%d" % (name, n, d), got, ref, torch.bfloat16)


def test_left_product_backward_config2_and_extreme_decays():
    for t in (workloads.CONFIG2.tensors(), make_inputs(1, 3, 300, 128, torch.bfloat16, seed=25, lam=[1.0, 1e-6, 0.43])):
        g = gpu(t)
        got = binding.la2_left_product_bwd(g["q"], g["k"], g["v"], g["d_o"], g["lam"])
        torch.cuda.synchronize()
        refs = oracle.bwd_direct(to64(t["q"]), to64(t["k"]), to64(t["v"]), to64(t["d_o"]), to64(t["lam"]))
        for name, x, ref in zip(("dq", "dk", "dv"), got, refs):
            assert_close("left product bwd " + name, x, ref, torch.bfloat16)
    # strided layout ([b, n, H, d] storage)
    t = make_inputs(2, 3, 333, 128, torch.bfloat16, seed=26)
    g = {}
    for name in ("q", "k", "v", "d_o"):
        g[name] = t[name].permute(0, 2, 1, 3).contiguous().to(DEV).permute(0, 2, 1, 3)
    lam = t["lam"].to(DEV)
    got = binding.la2_left_product_bwd(g["q"], g["k"], g["v"], g["d_o"], lam)
    torch.cuda.synchronize()
    refs = oracle.bwd_direct(to64(t["q"]), to64(t["k"]), to64(t["v"]), to64(t["d_o"]), to64(t["lam"]))
    for name, x, ref in zip(("dq", "dk", "dv"), got, refs):
        assert_close("left product bwd strided " + name, x, ref, torch.bfloat16)
    with pytest.raises(binding.LA2Error):
        f = gpu(make_inputs(1, 1, 64, 64, torch.float16, seed=1))
        binding.la2_left_product_bwd(f["q"], f["k"], f["v"], f["d_o"], f["lam"])
