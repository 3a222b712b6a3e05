"""GPU parity of la2_fwd_varlen_state / la2_bwd_varlen_state (packed sequences as segments with state hand-over)
against the fp64 oracle: every sequence is a chain of its own with its own start state, so the reference is the
oracle's recurrent form applied sequence by sequence (Sec. 3.2.1, recursive form; Sec. 3.2.2)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2401_04658_amd import binding, workloads
from parity import assert_close, to64

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(autouse=True)
def _defaults():
    binding.la2_set_chunk_tokens(0)
    binding.la2_set_scan_variant(0)
    yield
    binding.la2_set_chunk_tokens(0)
    binding.la2_set_scan_variant(0)


def packed_inputs(lengths, H, d, dtype, seed, lam=None):
    total = int(sum(lengths))
    t = workloads.Workload("packed", 1, H, max(total, 1), d, dtype, seed=seed, backward=True).tensors()
    out = {name: t[name][0, :, :total].permute(1, 0, 2).contiguous() for name in ("q", "k", "v", "d_o")}
    out["lam"] = t["lam"] if lam is None else torch.as_tensor(lam, dtype=torch.float32).reshape(-1).expand(H).contiguous()
    g = torch.Generator(device="cpu")
    g.manual_seed(seed + 1000)
    # states of the size a few hundred tokens of such inputs build up; gradients of the same order
    out["kv_init"] = torch.randn((len(lengths), H, d, d), generator=g, dtype=torch.float32) * 0.3
    out["d_kv_final"] = torch.randn((len(lengths), H, d, d), generator=g, dtype=torch.float32) * 0.3
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    return out, torch.from_numpy(cu)


def check_packed_state(lengths, H, d, dtype, seed, lam=None, use_init=True, use_final=True, total_hint=True):
    t, cu = packed_inputs(lengths, H, d, dtype, seed, lam)
    g = {k: v.to(DEV) for k, v in t.items()}
    cu_g = cu.to(DEV)
    max_len = int(max(lengths)) if len(lengths) else 0
    kv_init = g["kv_init"] if use_init else None
    d_fin = g["d_kv_final"] if use_final else None
    o = torch.full_like(g["q"], float("nan"))
    grads = tuple(torch.full_like(g["q"], float("nan")) for _ in range(3))
    kvf = torch.full_like(g["kv_init"], float("nan"))
    dkv0 = torch.full_like(g["kv_init"], float("nan"))
    binding.la2_fwd_varlen_state(g["q"], g["k"], g["v"], g["lam"], cu_g, max_len, kv_init=kv_init, want_final=use_final,
                                 out=o, kv_final=kvf)
    binding.la2_bwd_varlen_state(g["q"], g["k"], g["v"], g["d_o"], g["lam"], cu_g, max_len, kv_init=kv_init,
                                 d_kv_final=d_fin, out=grads, d_kv_init=dkv0)
    torch.cuda.synchronize()
    lam64 = to64(t["lam"])
    for b, n in enumerate(lengths):
        lo, hi = int(cu[b]), int(cu[b + 1])
        tag = "lengths %s seq %d (n %d) d%d %s init %s final %s" % (list(lengths)[:12], b, n, d, dtype, use_init, use_final)
        init64 = to64(t["kv_init"][b:b + 1]) if use_init else None
        fin64 = to64(t["d_kv_final"][b:b + 1]) if use_final else None
        if n == 0:   # the state and its gradient pass through
            if use_final:
                assert torch.equal(kvf[b].cpu(), t["kv_init"][b] if use_init else torch.zeros_like(t["kv_init"][b])), tag
            assert torch.equal(dkv0[b].cpu(), t["d_kv_final"][b] if use_final else torch.zeros_like(t["kv_init"][b])), tag
            continue
        seq = {name: to64(t[name][lo:hi]).transpose(1, 0, 2)[None] for name in ("q", "k", "v", "d_o")}   # [1, H, n, d]
        ro, rkvf = oracle.fwd_recurrent(seq["q"], seq["k"], seq["v"], lam64, kv_init=init64, return_state=True)
        rdq, rdk, rdv, rdkv0 = oracle.bwd_recurrent_state(seq["q"], seq["k"], seq["v"], seq["d_o"], lam64,
                                                          kv_init=init64, d_kv_final=fin64)
        assert_close(tag + " o", o[lo:hi].permute(1, 0, 2)[None], ro, dtype)
        if use_final:
            assert_close(tag + " kv_final", kvf[b:b + 1], rkvf, dtype)
        for name, got, ref in zip(("dq", "dk", "dv"), grads, (rdq, rdk, rdv)):
            assert_close(tag + " " + name, got[lo:hi].permute(1, 0, 2)[None], ref, dtype)
        assert_close(tag + " d_kv_init", dkv0[b:b + 1], rdkv0, dtype)
    if not use_final:
        assert torch.isnan(kvf).all()   # not asked for: not written


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("d", [64, 128])
def test_mixed_lengths_with_all_states(dtype, d):
    """Lengths on and off the block boundaries (32 positions), a single position, none at all."""
    check_packed_state([70, 0, 1, 31, 32, 33, 100, 517, 64, 3, 96], 3, d, dtype, seed=900 + d, lam=[0.5, 0.93, 1.0])


@pytest.mark.parametrize("d", [64, 128])
def test_either_end_only(d):
    lengths = [45, 64, 0, 130, 7]
    check_packed_state(lengths, 2, d, torch.bfloat16, seed=910 + d, lam=[0.8, 0.99], use_final=False)
    check_packed_state(lengths, 2, d, torch.bfloat16, seed=911 + d, lam=[0.8, 0.99], use_init=False)


@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.bfloat16, 64), (torch.float16, 128)])
@pytest.mark.parametrize("chunk", [64, 192])
def test_mixed_lengths_chunked(dtype, d, chunk):
    """Long sequences cut into sequence chunks (compact grid): their start states enter the chunk-state scan, their
    final states come from their own last chunk, whose last block is ragged."""
    binding.la2_set_chunk_tokens(chunk)
    check_packed_state([700, 130, 64, 1000, 5, 0, 383, 192], 2, d, dtype, seed=920 + d + chunk, lam=[0.8, 0.99])


def test_small_lambda_keeps_the_ragged_end_state_exact():
    """A decay so strong that lambda^31 underflows in fp32: the ragged block's weights are formed from
    non-negative exponents only, never as a correction by a negative power."""
    check_packed_state([33, 47, 1, 95], 2, 128, torch.bfloat16, seed=930, lam=[0.001, 0.05])


@pytest.mark.parametrize("d", [64, 128])
def test_skewed_lengths_with_many_chains(d):
    """Chains enough to fill the device and one long sequence: planned from the total (chunks of a quarter of the
    longest), short sequences single chunks among the long one's."""
    lengths = [61] * 150 + [2048 - 17] + [37] * 120 + [300, 0, 1]
    check_packed_state(lengths, 2, d, torch.bfloat16, seed=940 + d, lam=[0.7, 0.995])


def test_packed_prefill_then_decode_continues_the_sequences():
    """What the final states are for: a packed prefill, then decode steps from its states, equal the oracle's
    forward pass over each sequence with the decoded positions appended."""
    H, d, steps = 2, 128, 3
    lengths = [50, 0, 131, 64]
    dtype = torch.bfloat16
    ext = [n + steps for n in lengths]
    t, cu_ext = packed_inputs(ext, H, d, dtype, seed=950, lam=[0.9, 0.97])
    # the prompts: the first n positions of every extended sequence, packed
    rows = np.concatenate([np.arange(int(cu_ext[b]), int(cu_ext[b]) + n) for b, n in enumerate(lengths)]).astype(np.int64)
    g = {name: t[name][torch.from_numpy(rows)].contiguous().to(DEV) for name in ("q", "k", "v")}
    lam = t["lam"].to(DEV)
    cu = torch.from_numpy(np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)).to(DEV)
    _, kv = binding.la2_fwd_varlen_state(g["q"], g["k"], g["v"], lam, cu, max(lengths))
    lam64 = to64(t["lam"])
    ref = []
    for b, n in enumerate(ext):
        lo, hi = int(cu_ext[b]), int(cu_ext[b + 1])
        seq = {name: to64(t[name][lo:hi]).transpose(1, 0, 2)[None] for name in ("q", "k", "v")}
        ref.append(oracle.fwd_recurrent(seq["q"], seq["k"], seq["v"], lam64))   # [1, H, n + steps, d]
    for s in range(steps):
        at = torch.tensor([int(cu_ext[b]) + n + s for b, n in enumerate(lengths)])
        q1, k1, v1 = (t[name][at].contiguous().to(DEV) for name in ("q", "k", "v"))   # [sequences, H, d]
        o1 = binding.la2_decode_step(q1, k1, v1, lam, kv)
        torch.cuda.synchronize()
        want = np.stack([ref[b][0, :, n + s] for b, n in enumerate(lengths)])
        assert_close("decode step %d after the packed prefill" % s, o1, want, dtype)


def test_two_packed_calls_equal_one():
    """Every sequence fed in two pieces (the second call starts from the first call's states) against the oracle's
    direct form of the whole sequences; gradients flow back through the hand-over states."""
    H, d, dtype = 2, 128, torch.bfloat16
    first, second = [40, 100, 0, 64], [33, 29, 50, 0]
    whole = [a + b for a, b in zip(first, second)]
    t, cu_w = packed_inputs(whole, H, d, dtype, seed=960, lam=[0.85, 0.98])
    pick = lambda part: torch.from_numpy(np.concatenate(
        [np.arange(int(cu_w[b]) + (0 if part == 0 else first[b]), int(cu_w[b]) + (first[b] if part == 0 else whole[b]))
         for b in range(len(whole))]).astype(np.int64))
    cu_of = lambda lens: torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).to(DEV)
    lam = t["lam"].to(DEV)
    g = [{name: t[name][pick(part)].contiguous().to(DEV) for name in ("q", "k", "v", "d_o")} for part in (0, 1)]
    cu = [cu_of(first), cu_of(second)]
    o1, s1 = binding.la2_fwd_varlen_state(g[0]["q"], g[0]["k"], g[0]["v"], lam, cu[0], max(first))
    o2, _ = binding.la2_fwd_varlen_state(g[1]["q"], g[1]["k"], g[1]["v"], lam, cu[1], max(second), kv_init=s1,
                                         want_final=False)
    dq2, dk2, dv2, ds1 = binding.la2_bwd_varlen_state(g[1]["q"], g[1]["k"], g[1]["v"], g[1]["d_o"], lam, cu[1], max(second),
                                                      kv_init=s1)
    dq1, dk1, dv1, _ = binding.la2_bwd_varlen_state(g[0]["q"], g[0]["k"], g[0]["v"], g[0]["d_o"], lam, cu[0], max(first),
                                                    d_kv_final=ds1, want_d_kv_init=False)
    torch.cuda.synchronize()
    lam64 = to64(t["lam"])
    off = [np.concatenate([[0], np.cumsum(first)]), np.concatenate([[0], np.cumsum(second)])]
    for b, n in enumerate(whole):
        if n == 0:
            continue
        lo, hi = int(cu_w[b]), int(cu_w[b + 1])
        seq = {name: to64(t[name][lo:hi]).transpose(1, 0, 2)[None] for name in ("q", "k", "v", "d_o")}
        ro = oracle.fwd_direct(seq["q"], seq["k"], seq["v"], lam64)
        rg = oracle.bwd_direct(seq["q"], seq["k"], seq["v"], seq["d_o"], lam64)
        for name, parts, ref in (("o", (o1, o2), ro), ("dq", (dq1, dq2), rg[0]), ("dk", (dk1, dk2), rg[1]),
                                 ("dv", (dv1, dv2), rg[2])):
            got = torch.cat([parts[0][int(off[0][b]):int(off[0][b + 1])], parts[1][int(off[1][b]):int(off[1][b + 1])]])
            assert_close("two calls, seq %d %s" % (b, name), got.permute(1, 0, 2)[None], ref, dtype)


def test_hip_graph_capture_of_the_packed_entry_points():
    """The packed calls in one captured graph, cut into sequence chunks (pair map kernel, pre-pass, state scans,
    accumulating dQ launch, twin launch): replays, with the workspace scribbled over and eager work in between,
    reproduce the eager results bit for bit."""
    binding.la2_set_chunk_tokens(128)
    lengths, H, d, dtype = [300, 0, 77, 512, 33], 2, 128, torch.bfloat16
    t, cu = packed_inputs(lengths, H, d, dtype, seed=970, lam=[0.9, 0.99])
    g = {k: v.to(DEV) for k, v in t.items()}
    cu_g = cu.to(DEV)
    n_max = max(lengths)
    desc = binding._varlen_desc(g["q"], cu_g, n_max)
    import ctypes
    need = int(binding.load().la2_varlen_workspace_bytes(ctypes.byref(desc), g["q"].shape[0], binding.LA2_OP_BWD))
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)

    def buffers():
        like = lambda: torch.empty_like(g["q"])
        return {"o": like(), "kvf": torch.empty_like(g["kv_init"]), "grads": (like(), like(), like()),
                "dkv0": torch.empty_like(g["kv_init"]), "o_plain": like(), "g_plain": (like(), like(), like()),
                "on": like(), "rstd": torch.empty((H, g["q"].shape[0]), device=DEV)}

    def run(out):
        binding.la2_fwd_varlen_state(g["q"], g["k"], g["v"], g["lam"], cu_g, n_max, kv_init=g["kv_init"], out=out["o"],
                                     kv_final=out["kvf"], workspace=ws)
        binding.la2_bwd_varlen_state(g["q"], g["k"], g["v"], g["d_o"], g["lam"], cu_g, n_max, kv_init=g["kv_init"],
                                     d_kv_final=g["d_kv_final"], out=out["grads"], d_kv_init=out["dkv0"], workspace=ws)
        binding.la2_fwd_varlen(g["q"], g["k"], g["v"], g["lam"], cu_g, n_max, out=out["o_plain"], workspace=ws)
        binding.la2_bwd_varlen(g["q"], g["k"], g["v"], g["d_o"], g["lam"], cu_g, n_max, out=out["g_plain"], workspace=ws)
        binding.la2_fwd_varlen_norm(g["q"], g["k"], g["v"], g["lam"], cu_g, n_max, 1e-5, out=out["on"], rstd=out["rstd"],
                                    workspace=ws)

    def flat(out):
        return [out["o"], out["kvf"], *out["grads"], out["dkv0"], out["o_plain"], *out["g_plain"], out["on"]]

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
    rows = slice(int(cu[0]), int(cu[-1]))
    for replay in range(3):
        for x in flat(captured):
            x.fill_(float("nan"))
        ws.random_(0, 255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (got, ref) in enumerate(zip(flat(captured), flat(eager))):
            assert torch.equal(got[rows] if got.shape == g["q"].shape else got, ref[rows] if ref.shape == g["q"].shape else ref), (replay, i)
        scratch = buffers()            # eager work between the replays
        run(scratch)
        torch.cuda.synchronize()


def test_padded_rows_and_head_major_storage():
    """Packed tensors need not be dense: rows padded to d + 8 elements, and heads stored outermost ([H, total, d]
    viewed as [total, H, d]); states stay dense."""
    lengths, H, d, dtype = [75, 0, 200, 33], 3, 128, torch.bfloat16
    t, cu = packed_inputs(lengths, H, d, dtype, seed=980, lam=[0.9, 0.95, 0.99])
    cu_g = cu.to(DEV)
    total = int(sum(lengths))

    def padded(x):
        store = torch.zeros((total, H, d + 8), dtype=x.dtype, device=DEV)
        store[..., :d] = x.to(DEV)
        return store[..., :d]

    def head_major(x):
        return x.permute(1, 0, 2).contiguous().to(DEV).permute(1, 0, 2)

    dense = {k: v.to(DEV) for k, v in t.items()}
    ref_o, ref_kvf = binding.la2_fwd_varlen_state(dense["q"], dense["k"], dense["v"], dense["lam"], cu_g, max(lengths),
                                                  kv_init=dense["kv_init"])
    ref_g = binding.la2_bwd_varlen_state(dense["q"], dense["k"], dense["v"], dense["d_o"], dense["lam"], cu_g, max(lengths),
                                         kv_init=dense["kv_init"], d_kv_final=dense["d_kv_final"])
    for place in (padded, head_major):
        g = {name: place(t[name]) for name in ("q", "k", "v", "d_o")}
        assert not g["q"].is_contiguous()
        o, kvf = binding.la2_fwd_varlen_state(g["q"], g["k"], g["v"], dense["lam"], cu_g, max(lengths),
                                              kv_init=dense["kv_init"])
        got = binding.la2_bwd_varlen_state(g["q"], g["k"], g["v"], g["d_o"], dense["lam"], cu_g, max(lengths),
                                           kv_init=dense["kv_init"], d_kv_final=dense["d_kv_final"])
        torch.cuda.synchronize()
        assert o.stride() == g["q"].stride()
        assert torch.equal(o, ref_o) and torch.equal(kvf, ref_kvf), place.__name__
        for a, b in zip(got, ref_g):
            assert torch.equal(a, b), place.__name__
