"""GPU parity of the head dimensions 96 and 256 against the fp64 oracle: forward, backward, sequence chunks,
state hand-over at ragged ends, packed sequences, decode; 16-bit data through the block kernel of these head
dimensions, fp32 through the token recurrence."""
import numpy as np
import pytest
import torch

import oracle
from paper_2401_04658_amd import binding, workloads
from parity import assert_close, to64

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
DIMS = (96, 256)
LENGTHS = (1, 31, 32, 33, 100, 517)


@pytest.fixture(autouse=True)
def _defaults():
    binding.la2_set_chunk_tokens(0)
    binding.la2_set_scan_variant(0)
    yield
    binding.la2_set_chunk_tokens(0)
    binding.la2_set_scan_variant(0)


def inputs(b, H, n, d, dtype, seed, lam=None):
    t = workloads.Workload("wide", b, H, n, d, dtype, seed=seed, backward=True).tensors()
    if lam is not None:
        t["lam"] = torch.as_tensor(lam, dtype=torch.float32).reshape(-1).expand(H).contiguous()
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed + 1)
    t["kv_init"] = torch.randn((b, H, d, d), generator=gen, dtype=torch.float32) * 0.3
    t["d_kv_final"] = torch.randn((b, H, d, d), generator=gen, dtype=torch.float32) * 0.3
    return t, {k: v.to(DEV) for k, v in t.items()}


def check_plain(t, g, dtype, tag):
    o = binding.la2_fwd(g["q"], g["k"], g["v"], g["lam"])
    grads = binding.la2_bwd(g["q"], g["k"], g["v"], g["d_o"], g["lam"])
    torch.cuda.synchronize()
    q, k, v, do, lam = (to64(t[x]) for x in ("q", "k", "v", "d_o", "lam"))
    assert_close(tag + " o", o, oracle.fwd_direct(q, k, v, lam), dtype)
    for name, got, ref in zip(("dq", "dk", "dv"), grads, oracle.bwd_direct(q, k, v, do, lam)):
        assert_close(tag + " " + name, got, ref, dtype)


def check_state(t, g, dtype, tag, final=True):
    o, kvf = binding.la2_fwd_state(g["q"], g["k"], g["v"], g["lam"], kv_init=g["kv_init"], want_final=final)
    dq, dk, dv, dkv0 = binding.la2_bwd_state(g["q"], g["k"], g["v"], g["d_o"], g["lam"], kv_init=g["kv_init"],
                                             d_kv_final=g["d_kv_final"] if final else None)
    torch.cuda.synchronize()
    q, k, v, do, lam = (to64(t[x]) for x in ("q", "k", "v", "d_o", "lam"))
    init64 = to64(t["kv_init"])
    ro, rkvf = oracle.fwd_recurrent(q, k, v, lam, kv_init=init64, return_state=True)
    refs = oracle.bwd_recurrent_state(q, k, v, do, lam, kv_init=init64,
                                      d_kv_final=to64(t["d_kv_final"]) if final else None)
    assert_close(tag + " o", o, ro, dtype)
    if final:
        assert_close(tag + " kv_final", kvf, rkvf, dtype)
    for name, got, ref in zip(("dq", "dk", "dv", "d_kv_init"), (dq, dk, dv, dkv0), refs):
        assert_close(tag + " " + name, got, ref, dtype)


@pytest.mark.parametrize("n", LENGTHS)
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("d", DIMS)
def test_fwd_bwd(d, dtype, n):
    t, g = inputs(2, 3, n, d, dtype, seed=1000 + d + n, lam=[0.5, 0.93, 1.0])
    check_plain(t, g, dtype, "d%d %s n%d" % (d, dtype, n))


@pytest.mark.parametrize("d", DIMS)
def test_decay_schedule_and_small_decay(d):
    t, g = inputs(1, 4, 200, d, torch.bfloat16, seed=1100 + d)            # the benchmark's per-head schedule
    check_plain(t, g, torch.bfloat16, "d%d schedule" % d)
    t, g = inputs(1, 2, 77, d, torch.bfloat16, seed=1101 + d, lam=[1e-3, 0.05])   # every weight stays finite
    check_plain(t, g, torch.bfloat16, "d%d small decay" % d)
    check_state(t, g, torch.bfloat16, "d%d small decay, states" % d)


@pytest.mark.parametrize("chunk", [64, 192])
@pytest.mark.parametrize("n", [700, 1024, 129])
@pytest.mark.parametrize("d", DIMS)
def test_sequence_chunks(d, n, chunk):
    binding.la2_set_chunk_tokens(chunk)
    t, g = inputs(1, 2, n, d, torch.bfloat16, seed=1200 + d + n + chunk, lam=[0.8, 0.99])
    check_plain(t, g, torch.bfloat16, "d%d n%d chunk %d" % (d, n, chunk))
    check_state(t, g, torch.bfloat16, "d%d n%d chunk %d, states" % (d, n, chunk))


@pytest.mark.parametrize("d", DIMS)
def test_automatic_chunking_of_a_long_sequence(d):
    """Few chains, a long sequence: the planner cuts it into chunks on its own."""
    n = 8192 if d == 96 else 4096
    t, g = inputs(1, 2, n, d, torch.bfloat16, seed=1250 + d, lam=[0.9, 0.999])
    assert binding.la2_workspace_bytes(g["q"], 0) > 0
    o = binding.la2_fwd(g["q"], g["k"], g["v"], g["lam"])
    grads = binding.la2_bwd(g["q"], g["k"], g["v"], g["d_o"], g["lam"])
    torch.cuda.synchronize()
    q, k, v, do, lam = (to64(t[x]) for x in ("q", "k", "v", "d_o", "lam"))
    assert_close("d%d long o" % d, o, oracle.fwd_recurrent(q, k, v, lam), torch.bfloat16)
    for name, got, ref in zip(("dq", "dk", "dv"), grads, oracle.bwd_recurrent(q, k, v, do, lam)):
        assert_close("d%d long %s" % (d, name), got, ref, torch.bfloat16)


@pytest.mark.parametrize("final", [True, False])
@pytest.mark.parametrize("n", [1, 31, 32, 45, 64, 100, 300])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("d", DIMS)
def test_state_handover(d, dtype, n, final):
    t, g = inputs(2, 2, n, d, dtype, seed=1300 + d + n, lam=[0.7, 0.98])
    check_state(t, g, dtype, "d%d %s n%d final %s" % (d, dtype, n, final), final)


@pytest.mark.parametrize("d", DIMS)
def test_segments_compose(d):
    """Two segments with the state handed over reproduce the whole sequence (ragged cut)."""
    t, g = inputs(1, 2, 150, d, torch.bfloat16, seed=1400 + d, lam=[0.9, 0.97])
    cut = 77
    o1, s1 = binding.la2_fwd_state(g["q"][:, :, :cut].contiguous(), g["k"][:, :, :cut].contiguous(),
                                   g["v"][:, :, :cut].contiguous(), g["lam"])
    o2, s2 = binding.la2_fwd_state(g["q"][:, :, cut:].contiguous(), g["k"][:, :, cut:].contiguous(),
                                   g["v"][:, :, cut:].contiguous(), g["lam"], kv_init=s1)
    torch.cuda.synchronize()
    q, k, v, lam = (to64(t[x]) for x in ("q", "k", "v", "lam"))
    ro, rs = oracle.fwd_recurrent(q, k, v, lam, return_state=True)
    assert_close("segments o", torch.cat([o1, o2], dim=2), ro, torch.bfloat16)
    assert_close("segments state", s2, rs, torch.bfloat16)


@pytest.mark.parametrize("d", DIMS)
def test_strided_layout(d):
    """[b, n, H, d] storage viewed as [b, H, n, d]."""
    t, g = inputs(2, 3, 90, d, torch.bfloat16, seed=1500 + d)
    for name in ("q", "k", "v", "d_o"):
        g[name] = t[name].permute(0, 2, 1, 3).contiguous().to(DEV).permute(0, 2, 1, 3)
    check_plain(t, g, torch.bfloat16, "d%d bnhd" % d)


@pytest.mark.parametrize("d", DIMS)
def test_fp32_runs_the_token_recurrence(d):
    t, g = inputs(1, 2, 70, d, torch.float32, seed=1600 + d, lam=[0.6, 0.99])
    assert binding.la2_workspace_bytes(g["q"], 1) == 0
    check_plain(t, g, torch.float32, "d%d fp32" % d)
    check_state(t, g, torch.float32, "d%d fp32 states" % d)
    check_state(t, g, torch.float32, "d%d fp32 states, no final" % d, final=False)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("d", DIMS)
def test_packed_sequences(d, dtype):
    lengths = [70, 0, 1, 31, 32, 100, 260, 3]
    H = 2
    total = sum(lengths)
    wl = workloads.Workload("packed", 1, H, total, d, dtype, seed=1700 + d, backward=True).tensors()
    pk = {name: wl[name][0].permute(1, 0, 2).contiguous() for name in ("q", "k", "v", "d_o")}
    g = {name: x.to(DEV) for name, x in pk.items()}
    lam = torch.tensor([0.8, 0.99])
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lengths)]), dtype=torch.int32, device=DEV)
    for chunk in (0, 64):
        binding.la2_set_chunk_tokens(chunk)
        o = binding.la2_fwd_varlen(g["q"], g["k"], g["v"], lam.to(DEV), cu, max(lengths))
        grads = binding.la2_bwd_varlen(g["q"], g["k"], g["v"], g["d_o"], lam.to(DEV), cu, max(lengths))
        torch.cuda.synchronize()
        lo = 0
        for m in lengths:
            if m:
                sq = {name: to64(pk[name][lo:lo + m]).transpose(1, 0, 2)[None] for name in pk}
                tag = "d%d %s packed chunk %d seq at %d (n %d)" % (d, dtype, chunk, lo, m)
                assert_close(tag + " o", o[lo:lo + m].permute(1, 0, 2)[None],
                             oracle.fwd_direct(sq["q"], sq["k"], sq["v"], to64(lam)), dtype)
                for name, got, ref in zip(("dq", "dk", "dv"), grads,
                                          oracle.bwd_direct(sq["q"], sq["k"], sq["v"], sq["d_o"], to64(lam))):
                    assert_close(tag + " " + name, got[lo:lo + m].permute(1, 0, 2)[None], ref, dtype)
            lo += m


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16, torch.float32])
@pytest.mark.parametrize("d", DIMS)
def test_decode_steps_follow_the_forward_pass(d, dtype):
    b, H, n = 2, 3, 9
    t, g = inputs(b, H, n, d, dtype, seed=1800 + d, lam=[0.5, 0.9, 1.0])
    state = g["kv_init"].clone()
    outs = []
    for i in range(n):
        outs.append(binding.la2_decode_step(g["q"][:, :, i].contiguous(), g["k"][:, :, i].contiguous(),
                                            g["v"][:, :, i].contiguous(), g["lam"], state))
    torch.cuda.synchronize()
    q, k, v, lam = (to64(t[x]) for x in ("q", "k", "v", "lam"))
    ro, rs = oracle.fwd_recurrent(q, k, v, lam, kv_init=to64(t["kv_init"]), return_state=True)
    assert_close("d%d %s decode o" % (d, dtype), torch.stack(outs, dim=2), ro, dtype)
    assert_close("d%d %s decode state" % (d, dtype), state, rs, dtype)


@pytest.mark.parametrize("T", [1, 2, 7, 32, 33, 100])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("d", DIMS)
def test_decode_multi(d, dtype, T):
    t, g = inputs(2, 2, T, d, dtype, seed=1900 + d + T, lam=[0.6, 0.97])
    state = g["kv_init"].clone()
    o = binding.la2_decode_multi(g["q"], g["k"], g["v"], g["lam"], state)
    torch.cuda.synchronize()
    q, k, v, lam = (to64(t[x]) for x in ("q", "k", "v", "lam"))
    ro, rs = oracle.fwd_recurrent(q, k, v, lam, kv_init=to64(t["kv_init"]), return_state=True)
    assert_close("d%d %s decode_multi T%d o" % (d, dtype, T), o, ro, dtype)
    assert_close("d%d %s decode_multi T%d state" % (d, dtype, T), state, rs, dtype)


@pytest.mark.parametrize("n", [1, 33, 100, 517])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16, torch.float32])
@pytest.mark.parametrize("d", DIMS)
def test_normalised_operator(d, dtype, n):
    eps = 1e-3
    t, g = inputs(2, 2, n, d, dtype, seed=2000 + d + n, lam=[0.7, 0.98])
    for chunk in (0, 64):
        binding.la2_set_chunk_tokens(chunk)
        o, rstd = binding.la2_fwd_norm(g["q"], g["k"], g["v"], g["lam"], eps)
        grads = binding.la2_bwd_norm(g["q"], g["k"], g["v"], o, rstd, g["d_o"], g["lam"])
        torch.cuda.synchronize()
        q, k, v, do, lam = (to64(t[x]) for x in ("q", "k", "v", "d_o", "lam"))
        ref_o, ref_r = oracle.fwd_norm(q, k, v, lam, eps)
        tag = "d%d %s n%d chunk %d norm" % (d, dtype, n, chunk)
        assert_close(tag + " o", o, ref_o, dtype)
        assert_close(tag + " rstd", rstd, ref_r, dtype)
        if n > 1:   # a single position leaves dq, dk as pure cancellation
            for name, got, ref in zip(("dq", "dk", "dv"), grads, oracle.bwd_norm(q, k, v, do, lam, eps)):
                assert_close(tag + " " + name, got, ref, dtype)


def test_no_left_product_comparison_at_these_head_dimensions():
    t, g = inputs(1, 1, 40, 96, torch.bfloat16, seed=1)
    with pytest.raises(binding.LA2Error):
        binding.la2_left_product_fwd(g["q"], g["k"], g["v"], g["lam"])


@pytest.mark.parametrize("n", [700, 1024])
@pytest.mark.parametrize("d", DIMS)
def test_backward_reuses_the_forward_chunk_states(d, n):
    """la2_bwd_saved: the dQ scan starts from the chunk states the forward pass left in its workspace."""
    binding.la2_set_chunk_tokens(128)
    t, g = inputs(1, 2, n, d, torch.bfloat16, seed=2100 + d + n, lam=[0.85, 0.995])
    need = binding.la2_workspace_bytes(g["q"], binding.LA2_OP_BWD_STATE)
    assert need > 0
    ws_f = torch.empty(need, dtype=torch.uint8, device=DEV)
    ws_b = torch.empty(need, dtype=torch.uint8, device=DEV)
    for use_init in (False, True):
        kv_init = g["kv_init"] if use_init else None
        binding.la2_fwd_state(g["q"], g["k"], g["v"], g["lam"], kv_init=kv_init, want_final=False, workspace=ws_f)
        got = binding.la2_bwd_state(g["q"], g["k"], g["v"], g["d_o"], g["lam"], kv_init=kv_init,
                                    workspace=ws_b, fwd_workspace=ws_f)
        torch.cuda.synchronize()
        q, k, v, do, lam = (to64(t[x]) for x in ("q", "k", "v", "d_o", "lam"))
        refs = oracle.bwd_recurrent_state(q, k, v, do, lam, kv_init=to64(t["kv_init"]) if use_init else None)
        for name, x, ref in zip(("dq", "dk", "dv", "d_kv_init"), got, refs):
            assert_close("saved states d%d n%d init=%s %s" % (d, n, use_init, name), x, ref, torch.bfloat16)


@pytest.mark.parametrize("d", DIMS)
def test_hip_graph_capture_and_replay(d):
    """A sequence-chunked forward and backward (pre-pass, state scan, scans, dual reverse launch), the normalised
    operator and a packed batch at these head dimensions in one captured graph; every replay reproduces the
    eager results bit for bit."""
    binding.la2_set_chunk_tokens(128)
    b, H, n = 1, 2, 600
    t, g = inputs(b, H, n, d, torch.bfloat16, seed=2200 + d, lam=[0.9, 0.99])
    ws = torch.empty(max(256, binding.la2_workspace_bytes(g["q"], 1)), dtype=torch.uint8, device=DEV)
    lengths = [100, 0, 333, 167]
    pk = {name: g[name][0].permute(1, 0, 2).contiguous() for name in ("q", "k", "v", "d_o")}   # [n, H, d]
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lengths)]), dtype=torch.int32, device=DEV)
    ws_p = torch.empty(16 << 20, dtype=torch.uint8, device=DEV)

    def run(out):
        binding.la2_fwd(g["q"], g["k"], g["v"], g["lam"], out=out["o"], workspace=ws)
        binding.la2_bwd(g["q"], g["k"], g["v"], g["d_o"], g["lam"], out=out["grads"], workspace=ws)
        binding.la2_fwd_norm(g["q"], g["k"], g["v"], g["lam"], 1e-5, out=out["on"], rstd=out["rstd"], workspace=ws)
        binding.la2_bwd_norm(g["q"], g["k"], g["v"], out["on"], out["rstd"], g["d_o"], g["lam"], out=out["gn"],
                             d_u=out["du"], workspace=ws)
        binding.la2_fwd_varlen(pk["q"], pk["k"], pk["v"], g["lam"], cu, max(lengths), out=out["op"], workspace=ws_p)
        binding.la2_bwd_varlen(pk["q"], pk["k"], pk["v"], pk["d_o"], g["lam"], cu, max(lengths), out=out["gp"],
                               workspace=ws_p)

    def buffers():
        like, likep = (lambda: torch.empty_like(g["q"])), (lambda: torch.empty_like(pk["q"]))
        return {"o": like(), "grads": (like(), like(), like()), "on": like(), "rstd": torch.empty((b, H, n), device=DEV),
                "gn": (like(), like(), like()), "du": like(), "op": likep(), "gp": (likep(), likep(), likep())}

    def flat(out):
        return [out["o"], *out["grads"], out["on"], out["rstd"], *out["gn"], out["du"], out["op"], *out["gp"]]

    assert binding.la2_workspace_bytes(g["q"], 0) > 0
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
        ws_p.random_(0, 255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (got, ref) in enumerate(zip(flat(captured), flat(eager))):
            assert torch.equal(got, ref), (replay, i)
        run(buffers())                 # eager work between the replays
        torch.cuda.synchronize()
