"""Full-size parity of the benchmark configurations, every chain: la2_fwd / la2_bwd on the four points of the
sequence-length sweep and on the 3B-like layer against the fp64 token recurrence (Sec. 3.2.1 recursive form, Sec.
3.2.2 reverse recursion), element by element over the whole tensors, head by head (each head has its own decay,
hence its own output scale); rows around every planned chunk boundary against the O(n^2) definition as well; the
decode configuration for all its steps on several batch rows.  Launch configurations are the ones bench.py times
(automatic chunk plan, caller's workspace)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2401_04658_amd import binding, workloads
from parity import TOL, assert_close, max_rel, to64

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def boundary_rows(n, nchunks, chunk_tokens):
    rows = {0, 1, n - 2, n - 1}
    for c in range(1, nchunks):
        for off in (-2, -1, 0, 1):
            rows.add(c * chunk_tokens + off)
    return np.array(sorted(r for r in rows if 0 <= r < n), dtype=np.int64)


def check_every_chain(wl):
    t = wl.tensors()
    g = {k: v.to(DEV) for k, v in t.items()}
    nchunks, chunk_tokens = binding.la2_chunk_plan(g["q"])
    print(wl.name, "chunks", nchunks, "x", chunk_tokens, flush=True)
    need = max(binding.la2_workspace_bytes(g["q"], binding.LA2_OP_FWD), binding.la2_workspace_bytes(g["q"], binding.LA2_OP_BWD))
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=DEV)
    o = binding.la2_fwd(g["q"], g["k"], g["v"], g["lam"], workspace=ws)
    dq, dk, dv = binding.la2_bwd(g["q"], g["k"], g["v"], g["d_o"], g["lam"], workspace=ws)
    # the training-step path as well: the backward pass from the forward call's chunk states
    ws_b = torch.empty_like(ws)
    binding.la2_fwd(g["q"], g["k"], g["v"], g["lam"], workspace=ws)
    sq, sk, sv, _ = binding.la2_bwd_state(g["q"], g["k"], g["v"], g["d_o"], g["lam"], want_d_kv_init=False,
                                          workspace=ws_b, fwd_workspace=ws)
    torch.cuda.synchronize()
    got = {"o": o.cpu(), "dq": dq.cpu(), "dk": dk.cpu(), "dv": dv.cpu(), "dq saved": sq.cpu(), "dk saved": sk.cpu(),
           "dv saved": sv.cpu()}
    del g, o, dq, dk, dv, sq, sk, sv, ws, ws_b
    torch.cuda.empty_cache()
    q, k, v, do, lam = (to64(t[x]) for x in ("q", "k", "v", "d_o", "lam"))
    ref = {"o": oracle.fwd_recurrent(q, k, v, lam)}
    print(wl.name, "oracle forward done", flush=True)
    ref["dq"], ref["dk"], ref["dv"] = oracle.bwd_recurrent(q, k, v, do, lam)
    print(wl.name, "oracle backward done", flush=True)
    for name, x in got.items():
        r = ref[name.split()[0]]
        for h in range(wl.heads):
            assert_close("%s %s head %d" % (wl.name, name, h), x[:, h], r[:, h], wl.dtype)
    # rows around every chunk boundary, three chains, against the O(n^2) definition
    rows = boundary_rows(wl.seqlen, nchunks, chunk_tokens)
    for b, h in ((0, 0), (wl.batch - 1, wl.heads // 2), (wl.batch // 2, wl.heads - 1)):
        lam_h = float(lam[h])
        ro = oracle.fwd_rows(q[b, h], k[b, h], v[b, h], lam_h, rows)
        rq, rk, rv = oracle.bwd_rows(q[b, h], k[b, h], v[b, h], do[b, h], lam_h, rows)
        for name, r in (("o", ro), ("dq", rq), ("dk", rk), ("dv", rv)):
            x = to64(got[name][b, h])[rows]
            err = float(np.max(np.abs(x - r))) / float(np.max(np.abs(ref[name][b, h])))
            assert err <= TOL[wl.dtype], "%s %s boundary rows (b%d h%d): %.3e" % (wl.name, name, b, h, err)


@pytest.mark.parametrize("idx", range(4))
def test_config3_every_chain(idx):
    check_every_chain(workloads.CONFIG3[idx])


def test_config4_every_chain():
    check_every_chain(workloads.CONFIG4)


def test_config2_every_chain():
    check_every_chain(workloads.CONFIG2)


def test_config5_decode_1024_steps_eight_batch_rows():
    wl = workloads.CONFIG5
    batch = 8
    gen = wl.generator()
    state0 = wl.initial_state(gen)[:batch].contiguous()
    lam = wl.decay()
    kv_gpu, kv_ref = state0.to(DEV), state0.double().numpy().copy()
    lam_gpu, lam64 = lam.to(DEV), lam.double().numpy()
    for step in range(wl.steps):
        q, k, v = (x[:batch].contiguous() for x in wl.token(gen))
        o = binding.la2_decode_step(q.to(DEV), k.to(DEV), v.to(DEV), lam_gpu, kv_gpu)
        r = oracle.decode_step(to64(q), to64(k), to64(v), lam64, kv_ref)
        if step % 16 == 0 or step == wl.steps - 1:
            m = max_rel(to64(o), r)
            assert m <= TOL[torch.bfloat16], "decode o at step %d: %.3e" % (step, m)
    torch.cuda.synchronize()
    for b in range(batch):
        m = max_rel(to64(kv_gpu[b]), kv_ref[b])
        assert m <= 1e-5, "decode state of batch row %d after %d steps: %.3e" % (b, wl.steps, m)
