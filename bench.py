#!/usr/bin/env python3
"""Benchmark of the Lightning Attention-2 hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One "step" is a forward + backward pass (la2_fwd + la2_bwd) at each of the four points of the
sequence-length sweep -- (batch, n) = (64,1K), (16,4K), (4,16K), (1,64K), H=16, d=128, bf16, i.e.
4 x 65,536 tokens -- on seeded synthetic tensors that are resident in HBM before the timed region.
Prints ONE JSON line: whole-step tokens/s, the per-point table (tokens/s, TFLOP/s, fraction of the
bf16 MFMA peak, flatness), the other configurations (400M-like layer, 3B-like layer, decode), the
roofline of the dominant kernel measured live with events on the launch stream (and beside it a kernel that
only streams the same bytes in the same read : write mix, bench_probe.stream_probe: the rate the memory system gives
any kernel with that traffic), and the fp64 CPU oracle timed on a bounded sample as a baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
# rocprofv3 --pmc measurement of the dominant kernel's HBM traffic per launch: the committed summary carries a
# line "traffic_bytes_per_launch: N" (FETCH_SIZE and WRITE_SIZE, each scaled by the plain-copy reference)
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "la2_fwd_bwd_b16_n4096_h16_d128_kernel_trace_traffic_and_counters.txt")


def measured_traffic_bytes():
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary, or None."""
    try:
        for line in open(TRAFFIC_PROFILE):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(line.split(":")[1].split()[0])
    except OSError:
        pass
    return None


def mfma_peak_tflops(time_ms, bench_probe, dev):
    """What a register-only loop of v_mfma_f32_32x32x16_bf16 reaches on this machine right now (1024 workgroups
    x 4 waves; the clock under load is below the 2.4 GHz behind the data sheet's 2.5 PFLOP/s)."""
    import torch
    sink = torch.zeros(16, dtype=torch.float32, device=dev)
    flops = [0]

    def run():
        flops[0] = bench_probe.mfma_peak(1024, 2000, sink)
    ms = time_ms(run, 20, warm=5)
    return flops[0] / (ms * 1e-3) / 1e12


def flops_per_token_head(B, d, what):
    """FLOPs of Algorithms 1 / 2 per token per head (full B x B tiles counted, as the algorithms do)."""
    fwd = 4 * B * d + 4 * d * d
    bwd = 12 * B * d + 10 * d * d
    return {"fwd": fwd, "bwd": bwd, "fwd+bwd": fwd + bwd}[what]


def stream_reference(g, time_ms, bench_probe, iters):
    """A kernel that only streams (no arithmetic, no LDS, no dependences), timed on the buffers and byte counts
    of the scan launches: 3 tensors in, 1 out (forward scan, dQ scan) and 4 in, 2 out (the twin dK / dV scan);
    the better of the two store policies each.  What the memory system gives such a kernel is the bound the scan
    kernels can reach; the 8 TB/s of the roofline entry is the pin bandwidth."""
    import torch
    unit = g["q"].numel() * g["q"].element_size()
    src = torch.zeros(4 * unit, dtype=torch.uint8, device=g["q"].device)
    dst = torch.empty(2 * unit, dtype=torch.uint8, device=g["q"].device)
    out = {}
    for name, r, w in (("reads3_writes1", 3, 1), ("reads4_writes2", 4, 2), ("reads3", 3, 0)):
        best = min(time_ms(lambda: bench_probe.stream_probe(r, w, src, dst, unit, nt_stores=nts), iters, warm=20)
                   for nts in ((False, True) if w else (False,)))
        out[name] = {"launch_ms": round(best, 4), "GBs": round((r + w) * unit / (best * 1e-3) / 1e9, 1)}
    return out


def dominant_kernel_roofline(wl, g, fwd, time_ms, binding, iters):
    """The forward scan at (batch 16, n 4K): la2_fwd is exactly one launch of the scan kernel there."""
    assert binding.la2_workspace_bytes(g["q"]) == 0, "expected the un-chunked single-launch case"
    k_ms = time_ms(lambda: fwd(g), iters)
    th, d, B = wl.token_heads, wl.head_dim, g["B"]
    bytes_alg = 8 * d * th            # read Q, K, V and write O once, bf16
    flops_alg = flops_per_token_head(B, d, "fwd") * th
    return {
        "kernel": "scan_bf16_half_kernel<fwd, plain, 3 buffers> (la2_fwd, %s)" % wl.name,
        "bound": "hbm",
        "achieved": round(bytes_alg / (k_ms * 1e-3) / 1e9, 1),
        "peak": PEAK_HBM_GBS,
        "unit": "GB/s",
        "frac": round(bytes_alg / (k_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
        # HBM bytes per launch measured with rocprofv3 FETCH_SIZE / WRITE_SIZE, each scaled by the factor the
        # same counter shows for a plain copy of known size (2.00 and 1.00): read from
        # profiles/la2_fwd_bwd_b16_n4096_h16_d128_kernel_trace_traffic_and_counters.txt
        "traffic": measured_traffic_bytes(),
        "algorithmic_bytes": bytes_alg,
        "launch_ms": round(k_ms, 4),
        "mfma_tflops": round(flops_alg / (k_ms * 1e-3) / 1e12, 2),
        "mfma_frac_of_bf16_peak": round(flops_alg / (k_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "arith_intensity_flop_per_byte": round(flops_alg / bytes_alg, 1),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--roofline-only", action="store_true",
                    help="run only the dominant kernel's loop (for rocprofv3 counter passes); prints its roofline JSON")
    ap.add_argument("--roofline-op", choices=("fwd", "bwd"), default="fwd",
                    help="with --roofline-only: loop la2_fwd (one launch of the forward scan kernel) or la2_bwd "
                         "(the dQ forward scan and the twin dK/dV reverse scan) at (batch 16, n 4096)")
    ap.add_argument("--profile", metavar="OP:WORKLOAD",
                    help="for rocprofv3 passes: after the plain-copy reference and a warm-up, loop one operation on one "
                         "workload and print its time.  OP: fwd, bwd, bwd_saved (backward from the forward's chunk "
                         "states), fwd_norm, bwd_norm, decode, decode8 (8 tokens per launch).  WORKLOAD: c3_0 .. c3_3 "
                         "(the sweep points), c2, c4, w256, w96 (head_dim 256 / 96 at batch 64, n 1024), b20 (batch 20, n 4096: 320 "
                         "chains, run as two calls); decode ops take c5")
    ap.add_argument("--profile-chunk-tokens", type=int, default=0,
                    help="with --profile: the caller's chunk size (la2_set_chunk_tokens); the sequence length gives one "
                         "call with one chunk")
    ap.add_argument("--profile-iters", type=int, default=400)
    ap.add_argument("--profile-settle-ms", type=float, default=80.0,
                    help="with --profile: call the operation for this long before the timed loop (0 for counter passes, "
                         "whose values do not depend on the clocks); a kernel-trace summary then takes each kernel's "
                         "steady-state duration from the last third of its dispatches")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (one MI355X); --gpus %d is not supported. "
              "Run with --gpus 1." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2401_04658_amd as la2
    from paper_2401_04658_amd import bench_probe, binding, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    la2.load()   # raises if the HIP library has not been built: there is no fallback path
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    def stage(wl):
        t = wl.tensors()
        g = {k: v.to(dev) for k, v in t.items()}
        g["o"] = torch.empty_like(g["q"])
        g["grads"] = tuple(torch.empty_like(g["q"]) for _ in range(3))
        need = max(binding.la2_workspace_bytes(g["q"], binding.LA2_OP_FWD),
                   binding.la2_workspace_bytes(g["q"], binding.LA2_OP_BWD))
        g["ws"] = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
        g["B"] = binding.la2_block_size(g["q"])
        return g

    def fwd(g):
        binding.la2_fwd(g["q"], g["k"], g["v"], g["lam"], out=g["o"], workspace=g["ws"])

    def bwd(g):
        binding.la2_bwd(g["q"], g["k"], g["v"], g["d_o"], g["lam"], out=g["grads"], workspace=g["ws"])

    def time_ms(fn, iters, warm=2, settle_ms=0.0):
        """Average ms per call, HIP events on the stream the kernels are launched on.  settle_ms: keep calling for
        that long first, untimed.  After an idle spell (the host staging the next tensors) the device needs about
        40 ms of continuous work to reach its steady clocks: launches of 0.183 ms in the steady state take
        0.23-0.29 ms in the first 10 ms and 0.19 ms after 30 ms (measured with windows of 50 launches)."""
        if settle_ms > 0:
            t_end = time.perf_counter() + settle_ms * 1e-3
            while time.perf_counter() < t_end:
                for _ in range(20):
                    fn()
                torch.cuda.synchronize()
        for _ in range(warm):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    def copy_reference():
        # a plain copy of known size first: the reference that scales the FETCH_SIZE / WRITE_SIZE counters
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    if args.profile:
        op, _, wname = args.profile.partition(":")
        copy_reference()
        iters = args.profile_iters
        if op in ("decode", "decode8"):
            dw = workloads.CONFIG5
            gen = dw.generator()
            kv = dw.initial_state(gen).to(dev)
            lam5 = dw.decay().to(dev)
            toks = [tuple(x.to(dev) for x in dw.token(gen)) for _ in range(8)]
            if op == "decode":
                o5 = torch.empty_like(toks[0][0])
                ms = time_ms(lambda: binding.la2_decode_step(*toks[0], lam5, kv, out=o5), iters, warm=20,
                             settle_ms=args.profile_settle_ms)
            else:
                qm, km, vm = (torch.stack([toks[i][j] for i in range(8)], 2).contiguous() for j in range(3))
                om = torch.empty_like(qm)
                ms = time_ms(lambda: binding.la2_decode_multi(qm, km, vm, lam5, kv, out=om), iters, warm=20,
                             settle_ms=args.profile_settle_ms)
            print(json.dumps({"op": op, "workload": dw.name, "ms": round(ms, 5), "timed_calls": iters}))
            return
        table = {"c3_%d" % i: w_ for i, w_ in enumerate(workloads.CONFIG3)}
        table.update({"c2": workloads.CONFIG2, "c4": workloads.CONFIG4})
        # the other head dimensions, as in other_head_dims below
        table.update({"w256": workloads.Workload("b64_n1024_h8_d256", 64, 8, 1024, 256, torch.bfloat16, seed=60 + 256),
                      "w96": workloads.Workload("b64_n1024_h16_d96", 64, 16, 1024, 96, torch.bfloat16, seed=60 + 96)})
        table["b20"] = workloads.Workload("b20_n4096_h16_d128", 20, 16, 4096, 128, torch.bfloat16, seed=71)
        wl_p = table[wname]
        g_p = stage(wl_p)
        binding.la2_set_chunk_tokens(args.profile_chunk_tokens)
        settle = args.profile_settle_ms
        if op == "fwd":
            ms = time_ms(lambda: fwd(g_p), iters, settle_ms=settle)
        elif op == "bwd":
            ms = time_ms(lambda: bwd(g_p), iters, settle_ms=settle)
        elif op == "bwd_saved":
            ws_b = torch.empty_like(g_p["ws"])
            fwd(g_p)
            ms = time_ms(lambda: binding.la2_bwd_state(g_p["q"], g_p["k"], g_p["v"], g_p["d_o"], g_p["lam"],
                                                       want_d_kv_init=False, out=g_p["grads"], workspace=ws_b,
                                                       fwd_workspace=g_p["ws"]), iters, settle_ms=settle)
        elif op in ("fwd_norm", "bwd_norm"):
            rstd = torch.empty(g_p["q"].shape[:3], dtype=torch.float32, device=dev)
            d_u = torch.empty_like(g_p["q"])
            f_n = lambda: binding.la2_fwd_norm(g_p["q"], g_p["k"], g_p["v"], g_p["lam"], 1e-6, out=g_p["o"], rstd=rstd,
                                               workspace=g_p["ws"])
            f_n()
            ms = time_ms(f_n if op == "fwd_norm" else
                         (lambda: binding.la2_bwd_norm(g_p["q"], g_p["k"], g_p["v"], g_p["o"], rstd, g_p["d_o"],
                                                       g_p["lam"], out=g_p["grads"], d_u=d_u, workspace=g_p["ws"])), iters,
                         settle_ms=settle)
        else:
            raise SystemExit("bench.py: unknown --profile operation %r" % op)
        print(json.dumps({"op": op, "workload": wl_p.name, "ms": round(ms, 5), "timed_calls": iters,
                          "chunk_plan": binding.la2_chunk_plan(g_p["q"]),
                          "token_heads": wl_p.token_heads, "head_dim": wl_p.head_dim}))
        return

    if args.roofline_only:
        copy_reference()
        wl_r = workloads.CONFIG3[1]
        g_r = stage(wl_r)
        time_ms(lambda: fwd(g_r), 300)      # long warm-up: lets the clocks settle as in the full benchmark
        if args.roofline_op == "bwd":
            b_ms = time_ms(lambda: bwd(g_r), 200)
            bytes_alg = 20 * wl_r.head_dim * wl_r.token_heads   # dQ scan 8d, twin dK/dV scan 12d (bf16)
            print(json.dumps({"op": "la2_bwd (%s)" % wl_r.name, "ms": round(b_ms, 4), "algorithmic_bytes": bytes_alg,
                              "achieved_GBs": round(bytes_alg / (b_ms * 1e-3) / 1e9, 1)}))
            return
        print(json.dumps(dominant_kernel_roofline(wl_r, g_r, fwd, time_ms, binding, 200)))
        return

    sweep = [(wl, stage(wl)) for wl in workloads.CONFIG3]

    def step():
        for _, g in sweep:
            fwd(g)
            bwd(g)

    # ---- roofline of the dominant kernel: the forward scan at (16, 4K), one launch per call.  Measured first,
    # after 300 launches that let the clocks settle; the headline below then starts on a machine in its
    # steady state whatever --warmup says.
    wl_r, g_r = sweep[1]
    time_ms(lambda: fwd(g_r), 300)
    roofline = dominant_kernel_roofline(wl_r, g_r, fwd, time_ms, binding, max(100, args.steps))
    # ... and beside it a kernel that only streams the same bytes in the same read : write mix
    roofline["stream_reference"] = stream_reference(g_r, time_ms, bench_probe, max(100, args.steps))
    roofline["frac_of_stream_reference"] = round(
        roofline["stream_reference"]["reads3_writes1"]["launch_ms"] / roofline["launch_ms"], 4)
    bwd_r_ms = time_ms(lambda: bwd(g_r), max(100, args.steps), warm=20)
    roofline["bwd_vs_stream_reference"] = {
        "la2_bwd_ms": round(bwd_r_ms, 4),
        "stream_ms": round(roofline["stream_reference"]["reads3_writes1"]["launch_ms"]
                           + roofline["stream_reference"]["reads4_writes2"]["launch_ms"], 4)}
    roofline["bwd_vs_stream_reference"]["frac"] = round(
        roofline["bwd_vs_stream_reference"]["stream_ms"] / bwd_r_ms, 4)

    # ---- the timed region: W warm-up steps, then exactly K steps ----------------------------------
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_step = sum(wl.tokens for wl, _ in sweep)
    value = tokens_per_step / (ms_per_step * 1e-3)

    # ---- per-point table ----------------------------------------------------------------------------------
    iters = max(5, args.steps)
    points = []
    for wl, g in sweep:
        f_ms = time_ms(lambda: fwd(g), iters)
        b_ms = time_ms(lambda: bwd(g), iters)
        th, d, B = wl.token_heads, wl.head_dim, g["B"]
        tot = f_ms + b_ms
        fl = flops_per_token_head(B, d, "fwd+bwd") * th
        points.append({
            "workload": wl.name, "batch": wl.batch, "seq_len": wl.seqlen, "B": B,
            "fwd_ms": round(f_ms, 4), "bwd_ms": round(b_ms, 4),
            "tokens_per_s": round(wl.tokens / (tot * 1e-3), 1),
            "tflops": round(fl / (tot * 1e-3) / 1e12, 2),
            "frac_bf16_peak": round(fl / (tot * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
            # algorithmic HBM bytes (8 d forward, 20 d backward per token-head, bf16) over the time
            "algorithmic_GBs": round(28 * d * th / (tot * 1e-3) / 1e9, 1),
            "frac_hbm_peak": round(28 * d * th / (tot * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
            "fwd_tflops": round(flops_per_token_head(B, d, "fwd") * th / (f_ms * 1e-3) / 1e12, 2),
            "bwd_tflops": round(flops_per_token_head(B, d, "bwd") * th / (b_ms * 1e-3) / 1e12, 2),
            # device memory beside the 8 tensors of a training step (q, k, v, o, d_o, dq, dk, dv: linear in n):
            # the library's own workspace (chunk start states; 0 when the chains alone fill the GPU)
            "tensor_MiB": round(8 * th * d * 2 / 2**20, 1),
            "workspace_MiB": round(max(binding.la2_workspace_bytes(g["q"], binding.LA2_OP_FWD),
                                       binding.la2_workspace_bytes(g["q"], binding.LA2_OP_BWD)) / 2**20, 1),
        })
    tps = [p["tokens_per_s"] for p in points]
    flatness = min(tps) / max(tps)


    # ---- the other configurations -------------------------------------------------------------------------
    others = []
    for wl in (workloads.CONFIG2, workloads.CONFIG4):
        g = stage(wl)
        f_ms = time_ms(lambda: fwd(g), iters, warm=40, settle_ms=80)   # freshly staged tensors: warm up as the sweep is
        b_ms = time_ms(lambda: bwd(g), iters, warm=40, settle_ms=80)
        tot = f_ms + b_ms
        fl = flops_per_token_head(g["B"], wl.head_dim, "fwd+bwd") * wl.token_heads
        others.append({"workload": wl.name, "B": g["B"], "fwd_ms": round(f_ms, 4), "bwd_ms": round(b_ms, 4),
                       "tokens_per_s": round(wl.tokens / (tot * 1e-3), 1),
                       "tflops": round(fl / (tot * 1e-3) / 1e12, 2),
                       "frac_bf16_peak": round(fl / (tot * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)})
        del g
    # segments with state hand-over (start state in, final state out, their gradients) at the two middle
    # sweep points: the un-chunked and a sequence-chunked launch
    with_states = []
    for wl, g in sweep[1:3]:
        shape = (wl.batch, wl.heads, wl.head_dim, wl.head_dim)
        st = {n_: torch.zeros(shape, dtype=torch.float32, device=dev) for n_ in ("init", "fin", "d_fin", "d_init")}
        f_ms = time_ms(lambda: binding.la2_fwd_state(g["q"], g["k"], g["v"], g["lam"], kv_init=st["init"], out=g["o"],
                                                     kv_final=st["fin"], workspace=g["ws"]), iters, warm=40, settle_ms=80)
        b_ms = time_ms(lambda: binding.la2_bwd_state(g["q"], g["k"], g["v"], g["d_o"], g["lam"], kv_init=st["init"],
                                                     d_kv_final=st["d_fin"], out=g["grads"], d_kv_init=st["d_init"],
                                                     workspace=g["ws"]), iters, warm=40, settle_ms=80)
        with_states.append({"workload": wl.name + " + kv_init, kv_final, d_kv_final, d_kv_init",
                            "fwd_ms": round(f_ms, 4), "bwd_ms": round(b_ms, 4),
                            "tokens_per_s": round(wl.tokens / ((f_ms + b_ms) * 1e-3), 1)})
        del st
    # the operator with its output normalisation (eq. (2); la2_fwd_norm / la2_bwd_norm) beside the plain one
    normed = []
    # two sweep points, and head_dim 64: config 2 and a batch that gives every compute unit one chain
    wl_n64 = workloads.Workload("b16_n4096_h16_d64", 16, 16, 4096, 64, torch.bfloat16, seed=72)
    for wl, g in sweep[1:3] + [(workloads.CONFIG2, stage(workloads.CONFIG2)), (wl_n64, stage(wl_n64))]:
        rstd = torch.empty(g["q"].shape[:3], dtype=torch.float32, device=dev)
        d_u = torch.empty_like(g["q"])
        f_ms = time_ms(lambda: binding.la2_fwd_norm(g["q"], g["k"], g["v"], g["lam"], 1e-6, out=g["o"], rstd=rstd,
                                                    workspace=g["ws"]), iters, warm=40, settle_ms=80)
        b_ms = time_ms(lambda: binding.la2_bwd_norm(g["q"], g["k"], g["v"], g["o"], rstd, g["d_o"], g["lam"],
                                                    out=g["grads"], d_u=d_u, workspace=g["ws"]), iters, warm=40, settle_ms=80)
        pf_ms = time_ms(lambda: fwd(g), iters, warm=40, settle_ms=80)
        pb_ms = time_ms(lambda: bwd(g), iters, warm=40, settle_ms=80)
        normed.append({"workload": wl.name + " + Norm (rms over head_dim, eps 1e-6)",
                       "fwd_ms": round(f_ms, 4), "bwd_ms": round(b_ms, 4),
                       "tokens_per_s": round(wl.tokens / ((f_ms + b_ms) * 1e-3), 1),
                       "plain_fwd_ms": round(pf_ms, 4), "plain_bwd_ms": round(pb_ms, 4)})
        del rstd, d_u
    # a packed batch of sequences of different lengths (la2_fwd_varlen / la2_bwd_varlen): 65,536 positions as
    # 1 x 8192, 2 x 4096, 4 x 2048, 8 x 1024, 16 x 512, 32 x 256 and 128 x 128 positions, longest first
    lengths = [8192] + [4096] * 2 + [2048] * 4 + [1024] * 8 + [512] * 16 + [256] * 32 + [128] * 128
    wl_p = workloads.Workload("packed_lengths_128_to_8192_h16_d128", 1, 16, sum(lengths), 128, torch.bfloat16, seed=34)
    tp = wl_p.tensors()
    gp = {n_: tp[n_][0].permute(1, 0, 2).contiguous().to(dev) for n_ in ("q", "k", "v", "d_o")}   # [total, H, d]
    gp["lam"] = tp["lam"].to(dev)
    cu = torch.tensor([0] + list(__import__("itertools").accumulate(lengths)), dtype=torch.int32, device=dev)
    op_, gr_ = torch.empty_like(gp["q"]), tuple(torch.empty_like(gp["q"]) for _ in range(3))
    f_ms = time_ms(lambda: binding.la2_fwd_varlen(gp["q"], gp["k"], gp["v"], gp["lam"], cu, max(lengths), out=op_),
                   iters, warm=40, settle_ms=80)
    b_ms = time_ms(lambda: binding.la2_bwd_varlen(gp["q"], gp["k"], gp["v"], gp["d_o"], gp["lam"], cu, max(lengths),
                                                  out=gr_), iters, warm=40, settle_ms=80)
    packed = {"workload": wl_p.name, "sequences": len(lengths), "tokens": sum(lengths), "fwd_ms": round(f_ms, 4),
              "bwd_ms": round(b_ms, 4), "tokens_per_s": round(sum(lengths) / ((f_ms + b_ms) * 1e-3), 1),
              "note": "the library cuts the long sequences into chunks (planned from the longest length and the total)"}
    del gp, op_, gr_, tp
    # the same point in the library's other two data types (fp16: the same kernels as bf16; fp32: fp32 MFMA)
    other_dtypes = []
    wl1 = workloads.CONFIG3[1]
    for dt, tag in ((torch.float16, "f16"), (torch.float32, "f32")):
        wl_d = workloads.Workload(wl1.name + "_" + tag, wl1.batch, wl1.heads, wl1.seqlen, wl1.head_dim, dt, seed=wl1.seed)
        g_d = stage(wl_d)
        f_ms = time_ms(lambda: fwd(g_d), iters, warm=40, settle_ms=80)
        b_ms = time_ms(lambda: bwd(g_d), iters, warm=40, settle_ms=80)
        other_dtypes.append({"workload": wl_d.name, "dtype": tag, "fwd_ms": round(f_ms, 4), "bwd_ms": round(b_ms, 4),
                             "tokens_per_s": round(wl_d.tokens / ((f_ms + b_ms) * 1e-3), 1)})
        del g_d
    # the other head dimensions (one plain block kernel for both), at the tensor sizes of the sweep's first two
    # points (heads x head_dim = 2048 for 256, 1536 for 96)
    other_head_dims = []
    for hd, heads in ((256, 8), (96, 16)):
        for b_, n_ in ((64, 1024), (16, 4096)):
            wl_h = workloads.Workload("b%d_n%d_h%d_d%d" % (b_, n_, heads, hd), b_, heads, n_, hd, torch.bfloat16, seed=60 + hd)
            g_h = stage(wl_h)
            f_ms = time_ms(lambda: fwd(g_h), iters, warm=40, settle_ms=80)
            b_ms = time_ms(lambda: bwd(g_h), iters, warm=40, settle_ms=80)
            unit = wl_h.token_heads * hd * 2   # bytes of one tensor
            other_head_dims.append({"workload": wl_h.name, "fwd_ms": round(f_ms, 4), "bwd_ms": round(b_ms, 4),
                                    "tokens_per_s": round(wl_h.tokens / ((f_ms + b_ms) * 1e-3), 1),
                                    "fwd_algorithmic_GBs": round(4 * unit / f_ms / 1e6, 1),
                                    "bwd_algorithmic_GBs": round(10 * unit / b_ms / 1e6, 1)})
            del g_h
    # a batch a little above one chain per compute unit (320 chains on 256 units): the library runs it as two calls,
    # the first 256 chains whole and the other 64 in chunks; with a chunk size set by the caller (here the whole
    # sequence) it runs as one call, in which 64 units get a second workgroup and set the launch's time
    wl_u = workloads.Workload("b20_n4096_h16_d128", 20, 16, 4096, 128, torch.bfloat16, seed=71)
    g_u = stage(wl_u)
    f_ms = time_ms(lambda: fwd(g_u), iters, warm=40, settle_ms=80)
    b_ms = time_ms(lambda: bwd(g_u), iters, warm=40, settle_ms=80)
    binding.la2_set_chunk_tokens(wl_u.seqlen)
    try:
        assert binding.la2_workspace_bytes(g_u["q"], binding.LA2_OP_BWD) == 0
        f1_ms = time_ms(lambda: fwd(g_u), iters, warm=40, settle_ms=80)
        b1_ms = time_ms(lambda: bwd(g_u), iters, warm=40, settle_ms=80)
    finally:
        binding.la2_set_chunk_tokens(0)
    uneven = {"workload": wl_u.name, "fwd_ms": round(f_ms, 4), "bwd_ms": round(b_ms, 4),
              "tokens_per_s": round(wl_u.tokens / ((f_ms + b_ms) * 1e-3), 1),
              "as_one_call": {"fwd_ms": round(f1_ms, 4), "bwd_ms": round(b1_ms, 4),
                              "tokens_per_s": round(wl_u.tokens / ((f1_ms + b1_ms) * 1e-3), 1)}}
    del g_u
    # forward and backward pass as O(n^2 d) masked left products (comparison kernel) against the block recurrence
    crossover = []
    short = [(wl_, stage(wl_)) for wl_ in (workloads.Workload("config3_like_b%d_n%d_h16_d128" % (b_, n_), b_, 16, n_, 128,
                                                              torch.bfloat16, seed=40 + i_)
                                           for i_, (b_, n_) in enumerate(((512, 128), (256, 256), (128, 512))))]
    for wl, g in short + sweep:
        lp_iters = max(2, min(iters, int(50e9 // (wl.seqlen * wl.tokens))))   # ~n^2 work: fewer launches when long
        lp_ms = time_ms(lambda: binding.la2_left_product_fwd(g["q"], g["k"], g["v"], g["lam"], out=g["o"]), lp_iters)
        lpb_ms = time_ms(lambda: binding.la2_left_product_bwd(g["q"], g["k"], g["v"], g["d_o"], g["lam"], out=g["grads"]),
                         max(2, lp_iters // 3))
        f_ms = time_ms(lambda: fwd(g), iters)
        b_ms = time_ms(lambda: bwd(g), iters)
        crossover.append({"workload": wl.name, "left_product_fwd_ms": round(lp_ms, 4),
                          "block_recurrence_fwd_ms": round(f_ms, 4), "ratio": round(lp_ms / f_ms, 2),
                          "left_product_bwd_ms": round(lpb_ms, 4), "block_recurrence_bwd_ms": round(b_ms, 4),
                          "bwd_ratio": round(lpb_ms / b_ms, 2)})
    del short

    # training step that keeps the forward's workspace for the backward (la2_bwd_saved): the sequence-chunked
    # points then skip one of the backward's two chunk-state pre-passes.  Reported beside the headline, which
    # stays on the stand-alone la2_fwd + la2_bwd.
    saved = []
    for wl, g in sweep:
        ws_b = torch.empty_like(g["ws"])
        f_ms = time_ms(lambda: fwd(g), iters, settle_ms=40)
        b_ms = time_ms(lambda: binding.la2_bwd_state(g["q"], g["k"], g["v"], g["d_o"], g["lam"], want_d_kv_init=False,
                                                     out=g["grads"], workspace=ws_b, fwd_workspace=g["ws"]), iters)
        saved.append({"workload": wl.name + " (backward reuses the forward's chunk states)",
                      "fwd_ms": round(f_ms, 4), "bwd_ms": round(b_ms, 4),
                      "tokens_per_s": round(wl.tokens / ((f_ms + b_ms) * 1e-3), 1)})
        del ws_b
    tps_saved = [p_["tokens_per_s"] for p_ in saved]
    training_step = {"what": "la2_fwd, then la2_bwd_saved on the forward call's workspace, at the four sweep points",
                     "flatness_min_over_max": round(min(tps_saved) / max(tps_saved), 4),
                     "tokens_per_s": round(sum(wl.tokens for wl, _ in sweep)
                                           / sum((p_["fwd_ms"] + p_["bwd_ms"]) * 1e-3 for p_ in saved), 1),
                     "sweep": saved}
    torch.cuda.empty_cache()

    # decode: 1024 consecutive steps, state updated in place
    dw = workloads.CONFIG5
    gen = dw.generator()
    kv = dw.initial_state(gen).to(dev)
    lam5 = dw.decay().to(dev)
    toks = [tuple(x.to(dev) for x in dw.token(gen)) for _ in range(16)]
    o5 = torch.empty_like(toks[0][0])
    for i in range(768):   # about 60 ms: the host staged the state and the tokens, the device has been idle
        binding.la2_decode_step(*toks[i % 16], lam5, kv, out=o5)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(dw.steps):
        binding.la2_decode_step(*toks[i % 16], lam5, kv, out=o5)
    e1.record()
    torch.cuda.synchronize()
    dec_ms = e0.elapsed_time(e1) / dw.steps
    dd = dw.head_dim
    dec_bytes = dw.batch * dw.heads * (2 * dd * dd * 4 + 4 * dd * 2)
    decode = {"workload": dw.name, "steps": dw.steps, "us_per_step": round(dec_ms * 1e3, 2),
              "tokens_per_s": round(dw.batch / (dec_ms * 1e-3), 1),
              "achieved_GBs": round(dec_bytes / (dec_ms * 1e-3) / 1e9, 1),
              "frac_hbm_peak": round(dec_bytes / (dec_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
    # beside it: a kernel that only streams the state's bytes in and as many bytes out
    kv_bytes = kv.numel() * kv.element_size()
    kv_u8 = kv.view(torch.uint8).reshape(-1)
    kv_out = torch.empty_like(kv_u8)
    sref_ms = min(time_ms(lambda: bench_probe.stream_probe(1, 1, kv_u8, kv_out, kv_bytes, nt_stores=nts), 200, warm=20)
                  for nts in (False, True))
    del kv_out
    decode["stream_reference"] = {"kernel": "1 stream in, 1 out, the state's %d MiB each, no arithmetic" % (kv_bytes >> 20),
                                  "us_per_launch": round(sref_ms * 1e3, 2),
                                  "frac_of_stream_reference": round(sref_ms / dec_ms, 4)}
    # the same tokens 8 per launch (multi-token decode): the state is read and written once per launch
    T = 8
    qm, km, vm = (torch.stack([toks[i][j] for i in range(T)], 2).contiguous() for j in range(3))
    om = torch.empty_like(qm)
    for _ in range(4):
        binding.la2_decode_multi(qm, km, vm, lam5, kv, out=om)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(dw.steps // T):
        binding.la2_decode_multi(qm, km, vm, lam5, kv, out=om)
    e1.record()
    torch.cuda.synchronize()
    dm_ms = e0.elapsed_time(e1) / (dw.steps // T)
    decode["multi_token"] = {"tokens_per_launch": T, "us_per_launch": round(dm_ms * 1e3, 2),
                             "tokens_per_s": round(dw.batch * T / (dm_ms * 1e-3), 1)}
    del kv, qm, km, vm, om

    # ---- CPU baseline: the fp64 oracle (direct O(n^2) form) on a bounded sample ---------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        wl_c = workloads.CONFIG3[1]
        heads_c, rows_c = wl_c.heads, 4     # 64 (batch row, head) chains: about 10 s on 16 host threads
        t = wl_c.tensors()
        f64 = lambda x: x[0:rows_c, :heads_c].double().numpy()
        q, k, v, do = (f64(t[x]) for x in ("q", "k", "v", "d_o"))
        lam = t["lam"][:heads_c].double().numpy()
        c0 = time.perf_counter()
        oracle.fwd_direct(q, k, v, lam)
        oracle.bwd_direct(q, k, v, do, lam)
        c1 = time.perf_counter()
        # ... and the oracle's O(n d^2) recurrent form (what the all-chain full-size parity tests use) on the same sample
        oracle.fwd_recurrent(q, k, v, lam)
        oracle.bwd_recurrent(q, k, v, do, lam)
        c2 = time.perf_counter()
        cpu = {"value": round(wl_c.seqlen * rows_c / (c1 - c0), 2), "unit": "tokens/s",
               "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "fp64 direct O(n^2) oracle, fwd+bwd, all %d heads of batch rows 0..%d of %s (%.1f s)"
                         % (heads_c, rows_c - 1, wl_c.name, c1 - c0),
               "recurrent_form": {"value": round(wl_c.seqlen * rows_c / (c2 - c1), 2), "unit": "tokens/s",
                                  "sample": "fp64 token recurrence, fwd+bwd, same sample (%.1f s)" % (c2 - c1)}}

    out = {
        "metric": "causal linear-attn fwd+bwd tokens/s (sequence-length sweep n=1K-64K at 65,536 tokens per point)",
        "value": round(value, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "config3 sweep: (batch,n) in {(64,1K),(16,4K),(4,16K),(1,64K)}, H=16, d=128, "
                               "fwd+bwd, bf16 in/out, fp32 accumulate",
                   "tokens_per_step": tokens_per_step, "block_size_B": points[0]["B"],
                   "flops_per_token_head": "fwd 4Bd+4d^2, bwd 12Bd+10d^2"},
        "tflops": round(sum(flops_per_token_head(p["B"], 128, "fwd+bwd") for p in points) * 1048576
                        / (ms_per_step * 1e-3) / 1e12, 2),
        "flatness_min_over_max": round(flatness, 4),
        "sweep": points,
        "other_configs": others,
        "state_handover": with_states,
        "training_step_saved_forward_states": training_step,
        "normalised_operator": normed,
        "other_dtypes": other_dtypes,
        "other_head_dims": other_head_dims,
        "packed_varlen": packed,
        "batch_a_little_above_one_chain_per_unit": uneven,
        "left_product_comparison": crossover,
        "decode": decode,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    out["frac_bf16_peak"] = round(out["tflops"] / PEAK_BF16_TFLOPS, 4)
    # The matrix pipes' own rate on this machine, measured last (the loop heats the chip: run before the timed
    # region it costs the memory-bound kernels 3-5 %): a register-only loop of the same MFMA instruction.
    mfma_measured = mfma_peak_tflops(time_ms, bench_probe, dev)
    roofline["mfma_loop_tflops_measured_in_this_run"] = round(mfma_measured, 1)
    for p_ in points:
        p_["frac_measured_mfma_peak"] = round(p_["tflops"] / mfma_measured, 4)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
