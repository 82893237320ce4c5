#!/usr/bin/env python3
"""Benchmark of the cosine-attention hot path on ONE MI355X.

A step is one causal forward + backward (cottn_fwd_causal + cottn_bwd_causal through the C
ABI) over one synthetic batch of the GPT-shaped workload  B=8, H=12, N=1024, d=64, bf16
inputs / fp32 accumulation.  Inputs are resident in HBM before the timed region; the step
rotates over several independent buffer sets so that the tensors are not served from the
256 MB last-level cache left warm by the previous step.

Prints ONE JSON line: throughput in tokens/s (tokens = B*N per step), the roofline of the
dominant kernel (per-kernel durations from HIP events inside the library, a second pass of
the same steps), and the CPU oracle timed on the host cores as a reported baseline.

``--workload NAME`` times one of the other configurations alone (what the rocprofv3 summaries
under profiles/ are taken from) and prints that configuration's figures as one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 MFMA rate
TRAFFIC_FILE = os.path.join("profiles", "hbm_traffic_cfg2.json")


def flop_rates(token_heads, d, chunk, seconds, bidirectional=False):
    """Algorithmic flops of linear attention (14 d^2 per token-head for causal fwd+bwd, 12 d^2
    bidirectional) and those a chunked MFMA design executes (14 (C + d) d; the bidirectional
    path has no chunk-quadratic part), as rates and as fractions of the bf16 MFMA peak."""
    alg = (12 if bidirectional else 14) * d * d * token_heads
    exe = alg if bidirectional else 14 * (chunk + d) * d * token_heads
    return {"algorithmic_TFLOPs": alg / seconds / 1e12, "executed_TFLOPs": exe / seconds / 1e12,
            "executed_frac_of_mfma_peak": exe / seconds / 1e12 / MFMA_BF16_PEAK_TFLOPS}

# Algorithmic HBM bytes per token-head (one row of one (batch, head)) for each kernel, in
# units of d * element_size: the tensors the kernel must read plus those it must write.
KERNEL_ROW_TENSORS = {
    "fwd_causal_scan_bf16": 4,      # Q, K, V in; O out
    "bwd_dq_scan_bf16": 5,          # Q, K, V, dO in; dQ out
    "bwd_dkdv_scan_bf16": 6,        # Q, K, V, dO in; dK, dV out
    "fwd_segment_state_bf16": 2,    # K, V in (state totals are d*d per segment, added below)
}


def time_calls(torch, fn, iters, warmup):
    """Average milliseconds of fn(i) over `iters` calls on the current stream."""
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(iters):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def kernel_times(cottn, fn, iters):
    """Per-kernel average microseconds from the library's own HIP events over `iters` calls."""
    cottn.profile_start()
    for i in range(iters):
        fn(i)
    prof = cottn.profile_stop()
    return {name: {"launches_per_step": n / iters, "avg_us": 1e3 * ms / n} for name, (n, ms) in prof.items()}


def oracle_rate(fn, tokens, repeat=1):
    """tokens per second of the CPU oracle (fp64, as it stands) over `repeat` calls of fn, each
    of which processes `tokens` tokens; also the seconds all of them took."""
    t0 = time.perf_counter()
    for _ in range(repeat):
        fn()
    dt = time.perf_counter() - t0
    return repeat * tokens / dt, dt


# ---- the other configurations, each timed briefly (random bf16 values of the configured shapes;
# ---- correctness of these shapes is the parity tests' job)

def run_decode(torch, cottn, workloads, cpu):
    """256 sequences x 16 heads, d = 128; one call per token, the fp32 states stream through.
    The calls rotate over three sets of states (805 MB): more than the 256 MB last-level cache
    holds, so no step finds its states cached by the previous one."""
    dev = torch.device("cuda:0")
    rnd = lambda *shape: torch.randn(*shape, device=dev).to(torch.bfloat16)
    w = workloads.WORKLOADS["cfg5_decode_bf16"]
    B, H, d = w.B, w.H, w.d
    n_states = 3
    states = [torch.zeros(B, H, d, d, dtype=torch.float32, device=dev) for _ in range(n_states)]
    T = 32
    q, k, v = rnd(T, B, H, d), rnd(T, B, H, d), rnd(T, B, H, d)
    o = torch.empty_like(q)
    s = torch.ones(H, device=dev)
    call = lambda i: cottn.cottn_step(q[i % T], k[i % T], v[i % T], s, states[i % n_states], o=o[i % T])
    ms = time_calls(torch, call, 402, 21)
    byt = 2 * B * H * d * d * 4
    out = {"us_per_step": ms * 1e3, "tokens_per_s": B / (ms * 1e-3),
           "state_bytes_read_plus_written": byt, "state_sets_rotated": n_states,
           "achieved_GBs": byt / ms / 1e6, "frac_of_hbm_peak": byt / ms / 1e6 / HBM_PEAK_GBS,
           "kernels": kernel_times(cottn, call, 60)}
    if cpu:
        import numpy as np
        import oracle
        Bs = 16  # sequences of the sample
        rng = np.random.default_rng(0)
        qs, ks, vs = (rng.standard_normal((Bs, H, d)) for _ in range(3))
        S = np.zeros((Bs, H, d, d))
        rate, dt = oracle_rate(lambda: [oracle.step(qs, ks, vs, np.ones(H), S) for _ in range(8)], 8 * Bs, repeat=50)
        out["cpu_oracle"] = {"tokens_per_s": rate, "cores": oracle.num_threads(),
                             "sample": "400 steps of %d of the %d sequences (fp64 recurrence), %.1f s" % (Bs, B, dt)}
    return out


def run_bidir(torch, cottn, workloads, cpu):
    """BERT-shaped bidirectional forward + backward."""
    dev = torch.device("cuda:0")
    rnd = lambda *shape: torch.randn(*shape, device=dev).to(torch.bfloat16)
    w = workloads.WORKLOADS["cfg3_bert_bidir_fwdbwd_bf16"]
    B, H, N, d = w.B, w.H, w.N, w.d
    sets = []
    for _ in range(2):
        t = {n: rnd(B, H, N, d) for n in ("Q", "K", "V", "dO")}
        t.update({n: torch.empty_like(t["Q"]) for n in ("O", "dQ", "dK", "dV")})
        sets.append(t)
    s = torch.ones(H, device=dev)
    ds = torch.empty(H, device=dev)
    fwd_ws = torch.empty(max(cottn.cottn_workspace_bytes(cottn.OP_FWD_BIDIR, B, H, N, d), 256),
                         dtype=torch.uint8, device=dev)
    ws = torch.empty(cottn.cottn_workspace_bytes(cottn.OP_BWD_BIDIR, B, H, N, d),
                     dtype=torch.uint8, device=dev)

    def bidir(i):
        t = sets[i % 2]
        cottn.cottn_fwd_bidir(t["Q"], t["K"], t["V"], s, O=t["O"], workspace=fwd_ws)
        cottn.cottn_bwd_bidir(t["Q"], t["K"], t["V"], s, t["dO"], dQ=t["dQ"], dK=t["dK"],
                              dV=t["dV"], ds=ds, workspace=ws, fwd_workspace=fwd_ws)
    ms = time_calls(torch, bidir, 100, 10)
    byt = 11 * B * H * N * d * 2
    out = {"ms_per_step": ms, "tokens_per_s": B * N / (ms * 1e-3), "algorithmic_GBs": byt / ms / 1e6,
           "frac_of_hbm_peak": byt / ms / 1e6 / HBM_PEAK_GBS,
           "flops": flop_rates(B * H * N, d, 64, ms * 1e-3, True),
           "workspace_bytes": ws.numel() + fwd_ws.numel(), "kernels": kernel_times(cottn, bidir, 50)}
    if cpu:
        import oracle
        Bs = 4
        x = workloads.draw(Bs, H, N, d, "bf16", w.seed)
        rate, dt = oracle_rate(lambda: (oracle.fwd_quadratic(x["Q"], x["K"], x["V"], x["s"], causal=False),
                                        oracle.bwd_quadratic(x["Q"], x["K"], x["V"], x["s"], x["dO"], causal=False)),
                               Bs * N, repeat=10)
        out["cpu_oracle"] = {"tokens_per_s": rate, "cores": oracle.num_threads(),
                             "sample": "10 times %d of the %d sequences: fp64 quadratic-definition forward + backward, %.1f s" % (Bs, B, dt)}
    return out


def run_long(torch, cottn, workloads, cpu, chunks=(64, 128, 256)):
    """Long-context causal forward + backward, N = 65536, for each chunk size."""
    dev = torch.device("cuda:0")
    rnd = lambda *shape: torch.randn(*shape, device=dev).to(torch.bfloat16)
    w = workloads.WORKLOADS["cfg4_long_causal_fwdbwd_bf16"]
    B, H, N, d = w.B, w.H, w.N, w.d
    t = {n: rnd(B, H, N, d) * 0.5 for n in ("Q", "K", "V", "dO")}
    t.update({n: torch.empty_like(t["Q"]) for n in ("O", "dQ", "dK", "dV")})
    s = torch.ones(H, device=dev)
    ds = torch.empty(H, device=dev)
    out = {}
    for chunk in chunks:
        fwd_ws = torch.empty(max(cottn.cottn_workspace_bytes(cottn.OP_FWD_CAUSAL, B, H, N, d, chunk),
                                 256), dtype=torch.uint8, device=dev)
        ws = torch.empty(cottn.cottn_workspace_bytes(cottn.OP_BWD_CAUSAL, B, H, N, d, chunk),
                         dtype=torch.uint8, device=dev)

        def long_ctx(i):
            cottn.cottn_fwd_causal(t["Q"], t["K"], t["V"], s, O=t["O"], workspace=fwd_ws, chunk=chunk)
            cottn.cottn_bwd_causal(t["Q"], t["K"], t["V"], s, t["dO"], dQ=t["dQ"], dK=t["dK"],
                                   dV=t["dV"], ds=ds, workspace=ws, chunk=chunk, fwd_workspace=fwd_ws)
        ms = time_calls(torch, long_ctx, 20, 3)
        byt = 11 * B * H * N * d * 2
        out["cfg4_long_context_chunk%d" % chunk] = {
            "ms_per_step": ms, "tokens_per_s": B * N / (ms * 1e-3), "algorithmic_GBs": byt / ms / 1e6,
            "frac_of_hbm_peak": byt / ms / 1e6 / HBM_PEAK_GBS,
            "flops": flop_rates(B * H * N, d, chunk, ms * 1e-3),
            "segments": cottn.cottn_segments(cottn.OP_FWD_CAUSAL, B, H, N, d, chunk),
            "workspace_bytes": ws.numel() + fwd_ws.numel(),
            "tuned": chunk == 64,  # 128 and 256 are supported and parity-tested, not tuned
            "kernels": kernel_times(cottn, long_ctx, 10)}
    if cpu:
        import oracle
        Ns = 8192
        x = workloads.draw(B, H, Ns, d, "bf16", w.seed, w.value_scale)
        rate, dt = oracle_rate(lambda: (oracle.fwd_recurrent(x["Q"], x["K"], x["V"], x["s"]),
                                        oracle.bwd_recurrent(x["Q"], x["K"], x["V"], x["s"], x["dO"])),
                               B * Ns, repeat=10)
        out["cfg4_long_context_chunk64"]["cpu_oracle"] = {
            "tokens_per_s": rate, "cores": oracle.num_threads(),
            "sample": "10 times the first %d of the %d tokens of all %d heads: fp64 linear-time (recurrent) forward + backward, %.1f s" % (Ns, N, H, dt)}
    return out


def run_d128(torch, cottn, workloads, cpu):
    """The GPT-shaped step at head dimension 128 (4x the flops per byte of d = 64: the shape
    where the MFMA rate, not only HBM, is worth reporting)."""
    dev = torch.device("cuda:0")
    rnd = lambda *shape: torch.randn(*shape, device=dev).to(torch.bfloat16)
    B, H, N, d = 8, 12, 1024, 128
    t = {n: rnd(B, H, N, d) for n in ("Q", "K", "V", "dO")}
    t.update({n: torch.empty_like(t["Q"]) for n in ("O", "dQ", "dK", "dV")})
    s = torch.ones(H, device=dev)
    ds = torch.empty(H, device=dev)
    fwd_ws = torch.empty(max(cottn.cottn_workspace_bytes(cottn.OP_FWD_CAUSAL, B, H, N, d), 256),
                         dtype=torch.uint8, device=dev)
    ws = torch.empty(cottn.cottn_workspace_bytes(cottn.OP_BWD_CAUSAL, B, H, N, d),
                     dtype=torch.uint8, device=dev)

    def d128(i):
        cottn.cottn_fwd_causal(t["Q"], t["K"], t["V"], s, O=t["O"], workspace=fwd_ws)
        cottn.cottn_bwd_causal(t["Q"], t["K"], t["V"], s, t["dO"], dQ=t["dQ"], dK=t["dK"],
                               dV=t["dV"], ds=ds, workspace=ws, fwd_workspace=fwd_ws)
    ms = time_calls(torch, d128, 100, 10)
    byt = 11 * B * H * N * d * 2
    chunk = 64
    return {"ms_per_step": ms, "tokens_per_s": B * N / (ms * 1e-3), "algorithmic_GBs": byt / ms / 1e6,
            "frac_of_hbm_peak": byt / ms / 1e6 / HBM_PEAK_GBS,
            "flops": flop_rates(B * H * N, d, chunk, ms * 1e-3),
            "segments": cottn.cottn_segments(cottn.OP_FWD_CAUSAL, B, H, N, d),
            "kernels": kernel_times(cottn, d128, 50)}


def run_sweep(torch, cottn, workloads, cpu, dims=(32, 64, 128), max_n=1 << 20, heads=16):
    """Time and memory of forward + backward against sequence length and head dimension (the
    sweep of Sec. 7, this library's side; no comparison system): B = 1, `heads` heads, bf16, the
    backward handed the forward's workspace.  With the CPU leg, the linear-time oracle (fp64
    recurrence, forward + backward) is timed beside every row up to N = 4096, and the
    quadratic-definition oracle up to N = 1024: the first grows like N, the second like N^2."""
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    B, H = 1, heads
    rows = []
    for mode in ("causal", "bidirectional"):
        causal = mode == "causal"
        fwd = cottn.cottn_fwd_causal if causal else cottn.cottn_fwd_bidir
        bwd = cottn.cottn_bwd_causal if causal else cottn.cottn_bwd_bidir
        ops = (cottn.OP_FWD_CAUSAL, cottn.OP_BWD_CAUSAL) if causal else (cottn.OP_FWD_BIDIR, cottn.OP_BWD_BIDIR)
        for d in dims:
            N = 256
            while N <= max_n:
                t = {n: (torch.randn(B, H, N, d, device=dev, generator=gen) * 0.5).to(torch.bfloat16)
                     for n in ("Q", "K", "V", "dO")}
                t.update({n: torch.empty_like(t["Q"]) for n in ("O", "dQ", "dK", "dV")})
                s = torch.ones(H, device=dev)
                ds = torch.empty(H, device=dev)
                fb = max(cottn.cottn_workspace_bytes(ops[0], B, H, N, d), 256)
                bb = max(cottn.cottn_workspace_bytes(ops[1], B, H, N, d), 256)
                fws = torch.empty(fb, dtype=torch.uint8, device=dev)
                bws = torch.empty(bb, dtype=torch.uint8, device=dev)

                def step(i):
                    fwd(t["Q"], t["K"], t["V"], s, O=t["O"], workspace=fws)
                    bwd(t["Q"], t["K"], t["V"], s, t["dO"], dQ=t["dQ"], dK=t["dK"], dV=t["dV"], ds=ds,
                        workspace=bws, fwd_workspace=fws)
                ms = time_calls(torch, step, 50 if N <= 16384 else 10 if N <= 262144 else 4, 3)
                row = {"mode": mode, "d": d, "N": N, "ms": ms, "tokens_per_s": B * N / (ms * 1e-3),
                       "tensor_bytes": 8 * B * H * N * d * 2, "workspace_bytes": fb + bb,
                       "segments": cottn.cottn_segments(ops[0], B, H, N, d),
                       "oracle_linear_ms": None, "oracle_quadratic_ms": None}
                if cpu and N <= 4096:
                    import oracle
                    x = {n: t[n].double().cpu().numpy() for n in ("Q", "K", "V", "dO")}
                    one = s.double().cpu().numpy()
                    if causal:
                        lin = lambda: (oracle.fwd_recurrent(x["Q"], x["K"], x["V"], one),
                                       oracle.bwd_recurrent(x["Q"], x["K"], x["V"], one, x["dO"]))
                        row["oracle_linear_ms"] = 1e3 * oracle_rate(lin, B * N)[1]
                    if N <= 1024:
                        quad = lambda: (oracle.fwd_quadratic(x["Q"], x["K"], x["V"], one, causal=causal),
                                        oracle.bwd_quadratic(x["Q"], x["K"], x["V"], one, x["dO"], causal=causal))
                        row["oracle_quadratic_ms"] = 1e3 * oracle_rate(quad, B * N)[1]
                rows.append(row)
                print("sweep %s d=%d N=%d: %.3f ms" % (mode, d, N, ms), file=sys.stderr, flush=True)
                del t, fws, bws
                N *= 4
    out = {"batch": B, "heads": H, "dtype": "bf16", "rows": rows,
           "unsupported": "d = 256 (head dimensions are 32, 64, 128 in this library)"}
    if cpu:
        import oracle
        out["oracle_cores"] = oracle.num_threads()
    return out


OTHER = {"cfg5": ("cfg5_decode_step", run_decode), "cfg3": ("cfg3_bidir_fwd_bwd", run_bidir),
         "cfg4": (None, run_long), "d128": ("d128_causal_fwd_bwd_B8_H12_N1024", run_d128)}
# run only when named (--workload sweep): minutes of GPU and CPU time, not part of the default line
ON_REQUEST = {"sweep": ("time_memory_sweep", run_sweep)}


def other_workloads(torch, cottn, workloads, cpu, only=None):
    out = {}
    for key, (name, fn) in {**OTHER, **ON_REQUEST}.items():
        if key != only and (only is not None or key in ON_REQUEST):
            continue
        res = fn(torch, cottn, workloads, cpu)
        if name is None:
            out.update(res)
        else:
            out[name] = res
        torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--buffer-sets", type=int, default=4)
    ap.add_argument("--chunk", type=int, default=0)
    ap.add_argument("--segments", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the brief timings of the decode, bidirectional and long-context shapes")
    ap.add_argument("--workload", choices=sorted({**OTHER, **ON_REQUEST}), default=None,
                    help="time only this one of the other configurations (for profiling runs)")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run a plain device copy of this many MiB a few times before the "
                         "timed region: the reference dispatch for scaling rocprofv3 byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); no multi-GPU figure exists",
              file=sys.stderr)
        return 2

    import torch
    import paper_2409_18747_amd.binding as cottn
    from paper_2409_18747_amd import workloads

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.copy_calibration_mib:
        src = torch.empty(args.copy_calibration_mib << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.workload:
        print(json.dumps({"workload": args.workload,
                          **other_workloads(torch, cottn, workloads, not args.no_cpu_baseline, args.workload)}))
        return 0

    w = workloads.WORKLOADS["cfg2_gpt_causal_fwdbwd_bf16"]
    B, H, N, d = w.B, w.H, w.N, w.d
    if args.segments:
        cottn.cottn_tune_segments(args.segments)

    # buffer sets: the first holds the workload's seeded draw, the others are further draws
    sets = []
    for i in range(args.buffer_sets):
        x = workloads.draw(B, H, N, d, w.dtype, w.seed + 1000 * i, w.value_scale)
        t = {k: torch.from_numpy(x[k]).to(torch.bfloat16).to(dev) for k in ("Q", "K", "V", "dO")}
        t["s"] = torch.from_numpy(x["s"]).to(dev)
        for k in ("O", "dQ", "dK", "dV"):
            t[k] = torch.empty_like(t["Q"])
        t["ds"] = torch.empty(H, dtype=torch.float32, device=dev)
        sets.append(t)
        if i == 0:
            host_inputs = x
    # As in a training step, the backward is handed the forward's workspace: the forward-time
    # segment states it holds are what the forward saves for the backward.
    fwd_need = cottn.cottn_workspace_bytes(cottn.OP_FWD_CAUSAL, B, H, N, d, args.chunk)
    bwd_need = cottn.cottn_workspace_bytes(cottn.OP_BWD_CAUSAL, B, H, N, d, args.chunk)
    fwd_ws = torch.empty(max(fwd_need, 256), dtype=torch.uint8, device=dev)
    ws = torch.empty(max(bwd_need, 256), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def step(i):
        t = sets[i % len(sets)]
        cottn.cottn_fwd_causal(t["Q"], t["K"], t["V"], t["s"], O=t["O"], workspace=fwd_ws,
                               chunk=args.chunk, stream=stream)
        cottn.cottn_bwd_causal(t["Q"], t["K"], t["V"], t["s"], t["dO"], dQ=t["dQ"], dK=t["dK"],
                               dV=t["dV"], ds=t["ds"], workspace=ws, chunk=args.chunk,
                               stream=stream, fwd_workspace=fwd_ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for i in range(args.steps):
        step(i)
    e1.record(stream)
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / args.steps
    tokens_per_s = B * N / (ms_per_step * 1e-3)

    # second pass of the same steps with the library's per-kernel HIP events switched on
    kernels = kernel_times(cottn, step, args.steps)
    torch.cuda.synchronize()
    G_f = cottn.cottn_segments(cottn.OP_FWD_CAUSAL, B, H, N, d, args.chunk)
    G_b = cottn.cottn_segments(cottn.OP_BWD_CAUSAL, B, H, N, d, args.chunk)
    dom = max(kernels, key=lambda n: kernels[n]["avg_us"] * kernels[n]["launches_per_step"])
    rows = B * H * N
    elem = 2
    if dom not in KERNEL_ROW_TENSORS:
        raise SystemExit("bench.py: no algorithmic-bytes entry for the dominant kernel %r" % dom)
    alg_bytes = KERNEL_ROW_TENSORS[dom] * d * elem * rows
    dom_s = kernels[dom]["avg_us"] * 1e-6
    achieved = alg_bytes / dom_s / 1e9
    # Measured HBM bytes per launch of that kernel: NOT measured in this run (byte counters need a
    # rocprofv3 pass of their own) but read from the committed summary of such passes over this
    # same command; the source is named beside the figure, and a summary that does not know the
    # dominant kernel is an error, not a silent null.
    traffic = traffic_source = None
    tpath = os.path.join(ROOT, TRAFFIC_FILE)
    if not args.chunk and not args.segments:
        tj = json.load(open(tpath))
        if dom not in tj.get("bytes_per_launch", {}):
            raise SystemExit("bench.py: %s has no entry for the dominant kernel %r: re-run the "
                             "FETCH_SIZE / WRITE_SIZE passes it documents" % (TRAFFIC_FILE, dom))
        traffic = tj["bytes_per_launch"][dom]
        traffic_source = "%s (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes of this command, library source %s)" % (
            TRAFFIC_FILE, tj.get("library_source", "unrecorded"))
    roofline = {"kernel": dom, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "traffic": traffic, "traffic_source": traffic_source, "avg_us": dom_s * 1e6,
                "algorithmic_bytes": alg_bytes}
    # whole-step view: 11 tensors of B*H*N*d bf16 must cross HBM per fwd+bwd
    step_bytes = 11 * d * elem * rows
    step_gbs = step_bytes / (ms_per_step * 1e-3) / 1e9

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        hi = host_inputs
        # the linear-time oracle (the recurrence of Sec. 5 forward, the two cumulative sums of
        # Sec. 4 backward: the same O(N d^2) work as the GPU path), and the quadratic definition
        lin_rate, lin_dt = oracle_rate(lambda: (oracle.fwd_recurrent(hi["Q"], hi["K"], hi["V"], hi["s"]),
                                                oracle.bwd_recurrent(hi["Q"], hi["K"], hi["V"], hi["s"], hi["dO"])),
                                       B * N, repeat=40)
        quad_rate, quad_dt = oracle_rate(lambda: (oracle.fwd_quadratic(hi["Q"], hi["K"], hi["V"], hi["s"]),
                                                  oracle.bwd_quadratic(hi["Q"], hi["K"], hi["V"], hi["s"], hi["dO"])),
                                         B * N, repeat=8)
        cpu = {"value": lin_rate, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "40 full steps of the same workload (B=8,H=12,N=1024,d=64): fp64 linear-time "
                         "(recurrent) forward + backward, %.1f s" % lin_dt,
               "quadratic_definition": {"value": quad_rate, "unit": "tokens/s",
                                        "sample": "8 of the same steps by the fp64 quadratic definition "
                                                  "(forward + brute-force backward), %.1f s" % quad_dt}}

    out = {
        "metric": "causal cosine-attn fwd+bwd tokens/s (B8 H12 N1024 d64 bf16)",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "B": B, "H": H, "N": N, "d": d,
                   "chunk": args.chunk or 64, "segments_fwd": G_f, "segments_bwd": G_b,
                   "buffer_sets": len(sets), "workspace_bytes": fwd_need + bwd_need,
                   "step": "cottn_fwd_causal + cottn_bwd_causal (given the forward's workspace)"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "step_hbm": {"algorithmic_bytes": step_bytes, "achieved_GBs": step_gbs,
                     "frac_of_peak": step_gbs / HBM_PEAK_GBS},
        "step_flops": flop_rates(rows, d, args.chunk or 64, ms_per_step * 1e-3),
        "kernels": kernels,
    }
    if not args.no_other_workloads and not args.chunk and not args.segments:
        del sets
        torch.cuda.empty_cache()
        out["other_workloads"] = other_workloads(torch, cottn, workloads, not args.no_cpu_baseline)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
