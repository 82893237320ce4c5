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


def other_workloads(torch, cottn, workloads):
    """The other benchmark configurations, each timed briefly (random bf16 values of the
    configured shapes; correctness of these shapes is the parity tests' job)."""
    out = {}
    dev = torch.device("cuda:0")
    rnd = lambda *shape: torch.randn(*shape, device=dev).to(torch.bfloat16)

    # decode: 256 sequences x 16 heads, d = 128; one call per token, the fp32 state streams
    w = workloads.WORKLOADS["cfg5_decode_bf16"]
    B, H, d = w.B, w.H, w.d
    state = torch.zeros(B, H, d, d, dtype=torch.float32, device=dev)
    T = 32
    q, k, v = rnd(T, B, H, d), rnd(T, B, H, d), rnd(T, B, H, d)
    o = torch.empty_like(q)
    s = torch.ones(H, device=dev)
    ms = time_calls(torch, lambda i: cottn.cottn_step(q[i % T], k[i % T], v[i % T], s, state,
                                                      o=o[i % T]), 400, 20)
    byt = 2 * B * H * d * d * 4
    out["cfg5_decode_step"] = {"us_per_step": ms * 1e3, "tokens_per_s": B / (ms * 1e-3),
                               "state_bytes_read_plus_written": byt,
                               "achieved_GBs": byt / ms / 1e6, "frac_of_hbm_peak": byt / ms / 1e6 / HBM_PEAK_GBS}
    del state, q, k, v, o

    # BERT-shaped bidirectional forward + backward
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
    out["cfg3_bidir_fwd_bwd"] = {"ms_per_step": ms, "tokens_per_s": B * N / (ms * 1e-3),
                                 "algorithmic_GBs": byt / ms / 1e6,
                                 "frac_of_hbm_peak": byt / ms / 1e6 / HBM_PEAK_GBS,
                                 "flops": flop_rates(B * H * N, d, 64, ms * 1e-3, True)}
    del sets, ws, fwd_ws

    # long context causal forward + backward, N = 65536
    w = workloads.WORKLOADS["cfg4_long_causal_fwdbwd_bf16"]
    B, H, N, d = w.B, w.H, w.N, w.d
    t = {n: rnd(B, H, N, d) * 0.5 for n in ("Q", "K", "V", "dO")}
    t.update({n: torch.empty_like(t["Q"]) for n in ("O", "dQ", "dK", "dV")})
    s = torch.ones(H, device=dev)
    for chunk in (64, 128, 256):
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
            "workspace_bytes": ws.numel() + fwd_ws.numel()}

    # the GPT-shaped step at head dimension 128 (4x the flops per byte of d = 64: the shape
    # where the MFMA rate, not only HBM, is worth reporting)
    B, H, N, d = 8, 12, 1024, 128
    t = {n: rnd(B, H, N, d) for n in ("Q", "K", "V", "dO")}
    t.update({n: torch.empty_like(t["Q"]) for n in ("O", "dQ", "dK", "dV")})
    s = torch.ones(H, device=dev)
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
    out["d128_causal_fwd_bwd_B8_H12_N1024"] = {
        "ms_per_step": ms, "tokens_per_s": B * N / (ms * 1e-3), "algorithmic_GBs": byt / ms / 1e6,
        "frac_of_hbm_peak": byt / ms / 1e6 / HBM_PEAK_GBS,
        "flops": flop_rates(B * H * N, d, 64, ms * 1e-3),
        "segments": cottn.cottn_segments(cottn.OP_FWD_CAUSAL, B, H, N, d)}
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

    w = workloads.WORKLOADS["cfg2_gpt_causal_fwdbwd_bf16"]
    B, H, N, d = w.B, w.H, w.N, w.d
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
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
    fwd_ws = torch.empty(max(cottn.cottn_workspace_bytes(cottn.OP_FWD_CAUSAL, B, H, N, d, args.chunk),
                             256), dtype=torch.uint8, device=dev)
    ws = torch.empty(max(cottn.cottn_workspace_bytes(cottn.OP_BWD_CAUSAL, B, H, N, d, args.chunk),
                         256), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def step(i):
        t = sets[i % len(sets)]
        cottn.cottn_fwd_causal(t["Q"], t["K"], t["V"], t["s"], O=t["O"], workspace=fwd_ws,
                               chunk=args.chunk, stream=stream)
        cottn.cottn_bwd_causal(t["Q"], t["K"], t["V"], t["s"], t["dO"], dQ=t["dQ"], dK=t["dK"],
                               dV=t["dV"], ds=t["ds"], workspace=ws, chunk=args.chunk,
                               stream=stream, fwd_workspace=fwd_ws)

    if args.copy_calibration_mib:
        src = torch.empty(args.copy_calibration_mib << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

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
    cottn.profile_start()
    for i in range(args.steps):
        step(i)
    prof = cottn.profile_stop()
    torch.cuda.synchronize()
    G_f = cottn.cottn_segments(cottn.OP_FWD_CAUSAL, B, H, N, d, args.chunk)
    G_b = cottn.cottn_segments(cottn.OP_BWD_CAUSAL, B, H, N, d, args.chunk)
    kernels = {}
    for name, (launches, total_ms) in prof.items():
        kernels[name] = {"launches_per_step": launches / args.steps,
                         "avg_us": 1e3 * total_ms / launches}
    dom = max(prof, key=lambda n: prof[n][1])
    rows = B * H * N
    elem = 2
    alg_bytes = KERNEL_ROW_TENSORS.get(dom, 0) * d * elem * rows
    dom_s = prof[dom][1] / prof[dom][0] * 1e-3
    achieved = alg_bytes / dom_s / 1e9 if alg_bytes else None
    # measured HBM bytes per launch of that kernel, from the committed rocprofv3 counter summary
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_cfg2.json")
    if os.path.exists(tpath) and not args.chunk and not args.segments:
        traffic = json.load(open(tpath)).get("bytes_per_launch", {}).get(dom)
    roofline = {"kernel": dom, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": (achieved / HBM_PEAK_GBS) if achieved else None,
                "traffic": traffic, "avg_us": dom_s * 1e6, "algorithmic_bytes": alg_bytes}
    # whole-step view: 11 tensors of B*H*N*d bf16 must cross HBM per fwd+bwd
    step_bytes = 11 * d * elem * rows
    step_gbs = step_bytes / (ms_per_step * 1e-3) / 1e9

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        t0 = time.perf_counter()
        oracle.fwd_quadratic(host_inputs["Q"], host_inputs["K"], host_inputs["V"], host_inputs["s"])
        oracle.bwd_quadratic(host_inputs["Q"], host_inputs["K"], host_inputs["V"], host_inputs["s"],
                             host_inputs["dO"])
        dt = time.perf_counter() - t0
        cpu = {"value": B * N / dt, "unit": "tokens/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": "one full step of the same workload (B=8,H=12,N=1024,d=64): fp64 "
                         "quadratic-definition forward + brute-force backward, %.2f s" % dt}

    out = {
        "metric": "causal cosine-attn fwd+bwd tokens/s (B8 H12 N1024 d64 bf16)",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "B": B, "H": H, "N": N, "d": d,
                   "chunk": args.chunk or 64, "segments_fwd": G_f, "segments_bwd": G_b,
                   "buffer_sets": len(sets), "step": "cottn_fwd_causal + cottn_bwd_causal (given the forward's workspace)"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "step_hbm": {"algorithmic_bytes": step_bytes, "achieved_GBs": step_gbs,
                     "frac_of_peak": step_gbs / HBM_PEAK_GBS},
        "step_flops": flop_rates(rows, d, args.chunk or 64, ms_per_step * 1e-3),
        "kernels": kernels,
    }
    if not args.no_other_workloads and not args.chunk and not args.segments:
        del sets
        out["other_workloads"] = other_workloads(torch, cottn, workloads)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
