#!/usr/bin/env python3
"""Time and memory of the attention calls against sequence length and head dimension
(the sweep of Sec. 7 of the paper, this library's side only; no comparison system).

For each (mode, d, N): milliseconds of forward + backward (the backward is handed the forward's
workspace), tokens/s, bytes of the eight [B, H, N, d] bf16 tensors, workspace bytes of both calls.
Prints a markdown table.  Synthetic inputs (seeded torch generator on the device); B = 1.

    python bench_sweep.py [--heads 16] [--max-n 1048576] [--dims 32,64,128]
"""
import argparse
import sys

import torch


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--heads", type=int, default=16)
    ap.add_argument("--max-n", type=int, default=1 << 20)
    ap.add_argument("--dims", default="32,64,128")
    args = ap.parse_args()
    import paper_2409_18747_amd.binding as cottn
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    B, H = 1, args.heads
    print("| mode | d | N | fwd+bwd ms | tokens/s | tensors MB | workspace MB | segments |")
    print("|---|---|---|---|---|---|---|---|")
    for mode in ("causal", "bidirectional"):
        fwd = cottn.cottn_fwd_causal if mode == "causal" else cottn.cottn_fwd_bidir
        bwd = cottn.cottn_bwd_causal if mode == "causal" else cottn.cottn_bwd_bidir
        ops = (cottn.OP_FWD_CAUSAL, cottn.OP_BWD_CAUSAL) if mode == "causal" else \
              (cottn.OP_FWD_BIDIR, cottn.OP_BWD_BIDIR)
        for d in (int(x) for x in args.dims.split(",")):
            N = 256
            while N <= args.max_n:
                t = {n: (torch.randn(B, H, N, d, device=dev, generator=gen) * 0.5).to(torch.bfloat16)
                     for n in ("Q", "K", "V", "dO")}
                t.update({n: torch.empty_like(t["Q"]) for n in ("O", "dQ", "dK", "dV")})
                s = torch.ones(H, device=dev)
                ds = torch.empty(H, device=dev)
                fb = max(cottn.cottn_workspace_bytes(ops[0], B, H, N, d), 256)
                bb = max(cottn.cottn_workspace_bytes(ops[1], B, H, N, d), 256)
                fws = torch.empty(fb, dtype=torch.uint8, device=dev)
                bws = torch.empty(bb, dtype=torch.uint8, device=dev)

                def step():
                    fwd(t["Q"], t["K"], t["V"], s, O=t["O"], workspace=fws)
                    bwd(t["Q"], t["K"], t["V"], s, t["dO"], dQ=t["dQ"], dK=t["dK"], dV=t["dV"], ds=ds,
                        workspace=bws, fwd_workspace=fws)
                for _ in range(3):
                    step()
                torch.cuda.synchronize()
                iters = 50 if N <= 16384 else 10 if N <= 262144 else 4
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(iters):
                    step()
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / iters
                print("| %s | %d | %d | %.3f | %.3g | %.1f | %.2f | %d |" %
                      (mode, d, N, ms, B * N / (ms * 1e-3), 8 * B * H * N * d * 2 / 1e6, (fb + bb) / 1e6,
                       cottn.cottn_segments(ops[0], B, H, N, d)), flush=True)
                del t, fws, bws
                N *= 4
    return 0


if __name__ == "__main__":
    sys.exit(main())
