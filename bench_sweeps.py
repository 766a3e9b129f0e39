#!/usr/bin/env python3
"""Head-only sweeps in the shape of the paper's kernel benchmarks (Sec. 4: batch sweep at S=512,
sequence-length sweep at B=128, vocabulary sweep at B=256, S=512; D=768, |V|=30522 unless swept),
on synthetic inputs generated on the device.  One JSON line per shape: forward and backward time,
valid-token TFLOP/s, peak device memory, and the size of the logit tensor that is never formed.
Sequences are full length (no padding), as in a head-only kernel benchmark.

This is a second workload beside bench.py (which prints the headline line); nothing here calls the
CPU oracle, parity is covered by the GPU tests.  A sampled column check against a plain fp32 torch
matmul guards against timing a broken launch.
"""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def run_shape(torch, lsr, B, S, D, V, steps, warmup, backward=True):
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(20260325 + B * 7 + S * 3 + V)
    torch.cuda.empty_cache()
    torch.cuda.reset_peak_memory_stats()
    H = torch.randn((B, S, D), device=dev, generator=g, dtype=torch.float32).to(torch.bfloat16)
    W = (torch.randn((V, D), device=dev, generator=g, dtype=torch.float32) * 0.02).to(torch.bfloat16)
    bias = torch.randn((V,), device=dev, generator=g, dtype=torch.float32) * 0.02
    mask = torch.ones((B, S), device=dev, dtype=torch.uint8)
    Y = torch.empty((B, V), device=dev, dtype=torch.float32)
    I = torch.empty((B, V), device=dev, dtype=torch.int32)
    dt = lsr.LSR_BF16
    ws_f = torch.empty(lsr.lsr_head_workspace_bytes(B, S, D, V, dt, False), dtype=torch.uint8, device=dev)
    shape = (B, S, D, V, dt)
    if backward:
        dY = torch.randn((B, V), device=dev, generator=g, dtype=torch.float32)
        dH = torch.empty((B, S, D), device=dev, dtype=torch.float32)
        dW = torch.empty((V, D), device=dev, dtype=torch.float32)
        db = torch.empty((V,), device=dev, dtype=torch.float32)
        ws_b = torch.empty(lsr.lsr_head_workspace_bytes(B, S, D, V, dt, True), dtype=torch.uint8, device=dev)

    def fwd():
        lsr.lsr_head_forward(*shape, H, W, bias, mask, Y, I, ws_f)

    def bwd():
        lsr.lsr_head_backward(*shape, H, W, dY, Y, I, dH, dW, db, ws_b)

    for _ in range(warmup):
        fwd()
        if backward:
            bwd()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    for k in range(steps):
        ev[k][0].record()
        fwd()
        ev[k][1].record()
        if backward:
            bwd()
        ev[k][2].record()
    torch.cuda.synchronize()
    f_ms = sorted(e[0].elapsed_time(e[1]) for e in ev)
    b_ms = sorted(e[1].elapsed_time(e[2]) for e in ev) if backward else [0.0]
    peak = torch.cuda.max_memory_allocated()

    # sanity: 64 sampled vocabulary columns against fp32 torch on the same bf16 values
    vs = torch.linspace(0, V - 1, 64, device=dev).long()
    ref = torch.log1p(torch.relu((H.float().reshape(B * S, D) @ W[vs].float().t() + bias[vs]).reshape(B, S, -1).max(dim=1).values))
    err = float((Y[:, vs] - ref).abs().max())
    if not err < 2e-2:
        raise RuntimeError(f"sampled forward check failed at B={B} S={S} D={D} V={V}: max abs {err}")

    flops = 2.0 * B * S * D * V
    f_med = f_ms[len(f_ms) // 2]
    b_med = b_ms[len(b_ms) // 2]
    return {"B": B, "S": S, "D": D, "V": V, "fwd_ms": f_med, "fwd_ms_min": f_ms[0], "bwd_ms": b_med,
            "fwd_tflops": flops / (f_med * 1e-3) / 1e12, "fwd_frac_mfma_peak": flops / (f_med * 1e-3) / 2.5e15,
            "peak_hbm_bytes": int(peak), "logits_avoided_bytes_bf16": int(2 * B * S * V),
            "sampled_max_abs_err": err}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--sweep", choices=("batch", "seq", "vocab", "all"), default="all")
    args = ap.parse_args()
    import torch
    import paper_2603_25011_amd as lsr
    if not torch.cuda.is_available():
        sys.exit("bench_sweeps.py: no GPU visible; the HIP path has no CPU fallback")
    lsr.load_library()
    D, V0 = 768, 30522
    shapes = []
    if args.sweep in ("batch", "all"):
        shapes += [("batch", b, 512, D, V0) for b in (8, 32, 128, 256)]
    if args.sweep in ("seq", "all"):
        shapes += [("seq", 128, s, D, V0) for s in (1024, 2048, 4096, 8192)]
    if args.sweep in ("vocab", "all"):
        shapes += [("vocab", 256, 512, D, v) for v in (30522, 65536, 131072, 250002)]
    for tag, B, S, Dd, V in shapes:
        r = run_shape(torch, lsr, B, S, Dd, V, args.steps, args.warmup)
        r["sweep"] = tag
        print(json.dumps(r), flush=True)


if __name__ == "__main__":
    main()
