#!/usr/bin/env python3
"""Benchmark of the MI355X sparse-lexical LM head: one step = forward + backward of the whole
hot path over one synthetic batch, inputs resident in HBM.  Prints ONE JSON line.

value        = (valid-token forward flops + backward flops) / time, in TFLOP/s:
               2 * sum_b(len_b) * D * V  +  4 * nnz * D,  nnz = (b,v) pairs with a non-zero gate.
               Padded tokens are never counted.
roofline     = the fused forward kernel (dense contraction, bf16 MFMA) against the 2.5 PFLOP/s peak.
roofline_bwd = the backward (gathers, HBM-bound by its compulsory bytes) against 8 TB/s, with the
               cache-level gather traffic, a plain copy kernel and an L2-window gather measured beside it,
               and warm (same buffers every step) against rotated (three buffer sets) times.
cpu_baseline = the fp64 NumPy oracle, as it stands, on a bounded vocabulary sample of the same batch.
other_workloads, sweep_shapes, hybrid_alg2_reference, vendor_gemm_reference: context measured in the same run.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 matrix peak
HBM_PEAK_GBS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")


def measured_traffic(workload):
    """Bytes between L2 and the memory fabric per launch, from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs
    whose summary sits beside this file's source (profiles/traffic.json, written by
    paper_2603_25011_amd/profile_summary.py from the profiler's output).  None when no such run exists."""
    try:
        with open(TRAFFIC_FILE) as f:
            return json.load(f).get("workloads", {}).get(workload)
    except (OSError, ValueError):
        return None


def flops_forward(inp):
    w = inp.workload
    return 2.0 * inp.sum_len * w.D * w.V


def time_workload(name, steps, warmup, torch, wl, DeviceHead, rotate=False):
    w = wl.WORKLOADS[name]
    inp = wl.make_inputs(w)
    torch.cuda.reset_peak_memory_stats()
    head = DeviceHead(inp)
    do_bwd = head.has_backward

    def step():
        head.forward()
        if do_bwd:
            head.backward()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    t0 = time.perf_counter()
    for k in range(steps):
        ev[k][0].record()
        head.forward()
        ev[k][1].record()
        if do_bwd:
            head.backward()
        ev[k][2].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    peak_bytes = torch.cuda.max_memory_allocated()
    ms_step = (t1 - t0) * 1e3 / steps
    fwd_all = sorted(e[0].elapsed_time(e[1]) for e in ev)
    bwd_all = sorted(e[1].elapsed_time(e[2]) for e in ev) if do_bwd else [0.0]
    fwd_ms = sum(fwd_all) / steps
    bwd_ms = sum(bwd_all) / len(bwd_all)

    nnz = 0
    if do_bwd:
        nnz = int(((head.Y > 0) & (head.dY != 0)).sum().item())
    f_fwd = flops_forward(inp)
    f_bwd = 4.0 * nnz * w.D if do_bwd else 0.0
    res = {
        "workload": name, "B": w.B, "S": w.S, "D": w.D, "V": w.V, "sum_len": inp.sum_len, "nnz": nnz,
        "ms_per_step": ms_step, "fwd_ms": fwd_ms, "bwd_ms": bwd_ms,
        "fwd_ms_median": fwd_all[len(fwd_all) // 2], "fwd_ms_min": fwd_all[0],
        "bwd_ms_median": bwd_all[len(bwd_all) // 2], "bwd_ms_min": bwd_all[0],
        "tflops_step": (f_fwd + f_bwd) / (ms_step * 1e-3) / 1e12,
        "fwd_tflops_valid": f_fwd / (fwd_ms * 1e-3) / 1e12,
        "fwd_tflops_dense_equivalent": 2.0 * w.B * w.S * w.D * w.V / (fwd_ms * 1e-3) / 1e12,
        "fwd_frac_mfma_peak": f_fwd / (fwd_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "peak_hbm_bytes": int(peak_bytes),
        "logits_avoided_bytes_bf16": int(2 * w.B * w.S * w.V),
    }
    if do_bwd:
        esz = 2
        comp = (3 * w.B * w.V * 4 + w.B * w.S * w.D * esz + w.V * w.D * esz + w.V * w.D * 4 + w.B * w.S * w.D * 4 + w.V * 4)
        res["bwd_compulsory_bytes"] = int(comp)
        res["bwd_gbs_compulsory"] = comp / (bwd_ms * 1e-3) / 1e9
        res["bwd_gather_bytes_cache_level"] = int(2 * nnz * w.D * esz)      # nnz rows of H for dW + nnz rows of W for dH
        res["bwd_cache"] = "warm: the same buffers every step"
    # Per-kernel times from the event-bracketed entry points.  Each profiled call synchronises, and a
    # kernel that starts on an idle device runs at a lower clock for its first part (a profiled forward
    # from idle measured 7 % above the same kernel inside the timed loop), so every profiled call is
    # preceded by the ordinary, un-synchronised calls that keep the device busy.
    kf = [0.0] * 8
    kb = [0.0] * 8
    n = 3
    for _ in range(n):
        step()
        for i, x in enumerate(head.forward_profiled()):
            kf[i] += x / n
        if do_bwd:
            step()
            head.forward()
            for i, x in enumerate(head.backward_profiled()):
                kb[i] += x / n
    res["kernel_ms"] = {"fwd_pack": kf[0], "fwd_fused": kf[1], "fwd_merge": kf[2], "bwd_count": kb[0], "bwd_scan": kb[1],
                        "bwd_place": kb[2], "bwd_dH": kb[3], "bwd_dW_db": kb[4]}
    if rotate and do_bwd:
        # rotated buffers: three full sets (inputs, outputs, workspaces); a step never touches what the one before
        # it left in the caches
        heads = [head, DeviceHead(inp), DeviceHead(inp)]
        for h in heads:
            h.forward()
            h.backward()
        torch.cuda.synchronize()
        n_rot = max(6, steps // 2 * 2)
        evr = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n_rot)]
        for k in range(n_rot):
            h = heads[k % 3]
            evr[k][0].record()
            h.forward()
            evr[k][1].record()
            h.backward()
            evr[k][2].record()
        torch.cuda.synchronize()
        res["fwd_ms_rotated_buffers"] = sum(e[0].elapsed_time(e[1]) for e in evr) / n_rot
        res["bwd_ms_rotated_buffers"] = sum(e[1].elapsed_time(e[2]) for e in evr) / n_rot
        del heads[1:]
    if rotate:
        # The same step recorded once into a HIP graph and replayed: what a serving or training loop that
        # captures the head pays per step.  For the small configurations the gaps between the three to
        # twelve launches of a step are a visible share of it; at C5 they are not.
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    step()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            for _ in range(2):
                graph.replay()
            torch.cuda.synchronize()
            n_rep = max(6, steps)
            g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            g0.record()
            for _ in range(n_rep):
                graph.replay()
            g1.record()
            torch.cuda.synchronize()
            res["ms_per_step_graph_replay"] = g0.elapsed_time(g1) / n_rep
            del graph
        except Exception as exc:          # a failed capture must not cost the headline line
            res["ms_per_step_graph_replay"] = None
            res["graph_replay_error"] = repr(exc)
    return res, inp, head


def cpu_baseline(inp, n_rows, np):
    """The oracle on a vocabulary sample of the same batch (first, last and evenly spaced tiles)."""
    from oracle import lsr_head_oracle as orc
    w = inp.workload
    tile = 256
    n_tiles_all = (w.V + tile - 1) // tile
    n_tiles = max(2, min(n_tiles_all, n_rows // tile))
    tiles = np.unique(np.linspace(0, n_tiles_all - 1, n_tiles).round().astype(int))
    vs = np.concatenate([np.arange(t * tile, min(w.V, (t + 1) * tile)) for t in tiles])
    Wv, bv = inp.W[vs], inp.bias[vs]
    dYv = inp.dY[:, vs] if inp.dY is not None else None
    t0 = time.perf_counter()
    if dYv is not None:
        dH, dW, db, g, _ = orc.backward(inp.H, Wv, bv, inp.mask, dYv)     # forward + gate + routing
        nnz = int((g != 0).sum())
    else:
        orc.forward(inp.H, Wv, bv, inp.mask)
        nnz = 0
    dt = time.perf_counter() - t0
    fl = 2.0 * inp.sum_len * w.D * vs.size + 4.0 * nnz * w.D
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    return {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "seconds": dt,
            "sample": f"{vs.size} of {w.V} vocabulary rows ({tiles.size} tiles of 256 incl. first and last), "
                      f"all {w.B} sequences, forward+backward in fp64"}


def vendor_gemm_reference(torch, inp, n_cols=32768, iters=10):
    """Context, not part of the path: the vendor bf16 GEMM (torch.matmul -> hipBLASLt) on the packed
    valid-token matrix against one 32768-column slab of the vocabulary, logits written to memory."""
    w = inp.workload
    M, K, N = int(inp.sum_len), w.D, min(n_cols, w.V)
    a = torch.randn(M, K, device="cuda:0", dtype=torch.bfloat16)
    b = torch.randn(N, K, device="cuda:0", dtype=torch.bfloat16) * 0.02
    for _ in range(3):
        c = a @ b.t()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        c = a @ b.t()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    del a, b, c
    return {"M": M, "N": N, "K": K, "ms": ms, "tflops": 2.0 * M * N * K / (ms * 1e-3) / 1e12,
            "note": "library GEMM alone, bf16 logits written to HBM; no max/argmax/activation"}


def hybrid_reference(torch, np, inp, head, iters=3):
    """Context, not part of the path: the paper's hybrid forward (Sec. 3, Alg. 2) on the workload's own
    H, W, bias and mask: per vocabulary tile a library GEMM over the packed valid tokens writes the
    logits to memory, then a hand-written reduce kernel takes max and arg-max per sequence and applies the
    activation (paper_2603_25011_amd/alg2_comparator.py).  Timed for a few tile widths and for float32 and
    bfloat16 logits; every variant's Y and I are checked against the oracle on a vocabulary sample."""
    from oracle import lsr_head_oracle as orc
    from paper_2603_25011_amd.alg2_comparator import Alg2Forward
    w = inp.workload
    tile = 256
    n_tiles_all = (w.V + tile - 1) // tile
    tiles = np.unique(np.linspace(0, n_tiles_all - 1, 3).round().astype(int))
    vs = np.concatenate([np.arange(t * tile, min(w.V, (t + 1) * tile)) for t in tiles])
    Y_ref, I_ref, X_ref = orc.forward(inp.H, inp.W[vs], inp.bias[vs], inp.mask)
    out = []
    for dtype_name, dt in (("float32", torch.float32), ("bfloat16", torch.bfloat16)):
        for cols in (4096, 16384):
            try:
                alg = Alg2Forward(head.H, head.W, head.bias, head.mask, cols, dt)
                alg.forward()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(iters):
                    alg.forward()
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / iters
                Y = alg.Y[:, torch.as_tensor(vs, device=alg.Y.device)].cpu().numpy().astype(np.float64)
                I = alg.I[:, torch.as_tensor(vs, device=alg.I.device)].cpu().numpy().astype(np.int64)
                bi, vi = np.nonzero(I != I_ref)
                short = X_ref[bi, vi] - orc.logit_at(inp.H, inp.W[vs], inp.bias[vs], bi, I[bi, vi], vi) if bi.size else np.zeros(0)
                out.append({"logits": dtype_name, "tile_cols": cols, "ms": ms,
                            "tflops_valid": flops_forward(inp) / (ms * 1e-3) / 1e12,
                            "max_abs_err_Y_sample": float(np.abs(Y - Y_ref).max()),
                            "argmax_differs_sample": int(bi.size),
                            "argmax_outside_near_tie_rule_sample": int((short >= 1e-3).sum()),
                            "sample_pairs": int(I_ref.size)})
                del alg
                torch.cuda.empty_cache()
            except Exception as exc:          # a torch op missing on this build must not cost the headline line
                out.append({"logits": dtype_name, "tile_cols": cols, "error": repr(exc)})
    return {"variants": out,
            "note": "torch.mm (hipBLASLt) per vocabulary tile on the packed valid tokens + lsr_alg2_reduce (max, arg-max, "
                    "bias, ReLU, log1p); forward only; includes packing the tokens; sample = 3 vocabulary tiles x all sequences"}


def device_reference_rates(torch, lsr_binding):
    """A plain copy and the gather pattern of the backward at three window sizes, measured on this machine."""
    dev = "cuda:0"
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    copy = lsr_binding.lsr_copy_probe(dst, src, n, launches=4)
    del dst
    out = torch.empty(64 << 20, dtype=torch.uint8, device=dev)
    table = src.view(torch.int16)
    table.fill_(0x3C00)           # any finite bf16 pattern
    res = {"plain_copy_gbs_read_plus_write": copy, "plain_copy_bytes": n}
    for label, window, steps in (("gather_gbs_window_2MiB", 2 << 20, 2048), ("gather_gbs_window_32MiB", 32 << 20, 1024),
                                 ("gather_gbs_window_1GiB", 1 << 30, 256)):
        res[label] = lsr_binding.lsr_gather_probe(table, window, steps, out, launches=3)
    res["gather_note"] = ("lsr_gather_probe: 128-byte row pieces at random rows of the window, 8 lanes per piece, 4 in "
                          "flight per lane; 2 MiB stays in every L2, 32 MiB in the memory-side cache, 1 GiB goes to HBM")
    del src, out, table
    torch.cuda.empty_cache()
    return res


def sweep_shapes(torch, lsr_binding, steps, warmup):
    """Three shapes of the paper's head-only sweeps (Sec. 4: sequence-length sweep at B=128, vocabulary sweep
    at B=256 S=512, the small end of the batch sweep), full-length sequences, inputs generated on the device."""
    import bench_sweeps
    rows = []
    for B, S, D, V in ((128, 8192, 768, 30522), (256, 512, 768, 250002), (8, 512, 768, 30522)):
        r = bench_sweeps.run_shape(torch, lsr_binding, B, S, D, V, max(3, steps // 4), min(warmup, 2))
        rows.append(r)
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c5_large_fwdbwd")
    ap.add_argument("--no-extra", action="store_true", help="skip the other configurations, sweeps and comparators")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--cpu-rows", type=int, default=16384)
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run three 1 GiB plain copies (lsr_copy_probe): the known-size reference for rocprofv3 byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus must be 1 (no multi-GPU path exists)")

    import numpy as np
    import torch
    from paper_2603_25011_amd import binding as lsr_binding
    from paper_2603_25011_amd import inputs as wl
    from paper_2603_25011_amd.harness import DeviceHead

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")

    res, inp, head = time_workload(args.workload, args.steps, args.warmup, torch, wl, DeviceHead, rotate=not args.no_extra)
    w = inp.workload
    fwd_flops = flops_forward(inp)
    traffic = measured_traffic(args.workload) or {}
    roof = {"bound": "mfma", "kernel": "fwd_bf16_kernel (fused GEMM + max/argmax + activation)",
            "achieved": fwd_flops / (res["fwd_ms"] * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "traffic": traffic.get("fwd_bytes"), "traffic_unit": "bytes per launch",
            "traffic_source": traffic.get("source"),
            "algorithmic_bytes": int(w.B * w.S * w.D * 2 + w.V * w.D * 2 + w.B * w.V * 8 + w.V * 4),
            "flops_per_launch": fwd_flops, "avg_launch_ms": res["fwd_ms"],
            "fused_kernel_alone_ms": res["kernel_ms"]["fwd_fused"],
            "note": "flops count valid tokens only; avg_launch_ms is the whole forward call (packing, the fused kernel, "
                    "the join of cut sequences) from events on the launch stream over the timed steps"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    # second denominator: register-only MFMAs on this machine, at the clock it sustains under that load
    # (five launches of about 20 ms; the last one is timed)
    sink = torch.zeros(1, dtype=torch.float32, device="cuda:0")
    probe = lsr_binding.lsr_mfma_peak_probe(150000, 5, sink)
    roof["achievable_peak"] = probe
    roof["frac_of_achievable"] = roof["achieved"] / probe
    roof["achievable_note"] = ("lsr_mfma_peak_probe: bf16 32x32x16 MFMAs from registers only, two waves per SIMD; "
                               "context beside the nominal peak, which stays the denominator of frac")

    roof_bwd = None
    if w.backward:
        comp = res["bwd_compulsory_bytes"]
        roof_bwd = {"bound": "hbm", "kernels": "bucket sort (count, scan, place, chunk bounds) + dH gather + dW/db gather",
                    "achieved": comp / (res["bwd_ms"] * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "algorithmic_bytes": comp, "avg_backward_ms": res["bwd_ms"], "cache_state": "warm (same buffers every step)",
                    "avg_backward_ms_rotated_buffers": res.get("bwd_ms_rotated_buffers"),
                    "traffic": traffic.get("bwd_bytes"), "traffic_unit": "bytes per backward (FETCH_SIZE + WRITE_SIZE, scaled)",
                    "gather_bytes_cache_level": res["bwd_gather_bytes_cache_level"],
                    "gather_rate_cache_level_gbs": res["bwd_gather_bytes_cache_level"]
                    / ((res["kernel_ms"]["bwd_dH"] + res["kernel_ms"]["bwd_dW_db"]) * 1e-3) / 1e9,
                    "l2_counters": traffic.get("bwd_l2"),
                    "sq_counters": traffic.get("bwd_sq"),
                    # second bound of the gathers: one unpack and one FMA per gathered bf16 element, a wave-wide
                    # instruction holding its SIMD for 4 cycles (no packed fp32): lane-ops / (CUs x 64 lanes per clock x clock)
                    "gather_valu_floor_ms": 2.0 * res["nnz"] * w.D * 2.0 / (256 * 64 * 2.4e9) * 1e3,
                    "note": "achieved = compulsory bytes (every array once) / backward time; the gathers re-read rows of H and W "
                            "from the caches or LDS (gather_bytes_cache_level) and spend two VALU operations per gathered element "
                            "(gather_valu_floor_ms: both gathers at full VALU issue rate, 2.4 GHz), which is what bounds them"}
        roof_bwd["frac"] = roof_bwd["achieved"] / roof_bwd["peak"]
        if traffic.get("bwd_bytes"):
            roof_bwd["traffic_rate_gbs"] = traffic["bwd_bytes"] / (res["bwd_ms"] * 1e-3) / 1e9
    # the hybrid comparator needs the workload's device tensors
    hybrid = None
    if not args.no_extra:
        try:
            hybrid = hybrid_reference(torch, np, inp, head)
        except Exception as exc:
            hybrid = {"error": repr(exc)}
    del head
    torch.cuda.empty_cache()

    rates = None
    if not args.no_extra or args.calib_copy:
        rates = device_reference_rates(torch, lsr_binding)
        if roof_bwd is not None:
            roof_bwd["reference_rates"] = rates

    extra = {}
    sweeps = None
    if not args.no_extra:
        for name in ("c2_doc_fwd", "c3_query_fwdbwd", "c4_xlmr_fwdbwd"):
            if name == args.workload:
                continue
            r, _, h = time_workload(name, max(5, args.steps), args.warmup, torch, wl, DeviceHead, rotate=True)
            extra[name] = r
            del h
            torch.cuda.empty_cache()
        try:
            sweeps = sweep_shapes(torch, lsr_binding, args.steps, args.warmup)
        except Exception as exc:
            sweeps = {"error": repr(exc)}

    vendor = None if args.no_extra else vendor_gemm_reference(torch, inp)
    cpu = None if args.no_cpu else cpu_baseline(inp, args.cpu_rows, np)

    out = {
        "metric": "fused LM-head fwd+bwd TFLOP/s and % MFMA peak; peak HBM bytes, |V|=30k/250k",
        "value": res["tflops_step"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: B={w.B} S={w.S} D={w.D} V={w.V}, valid lengths {w.len_lo}..{w.len_hi}, "
                               + ("forward+backward" if w.backward else "forward only"),
                   "sum_len": inp.sum_len, "nnz": res["nnz"], "flops": "valid tokens only: 2*sum_len*D*V + 4*nnz*D",
                   "peak_hbm_bytes": res["peak_hbm_bytes"]},
        "roofline": roof,
        "roofline_bwd": roof_bwd,
        "cpu_baseline": cpu,
        "detail": res,
        "vendor_gemm_reference": vendor,
        "hybrid_alg2_reference": hybrid,
        "other_workloads": extra,
        "sweep_shapes": sweeps,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
