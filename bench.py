#!/usr/bin/env python3
"""Benchmark of the encode stage on one MI355X.

One "step" is one epd_encode call over the whole synthetic batch of the
chosen workload (default: the InternViT-300M-shaped configuration, 8 requests
of 13 slices).  Inputs and packed weights are resident in HBM before the
timed region.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak
PEAK_FP32_TFLOPS = 157.3

TOL = {"bf16": 2e-2, "f32": 1e-4}   # max |gpu - oracle| / max |oracle| the parity sample must meet


def traffic_from_profile(workload: str):
    """L2 <-> fabric bytes per GEMM launch (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, the factors a plain 1 GiB
    copy kernel gives on the same counters), as the committed rocprofv3 --pmc summary of this command states
    it: the line `traffic_bytes_per_gemm_launch: <number>` of profiles/<workload>_bench_hbm_traffic.txt.
    Returns (bytes or None, source)."""
    rel = os.path.join("profiles", f"{workload}_bench_hbm_traffic.txt")
    try:
        for line in open(os.path.join(ROOT, rel)):
            if line.startswith("traffic_bytes_per_gemm_launch:"):
                return float(line.split(":", 1)[1].split()[0]), rel
    except OSError:
        pass
    return None, None


def roof_report(B, torch):
    """Measured ceilings of this machine, one JSON line: register-resident MFMA loop (random and constant
    operands), streaming copy, and the vendor BLAS (through torch.matmul) next to this library's plain
    bias-epilogue product on the four per-layer shapes of the C3 workload and a large cube, ten launches
    back to back each, random operands."""
    out = {"mfma_loop_tflops_random_operands": round(B.op_mfma_peak(True), 1),
           "mfma_loop_tflops_constant_operands": round(B.op_mfma_peak(False), 1),
           "copy_GBps_read_plus_write_1GiB": round(B.op_copy_peak(), 1), "gemm": []}
    # issue port of a SIMD: a wave of MFMAs and a wave of exp + fma pairs, each alone and both together (three rounds)
    co = []
    for _ in range(3):
        m, v, both = B.op_coissue(1), B.op_coissue(2), B.op_coissue(3)
        co.append({"mfma_wave_alone_ms": round(m, 3), "valu_wave_alone_ms": round(v, 3), "both_ms": round(both, 3),
                   "valu_plus_0.53_mfma_ms": round(v + 0.53 * m, 3)})
    out["mfma_valu_coissue"] = co
    g = torch.Generator(device="cuda").manual_seed(2)
    for name, (M, N, K) in (("qk", (106496, 2048, 1024)), ("out_proj", (106496, 1024, 1024)),
                            ("fc1", (106496, 4096, 1024)), ("fc2", (106496, 1024, 4096)), ("cube", (8192, 8192, 8192))):
        A = torch.randn((M, K), device="cuda", generator=g).to(torch.bfloat16)
        W = (torch.randn((N, K), device="cuda", generator=g) * 0.02).to(torch.bfloat16)
        bias = torch.zeros(N, dtype=torch.float32, device="cuda")
        C = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        torch.matmul(A, W.t(), out=C)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            torch.matmul(A, W.t(), out=C)
        e1.record()
        torch.cuda.synchronize()
        vendor_ms = e0.elapsed_time(e1) / 10
        _, lib_ms = B.op_gemm_bf16(A, W, bias, iters=10)
        fl = 2.0 * M * N * K
        out["gemm"].append({"shape": name, "M": M, "N": N, "K": K,
                            "vendor_blas_tflops": round(fl / vendor_ms / 1e9, 1),
                            "this_library_tflops": round(fl / lib_ms / 1e9, 1)})
        del A, W, C
    return out


def gemm_flops_per_tile(desc):
    """Dense-contraction flops of the GEMM kernel family per slice, by profile family."""
    N, D, F, L = desc.seq_len, desc.hidden, desc.mlp, desc.layers   # real tokens, the row padding is not counted
    No, Pi = desc.tokens_per_tile, desc.proj_in
    if desc.proj_kind == 2:   # resampler: kv projection, key / value in-projections, out-projection + last matrix
        E, Np = desc.proj_out, desc.n_patches
        proj = 2 * Np * D * E + 4 * Np * E * E + 4 * No * E * E
    elif desc.proj_kind == 0:
        proj = 2 * No * Pi * desc.proj_out
    else:
        proj = 2 * No * Pi * desc.proj_mid + 2 * No * desc.proj_mid * desc.proj_out
    return {
        "gemm_qkv": L * 2 * N * D * 3 * D,
        "gemm_out": L * 2 * N * D * D,
        "gemm_fc1": L * 2 * N * D * F,
        "gemm_fc2": L * 2 * N * D * F,
        "gemm_proj": proj,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5", "c6", "c7", "c8"])
    ap.add_argument("--micro-batch", type=int, default=0, help="slices per micro-batch (0: workload default)")
    ap.add_argument("--first-tiles", type=int, default=0,
                    help="encode only the first N slices of the first request: one worker's share under "
                         "intra-request parallelism (Section 3.2.2) as the timed step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-mm-cache", action="store_true", help="skip the paged-cache encode / block-transfer leg")
    ap.add_argument("--cpu-tiles", type=int, default=0, help="slices the oracle encodes (0: bounded default)")
    ap.add_argument("--batch-sweep", action="store_true",
                    help="also encode the batch in FCFS groups of 1, 2, 4, ... requests per call (maximum encode "
                         "batch size) and report per-call latency and throughput for each")
    ap.add_argument("--shard-sweep", action="store_true",
                    help="also encode the first 1, 2, 4, ... slices of the first request alone (what one encode "
                         "worker sees when a request's slices are cut over several workers) and report the "
                         "latency of each share next to that of the whole request")
    ap.add_argument("--no-shard-sweep", action="store_true",
                    help="skip the brief per-worker-share sweep a default run takes (profiling runs of the headline step)")
    ap.add_argument("--roof", action="store_true",
                    help="measure this box's ceilings instead of the workload (MFMA loop, streaming copy, vendor "
                         "BLAS and this library on the per-layer shapes) and print them as one JSON line")
    ap.add_argument("--mx-fp8", action="store_true",
                    help="the checkpoint-fidelity option epd_model_desc::mx_fp8: q/k/v, out-projection, FC1 and FC2 products on MXFP8 "
                         "operands (narrower than the headline precision: an extra line, never the headline)")
    ap.add_argument("--no-mx-option", action="store_true",
                    help="skip the extra timing of the same workload with the MXFP8 option on (reported as mx_fp8_option)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB elementwise copy kernel (scale for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (slices are independent, so more GPUs would each "
              "run this same kernel path on a share of the slices); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as wl
    from paper_2501_05460_amd import binding as B
    if not os.path.exists(B.LIB_PATH):
        from paper_2501_05460_amd.build import build
        build()

    if args.roof:
        print(json.dumps({"roof": roof_report(B, torch)}))
        return

    wk = wl.workload(args.workload)
    desc = wk.desc
    if args.micro_batch > 0:
        desc = desc.replace(max_tiles_per_call=args.micro_batch)
    if args.mx_fp8:
        desc = desc.replace(mx_fp8=1)
    bf16 = desc.dtype == wl.DT_BF16
    T = wk.n_tiles
    n_requests = wk.n_requests
    offsets = list(wk.tile_offsets)
    sample_tiles = list(wk.oracle_sample_tiles)
    if args.first_tiles > 0:
        T = min(args.first_tiles, offsets[1] - offsets[0])
        n_requests, offsets = 1, [0, T]
        sample_tiles = [t for t in sample_tiles if t < T] or [0]

    t0 = time.time()
    weights_dev = []
    last_note = time.time()

    def note(what):   # a line on stderr every ~20 s of host-side setup (the 6B shape draws 5.6 G weights on the host)
        nonlocal last_note
        if time.time() - last_note > 20.0:
            print(f"bench.py: setup, {what}", file=sys.stderr, flush=True)
            last_note = time.time()
    n_w = len(wl.weight_specs(desc))
    for i in range(n_w):
        weights_dev.append(B.to_device(wl.gen_weight(desc, wk.weight_seed, i), bf16))
        note(f"weight tensor {i + 1} of {n_w}")
    enc = B.Encoder(desc, weights_dev)
    del weights_dev
    S = desc.tile_size
    tiles = torch.empty((T, 3, S, S), dtype=torch.float32, device="cuda")
    for t in range(T):
        tiles[t] = torch.from_numpy(wl.gen_tile(desc, wk.input_seed, t))
        note(f"slice {t + 1} of {T}")
    out = enc.alloc_out(T)
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB read, 1 GiB written
        dst = torch.empty_like(src)
        torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        enc.encode(tiles, offsets, out)
    # every step also sits between two events on the call's stream (torch's current stream is the one the
    # binding hands to the library): their median is reported next to the wall-clock mean
    step_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for e0, e1 in step_ev:
        e0.record()
        enc.encode(tiles, offsets, out)
        e1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    ms_per_step = elapsed / args.steps * 1e3
    ms_median = float(np.median([e0.elapsed_time(e1) for e0, e1 in step_ev]))
    tiles_per_s = T * args.steps / elapsed
    tokens_per_s = tiles_per_s * desc.tokens_per_tile
    total_flops = wl.flops_per_tile(desc) * T
    tflops = total_flops / (elapsed / args.steps) / 1e12
    peak = PEAK_BF16_TFLOPS if bf16 else PEAK_FP32_TFLOPS

    # ---- per-kernel-family timing with HIP events on the call's stream ----
    enc.profile_enable(True)
    prof_steps = max(1, min(3, args.steps))
    fam = {}
    for _ in range(prof_steps):
        enc.encode(tiles, offsets, out)
        for k, v in enc.profile_read().items():
            f = fam.setdefault(k, {"ms": 0.0, "launches": 0})
            f["ms"] += v["ms"]
            f["launches"] += v["launches"]
    enc.profile_enable(False)
    gf = gemm_flops_per_tile(desc)
    gemm_ms = sum(fam[k]["ms"] for k in gf)
    gemm_launches = sum(fam[k]["launches"] for k in gf)
    gemm_flops = sum(gf.values()) * T * prof_steps
    achieved = gemm_flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    traffic, traffic_source = (traffic_from_profile(args.workload)
                               if desc.max_tiles_per_call == wk.desc.max_tiles_per_call and not args.mx_fp8 else (None, None))
    roofline = {
        "bound": "mfma", "kernel": ("k_gemm_mxfp8 (q/k/v, out-proj, FC1, FC2) + k_gemm_bf16 (the rest)" if args.mx_fp8 else "k_gemm_bf16 (all epilogue variants)") if bf16 else "k_f32_gemm",
        "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
        # what a register-resident MFMA loop reaches on this machine right now (random operands; no memory, no LDS)
        "achievable_peak": round(B.op_mfma_peak(True), 1) if bf16 else None,
        "traffic": traffic, "traffic_source": traffic_source,
        "flops_per_launch": gemm_flops / max(gemm_launches, 1),
        "avg_launch_ms": gemm_ms / max(gemm_launches, 1),
        "families_ms_per_step": {k: round(v["ms"] / prof_steps, 3) for k, v in fam.items()},
        "families_tflops": {k: round(gf[k] * T * prof_steps / (fam[k]["ms"] * 1e-3) / 1e12, 1)
                            for k in gf if fam[k]["ms"] > 0},
    }

    if args.mx_fp8:
        # the converted products against the dense FP8 peak of the matrix cores (5.0 PFLOP/s)
        fams = ("gemm_qkv", "gemm_out", "gemm_fc1", "gemm_fc2")   # out-proj: converted for the head dims of the named workloads
        mx_ms = sum(fam[k]["ms"] for k in fams)
        mx_tf = sum(gf[k] for k in fams) * T * prof_steps / (mx_ms * 1e-3) / 1e12 if mx_ms > 0 else 0.0
        roofline["mx_products"] = {"achieved": round(mx_tf, 1), "peak": 5000.0, "unit": "TFLOP/s", "frac": round(mx_tf / 5000.0, 4)}

    # ---- the kernels bound by memory bandwidth: algorithmic bytes / event-bracketed time ----
    hbm = None
    if bf16:
        M_rows = T * desc.seq_len
        Dq = desc.hidden                      # q and k rows as stored (head padding not counted)
        per_launch = {
            # fp32 row in, bf16 row out (MXFP8: one byte per element and one scale byte per 32)
            "norm": int(M_rows * desc.hidden * (4 + (1 + 1 / 32 if args.mx_fp8 else 2))),
            "qk_norm": M_rows * 2 * Dq * (2 + 2),                                    # q and k, read and written, bf16
            "proj_input": T * desc.tokens_per_tile * desc.proj_in * (4 + 2) if desc.proj_kind != 2 else None,
        }
        hbm = {"peak_GBps": 8000.0, "copy_GBps_measured": round(B.op_copy_peak(), 1)}
        # a call of more slices than max_tiles_per_call runs micro-batches: a launch covers one of them, so the
        # whole-batch byte counts above are spread over n_mb launches (mean bytes per launch)
        n_mb = -(-T // desc.max_tiles_per_call)
        for k, nbytes in per_launch.items():
            if nbytes and fam[k]["launches"] > 0 and fam[k]["ms"] > 0:
                gbps = nbytes / n_mb * fam[k]["launches"] / (fam[k]["ms"] * 1e-3) / 1e9
                hbm[k] = {"GBps": round(gbps, 1), "frac_of_peak": round(gbps / 8000.0, 3),
                          "bytes_per_launch": nbytes // n_mb, "launches_per_step": fam[k]["launches"] // prof_steps}

    # ---- maximum encode batch size: latency of one call against throughput ----
    sweep = None
    if args.batch_sweep:
        sweep = []
        n_out = desc.tokens_per_tile
        b = 1
        while True:
            groups = [(r, min(r + b, n_requests)) for r in range(0, n_requests, b)]
            lat = []
            for rep in range(2):                                  # first pass warms
                evs = [torch.cuda.Event(enable_timing=True) for _ in range(len(groups) + 1)]
                evs[0].record()
                for gi, (r0, r1) in enumerate(groups):
                    t_lo, t_hi = offsets[r0], offsets[r1]
                    enc.encode(tiles[t_lo:t_hi], [o - t_lo for o in offsets[r0:r1 + 1]], out[t_lo * n_out:t_hi * n_out])
                    evs[gi + 1].record()
                torch.cuda.synchronize()
                lat = [evs[i].elapsed_time(evs[i + 1]) for i in range(len(groups))]
            sweep.append({"max_batch_requests": b, "calls": len(groups), "mean_call_ms": round(sum(lat) / len(lat), 3),
                          "max_call_ms": round(max(lat), 3), "tiles_per_s": round(T / (sum(lat) * 1e-3), 1)})
            if b >= n_requests:
                break
            b *= 2

    # ---- intra-request parallelism: one worker's share of the first request ----
    shard = None
    # (always taken in brief — the shares of 2, 3, 4 and n workers — since a default run is what gets recorded;
    # --shard-sweep adds the other sizes)
    if args.shard_sweep or (not args.no_shard_sweep and not args.mx_fp8 and bf16 and args.first_tiles == 0 and offsets[1] - offsets[0] > 1 and T <= 256):
        n_req = offsets[1] - offsets[0]
        n_out = desc.tokens_per_tile
        sizes = sorted({-(-n_req // w) for w in (2, 3, 4)} | {1, n_req})
        if args.shard_sweep:
            sizes = sorted(set(sizes) | {n for n in (1, 2, 4, 8, 16, 32) if n < n_req})
        lat, wall = {}, {}
        for n in sizes:
            for _ in range(3):
                enc.encode(tiles[:n], [0, n], out[:n * n_out])
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 20
            ev0.record()
            for _ in range(reps):
                enc.encode(tiles[:n], [0, n], out[:n * n_out])
            ev1.record()
            torch.cuda.synchronize()
            lat[n] = ev0.elapsed_time(ev1) / reps
            # one call alone, as a worker sees it: host clock from the call to the end of the stream's work
            ws = []
            for _ in range(10):
                torch.cuda.synchronize()
                h0 = time.perf_counter()
                enc.encode(tiles[:n], [0, n], out[:n * n_out])
                torch.cuda.synchronize()
                ws.append((time.perf_counter() - h0) * 1e3)
            wall[n] = float(np.median(ws))
        shard = {"request_tiles": n_req,
                 "ms_by_tiles": {str(n): round(v, 3) for n, v in lat.items()},
                 # wall latency of a single call against its time on the GPU: what issuing ~200 launches from the host costs
                 "wall_ms_single_call_by_tiles": {str(n): round(v, 3) for n, v in wall.items()},
                 "wall_over_gpu": {str(n): round(wall[n] / lat[n], 3) for n in sizes},
                 # a request cut over w workers takes as long as its largest share
                 "speedup_by_workers": {str(w): round(lat[n_req] / lat[-(-n_req // w)], 2) for w in (2, 3, 4, n_req)}}
        enc.encode(tiles, offsets, out)    # the whole batch again: the parity sample below reads `out`
        torch.cuda.synchronize()

    # ---- paged cache: encode into blocks of 16 tokens, then move every block to a second cache ----
    mm = None
    if not args.no_mm_cache and desc.tokens_per_tile % 16 == 0:
        n_blocks = T * desc.tokens_per_tile // 16
        e_cache = B.MMCache(n_blocks, 16, desc.out_dim, bf16)
        p_cache = B.MMCache(n_blocks, 16, desc.out_dim, bf16)
        tables = [e_cache.alloc((offsets[r + 1] - offsets[r]) * desc.tokens_per_tile) for r in range(n_requests)]
        p_tables = [p_cache.alloc(len(t) * 16) for t in tables]
        flat_e = [b for t in tables for b in t]
        flat_p = [b for t in p_tables for b in t][::-1]          # scattered destination order
        B.encode_paged(enc, tiles, offsets, e_cache, tables)     # warm
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        n_paged = max(1, min(3, args.steps))
        for _ in range(n_paged):
            B.encode_paged(enc, tiles, offsets, e_cache, tables)
        torch.cuda.synchronize()
        paged_ms = (time.perf_counter() - t2) / n_paged * 1e3
        e_cache.transfer_to(flat_e, p_cache, flat_p)             # warm
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n_xfer = 10
        ev0.record()
        for _ in range(n_xfer):
            e_cache.transfer_to(flat_e, p_cache, flat_p)
        ev1.record()
        torch.cuda.synchronize()
        xfer_ms = ev0.elapsed_time(ev1) / n_xfer
        nbytes = n_blocks * 16 * desc.out_dim * (2 if bf16 else 4)
        mm = {"block_tokens": 16, "blocks": n_blocks, "paged_encode_ms_per_step": round(paged_ms, 3),
              "transfer_ms": round(xfer_ms, 4), "transfer_bytes": nbytes,
              "transfer_GBps_read_plus_write": round(2 * nbytes / (xfer_ms * 1e-3) / 1e9, 1)}
        if hbm is not None:
            hbm["block_copy"] = {"GBps": mm["transfer_GBps_read_plus_write"],
                                 "frac_of_peak": round(mm["transfer_GBps_read_plus_write"] / 8000.0, 3),
                                 "bytes_per_launch": 2 * nbytes, "note": "whole epd_mm_transfer call incl. the id upload"}
        e_cache.close()
        p_cache.close()
        # projection on the prefill side: cache and move pre-projection tokens, project after the move
        if desc.n_patches % 16 == 0:
            nb = T * desc.n_patches // 16
            e_pre = B.MMCache(nb, 16, desc.hidden, bf16)
            p_pre = B.MMCache(nb, 16, desc.hidden, bf16)
            src, dst = e_pre.alloc(nb * 16), p_pre.alloc(nb * 16)[::-1]
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            out2 = enc.alloc_out(T)
            for it in range(2):                                   # first pass warms
                evs[0].record()
                B.encode_trunk_paged(enc, tiles, 0, T, e_pre, src)
                evs[1].record()
                e_pre.transfer_to(src, p_pre, dst)
                evs[2].record()
                B.project_merge(enc, p_pre, dst, T, out2)
                evs[3].record()
                torch.cuda.synchronize()
            pre_bytes = nb * 16 * desc.hidden * (2 if bf16 else 4)
            mm["prefill_side_projection"] = {
                "trunk_ms": round(evs[0].elapsed_time(evs[1]), 3), "transfer_ms": round(evs[1].elapsed_time(evs[2]), 4),
                "project_merge_ms": round(evs[2].elapsed_time(evs[3]), 3),
                "transfer_bytes": pre_bytes, "bytes_vs_projected_tokens": round(pre_bytes / nbytes, 3)}
            e_pre.close()
            p_pre.close()
            del out2

    # ---- the same workload with the MXFP8 option on: an extra figure next to the headline, never the headline ----
    mx_opt = None
    if bf16 and not args.mx_fp8 and not args.no_mx_option and desc.hidden % 128 == 0 and desc.layers > 0:
        wdev = [B.to_device(wl.gen_weight(desc, wk.weight_seed, i), True) for i in range(len(wl.weight_specs(desc)))]
        enc_mx = B.Encoder(desc.replace(mx_fp8=1), wdev)
        del wdev
        out_mx = enc_mx.alloc_out(T)
        for _ in range(2):
            enc_mx.encode(tiles, offsets, out_mx)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(5)]
        for e0, e1 in evs:
            e0.record()
            enc_mx.encode(tiles, offsets, out_mx)
            e1.record()
        torch.cuda.synchronize()
        mx_ms = float(np.median([e0.elapsed_time(e1) for e0, e1 in evs]))
        mx_opt = {"ms_per_step": round(mx_ms, 3), "tiles_per_s": round(T / mx_ms * 1e3, 1),
                  "speedup_vs_bf16": round(ms_median / mx_ms, 3),
                  "dtype": "mxfp8 (q/k/v, out-proj, FC1, FC2 operands) + bf16",
                  "distance_from_bf16_output": round(float((out_mx.float() - out.float()).abs().max() / out.float().abs().max()), 4),
                  "note": "epd_model_desc::mx_fp8; parity of the option: tests/test_gpu_mx.py, tests/test_gpu_fullsize.py"}
        enc_mx.close()
        del out_mx

    # ---- parity spot check and CPU baseline: the oracle on a bounded sample ----
    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle import epd_oracle as O
        n_cpu = args.cpu_tiles or {"c1": 1, "c2": 2, "c3": 3, "c4": 1, "c5": 2, "c6": 2, "c7": 3, "c8": 2}[args.workload]
        sample = sample_tiles[:n_cpu]
        w_host = wl.gen_weights(desc, wk.weight_seed)
        host_tiles = [wl.gen_tile(desc, wk.input_seed, t) for t in sample]
        c0 = time.perf_counter()
        ref = O.encode_sample(host_tiles, w_host, desc)
        cpu_s = time.perf_counter() - c0
        n_out = desc.tokens_per_tile
        got = np.concatenate([out[t * n_out:(t + 1) * n_out].float().cpu().numpy() for t in sample])
        parity = float(np.abs(got - ref).max() / np.abs(ref).max())
        try:
            from threadpoolctl import threadpool_info
            threads = max([p["num_threads"] for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
        except Exception:
            threads = len(os.sched_getaffinity(0))
        cpu = {"value": round(len(sample) / cpu_s, 4), "unit": "tiles/s", "cores": threads,
               "kind": "oracle",
               "sample": f"slices {sample} of the same batch at full depth, {cpu_s:.1f} s, numpy fp64"}

    # the MXFP8 option against the oracle that converts at the same places: its own bound (two independent draws of
    # the format's noise once the computations have drifted apart), not the bf16 one
    tol_line = 1e-1 if args.mx_fp8 else TOL["bf16" if bf16 else "f32"]
    line = {
        "metric": "image_tiles_per_sec", "value": round(tiles_per_s, 2), "unit": "tiles/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("mxfp8 (q/k/v, out-proj, FC1, FC2 operands) + bf16" if args.mx_fp8 else "bf16") if bf16 else "f32", "data": "synthetic",
        "config": {"workload": wk.name + (f", first {T} slices of the first request" if args.first_tiles > 0 else ""),
                   "tiles": T, "requests": n_requests,
                   "tokens_per_tile": desc.tokens_per_tile, "out_dim": desc.out_dim,
                   "micro_batch_tiles": desc.max_tiles_per_call},
        "vision_tokens_per_sec": round(tokens_per_s, 1),
        "patch_tokens_per_sec": round(tiles_per_s * desc.n_patches, 1),
        "algorithmic_tflops": round(tflops, 2),
        "mfma_util_pct_of_peak": round(100.0 * tflops / peak, 2),
        "ms_per_step_median_events": round(ms_median, 3),
        "parity_max_rel_err_sample": parity,
        "parity_tolerance": tol_line,
        "parity_ok": None if parity is None else bool(parity < tol_line),
        "setup_s": round(setup_s, 1),
        "roofline": roofline,
        "hbm_kernels": hbm,
        "cpu_baseline": cpu,
        "mx_fp8_option": mx_opt,
        "mm_cache": mm,
        "batch_sweep": sweep,
        "shard_sweep": shard,
    }
    print(json.dumps(line))
    if line["parity_ok"] is False:
        print(f"bench.py: parity sample {parity:.3e} exceeds the tolerance {line['parity_tolerance']:.0e}: "
              "the throughput above is not a valid result", file=sys.stderr)
        sys.exit(3)


if __name__ == "__main__":
    main()
