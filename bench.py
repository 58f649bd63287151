#!/usr/bin/env python3
"""Benchmark of one Chimera worker on one MI355X.

One step = one training iteration of the worker: zero both stages' gradient
buffers, then chimera_run_worker(rank, D, N) - N forwards and N backwards over
the worker's two stages in Chimera's schedule order, one stream wait at the end.
All inputs (weights, N activations, N upstream gradients) are resident in HBM
before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 matrix throughput
HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of the grouped weight-gradient kernel, from two rocprofv3 --pmc runs of
# this script (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch averaged over the kernel's
# launches), each scaled by what the same counter reads for a streaming kernel of known size
# (FETCH_SIZE x 2.00, WRITE_SIZE x 1.00): (209221.5 * 2.00 + 49188.1) KiB.
WGRAD_TRAFFIC_BYTES = {"bert48-bf16": int((209221.5 * 2.00 + 49188.1) * 1024)}


def _cpu_baseline(cfg, blocks=6):
    """The oracle as it stands, timed on the host cores: one micro-batch forward +
    backward through `blocks` of the stage's Transformer blocks at full shape."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import block_oracle as bo
    from paper_2107_06925_amd import synth
    params = synth.make_stage_params(cfg.hidden, blocks, 0, seed=0, dtype=cfg.dtype)
    x, dy = synth.make_microbatch(cfg.tokens, cfg.hidden, 0, seed=0, dtype=cfg.dtype)
    t0 = time.perf_counter()
    bo.stage_pass(x, dy, params, cfg.microbatch, cfg.seq, cfg.heads, cfg.causal)
    dt = time.perf_counter() - t0
    stage_pass_s = dt * cfg.layers / blocks            # a full stage has cfg.layers blocks
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    return {
        "value": cfg.microbatch / stage_pass_s,         # = N*B / (N stage passes)
        "unit": "sequences/s",
        "cores": int(threads),
        "kind": "oracle",
        "sample": "1 micro-batch (%d sequences) forward+backward through %d of the stage's %d blocks at full shape, "
                  "fp64 numpy, %.1f s; scaled to the whole stage" % (cfg.microbatch, blocks, cfg.layers, dt),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="bert48-bf16")
    ap.add_argument("--rank", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--no-overlap", action="store_true", help="single stream per stage (analysis only)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs one Chimera worker on ONE GPU; --gpus %d is not supported "
                 "(no collectives or sharding in this build)" % args.gpus)

    import numpy as np
    import torch
    from paper_2107_06925_amd import binding as b
    from paper_2107_06925_amd import synth

    cfg = synth.CONFIGS[args.config]
    dtype = b.F32 if cfg.dtype == "f32" else b.BF16
    D, N, rank = cfg.D, cfg.N, args.rank
    need = b.stash_slots_needed(b.DIRECT, D, N, rank)
    stages = []
    for pipe, stage_id in ((0, rank), (1, D - 1 - rank)):
        st = b.Stage(cfg.layers, cfg.hidden, cfg.heads, cfg.seq, cfg.microbatch, dtype, causal=cfg.causal,
                     stash_slots=need[pipe], overlap=not args.no_overlap)
        st.set_weights(synth.flatten_params(synth.make_stage_params(cfg.hidden, cfg.layers, stage_id, 0, cfg.dtype)))
        stages.append(st)
    tdt = torch.float32 if dtype == b.F32 else torch.bfloat16
    for g in range(N):
        x, dy = synth.make_microbatch(cfg.tokens, cfg.hidden, g, 0, cfg.dtype)
        pipe = 0 if (g % D) < D // 2 else 1
        stages[pipe].set_io(g, torch.from_numpy(x).cuda().to(tdt), torch.from_numpy(dy).cuda().to(tdt))
    b.chimera_worker_bind(stages[0], stages[1])

    def step():
        stages[0].zero_grads()
        stages[1].zero_grads()
        b.chimera_run_worker(rank, D, N)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    enqueue = time.perf_counter() - t0            # host time to issue every launch of the timed steps
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    seq_per_s = N * cfg.microbatch * args.steps / elapsed

    out = {
        "metric": "sequences/sec per Chimera worker (1 MI355X) + % bf16 MFMA peak in stage GEMMs",
        "value": seq_per_s, "unit": "sequences/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "host_enqueue_ms_per_step": enqueue * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "D": D, "N": N, "rank": rank, "blocks_per_stage": cfg.layers,
                   "hidden": cfg.hidden, "heads": cfg.heads, "seq": cfg.seq, "microbatch": cfg.microbatch,
                   "causal": cfg.causal, "stash_slots": {"down": need[0], "up": need[1]},
                   "stash_bytes": int(stages[0].slot_bytes * need[0] + stages[1].slot_bytes * need[1])},
    }

    if not args.no_profile:
        # one more iteration, same launches, with a HIP event pair around every kernel launch class
        b.chimera_profile_reset()
        b.chimera_profile_enable(True)
        b.chimera_worker_set_timing(True)
        step()
        torch.cuda.synchronize()
        b.chimera_profile_enable(False)
        b.chimera_worker_set_timing(False)
        prof = b.chimera_profile_read()
        tm = b.chimera_worker_last_timing()
        # dominant kernel by total time (rocprofv3 kernel trace): the weight-gradient GEMM instance
        wg = prof["gemm_wgrad"]
        achieved = wg["work"] / (wg["ms"] * 1e-3) / 1e12 if wg["ms"] else 0.0
        out["roofline"] = {
            "kernel": ("gemm_bf16_async_group_kernel<128,128,2,2,1,2,0,0> (the four weight gradients of a block, "
                       "dW += X^T dY in fp32, and their bias gradients, one launch per block and micro-batch)"
                       if dtype == b.BF16 else "gemm_ref_kernel (weight-gradient GEMMs)"),
            "bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
            "traffic": WGRAD_TRAFFIC_BYTES.get(cfg.name) if not args.no_overlap else None,
            "launches_per_step": wg["launches"], "avg_launch_us": wg["ms"] * 1e3 / max(wg["launches"], 1),
            "flop_per_launch": wg["work"] / max(wg["launches"], 1),
        }
        gemm_ms = sum(prof[k]["ms"] for k in ("gemm_fwd", "gemm_dgrad", "gemm_wgrad"))
        gemm_flop = sum(prof[k]["work"] for k in ("gemm_fwd", "gemm_dgrad", "gemm_wgrad"))
        all_tf = gemm_flop / (gemm_ms * 1e-3) / 1e12 if gemm_ms else 0.0
        out["all_stage_gemms"] = {"TFLOP/s": all_tf, "frac_mfma_peak": all_tf / MFMA_BF16_PEAK_TFLOPS,
                                  "flop_per_step": gemm_flop, "ms": gemm_ms}
        classes = {}
        for k, v in prof.items():
            if not v["launches"]:
                continue
            rate = v["work"] / (v["ms"] * 1e-3) if v["ms"] else 0.0
            if k.startswith(("gemm", "attn")):
                classes[k] = {"ms": v["ms"], "launches": v["launches"], "TFLOP/s": rate / 1e12,
                              "frac_mfma_peak": rate / 1e12 / MFMA_BF16_PEAK_TFLOPS}
            else:
                classes[k] = {"ms": v["ms"], "launches": v["launches"], "GB/s": rate / 1e9,
                              "frac_hbm_peak": rate / 1e9 / HBM_PEAK_GBS}
        out["kernel_classes"] = classes
        out["stage_times"] = {"F_t_ms": tm["fwd_ms"] / max(tm["n_fwd"], 1), "B_t_ms": tm["bwd_ms"] / max(tm["n_bwd"], 1),
                              "B_over_F": (tm["bwd_ms"] / max(tm["n_bwd"], 1)) / max(tm["fwd_ms"] / max(tm["n_fwd"], 1), 1e-9)}
        # what the measured F_t, B_t mean for a full D-worker pipeline (unit: iterations of N micro-batches)
        f_us = max(1, int(round(out["stage_times"]["F_t_ms"] * 1e3)))
        b_us = max(1, int(round(out["stage_times"]["B_t_ms"] * 1e3)))
        proj = {}
        for name, algo in (("chimera", b.DIRECT), ("1f1b", b.ONE_F_ONE_B), ("gpipe", b.GPIPE)):
            st = b.chimera_schedule_stats(algo, D, N, f_us, b_us)
            proj[name] = {"makespan_ms": st["makespan"] / 1e3,
                          "sequences_per_s_per_pipeline": N * cfg.microbatch / (st["makespan"] * 1e-6),
                          "bubble_frac": st["bubbles"][rank] / st["makespan"], "stash_peak": max(st["stash_peak"])}
        out["pipeline_projection"] = proj

    if dtype == b.BF16:
        # what this chip sustains: register-resident MFMA loop on every SIMD, and a streaming copy
        sink = torch.zeros(1, device="cuda")
        src = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        out["measured_ceiling"] = {"mfma_bf16_TFLOP/s": b.chimera_probe_mfma_bf16(sink),
                                   "stream_copy_GB/s": b.chimera_probe_copy(src, dst),
                                   "note": "register-resident 32x32x16 bf16 MFMA loop on all SIMDs; 256 MiB copy, read+write"}
        del src, dst
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = _cpu_baseline(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
