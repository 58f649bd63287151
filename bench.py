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
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 matrix throughput
HBM_PEAK_GBS = 8000.0

PROFILES = os.path.join(ROOT, "profiles")


def _roofline_traffic(workload):
    """HBM bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc summary of this
    workload (profiles/bench_<workload>_hbm_traffic.txt, line `roofline_traffic_bytes_per_launch = N`);
    None when no summary exists for it."""
    path = os.path.join(PROFILES, "bench_%s_hbm_traffic.txt" % workload.replace("-bf16", "").replace("-", "_"))
    try:
        with open(path) as f:
            for line in f:
                if "roofline_traffic_bytes_per_launch" in line and "=" in line:
                    return int(float(line.split("=")[1].split()[0]))
    except OSError:
        pass
    return None


def _cpu_baseline(cfg):
    """The oracle as it stands, timed on the host cores: one micro-batch forward + backward through a whole
    stage (all of its Transformer blocks) at full shape.  An iteration is N such stage passes, so
    sequences/s = N*B / (N * t_pass) = B / t_pass."""
    from threadpoolctl import threadpool_info
    from oracle import block_oracle as bo
    from paper_2107_06925_amd import synth
    params = synth.make_stage_params(cfg.hidden, cfg.layers, 0, seed=0, dtype=cfg.dtype)
    x, dy = synth.make_microbatch(cfg.tokens, cfg.hidden, 0, seed=0, dtype=cfg.dtype)
    t0 = time.perf_counter()
    bo.stage_pass(x, dy, params, cfg.microbatch, cfg.seq, cfg.heads, cfg.causal)
    dt = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    return {
        "value": cfg.microbatch / dt,
        "unit": "sequences/s",
        "cores": int(threads),
        "kind": "oracle",
        "sample": "1 of the iteration's %d micro-batches (%d sequences) forward+backward through one whole stage "
                  "(%d blocks) at full shape, fp64 numpy, %.1f s" % (cfg.N, cfg.microbatch, cfg.layers, dt),
    }


def _single_stream(args):
    """This benchmark again in a child process with --no-overlap: iteration time and per-kernel-class
    fractions when no two kernels share the chip."""
    import subprocess
    cmd = [sys.executable, os.path.abspath(__file__), "--no-overlap", "--no-cpu-baseline", "--config", args.config,
           "--rank", str(args.rank), "--steps", str(max(3, args.steps // 2)), "--warmup", "2", "--schedule", args.schedule,
           "--micro-batches", str(args.micro_batches), "--f", str(args.f)]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    if r.returncode:
        return {"error": (r.stderr or r.stdout)[-300:]}
    d = json.loads(r.stdout.strip().splitlines()[-1])
    return {"value": d["value"], "ms_per_step": d["ms_per_step"],
            "roofline_kernel_frac": d["roofline"]["frac"], "roofline_kernel_avg_launch_us": d["roofline"]["avg_launch_us"],
            "all_stage_gemms_frac_mfma_peak": d["all_stage_gemms"]["frac_mfma_peak"],
            "kernel_classes": {k: v.get("frac_mfma_peak", v.get("frac_hbm_peak")) for k, v in d["kernel_classes"].items()},
            "note": "bench.py --no-overlap: weight gradients on the stage's own stream, every kernel alone on the chip"}


def _time_edges(cfg, dtype, vocab):
    """The pipeline's two ends on one micro-batch of the workload (section 4.1): embedding
    forward + backward, and final LayerNorm + vocabulary projection + cross-entropy, forward
    and backward."""
    import torch
    from paper_2107_06925_amd import binding as b
    tdt = torch.float32 if dtype == b.F32 else torch.bfloat16
    M, H, S = cfg.tokens, cfg.hidden, cfg.seq
    gen = torch.Generator(device="cuda").manual_seed(0)
    tokens = torch.randint(0, vocab, (M,), device="cuda", dtype=torch.int32, generator=gen)
    wte = (0.02 * torch.randn((vocab, H), device="cuda", generator=gen)).to(tdt)
    wpe = (0.02 * torch.randn((S, H), device="cuda", generator=gen)).to(tdt)
    x = torch.empty((M, H), device="cuda", dtype=tdt)
    dx = torch.randn((M, H), device="cuda", generator=gen).to(tdt)
    dwte, dwpe = torch.zeros((vocab, H), device="cuda"), torch.zeros((S, H), device="cuda")
    y = torch.randn((M, H), device="cuda", generator=gen).to(tdt)
    g, be = torch.ones(H, device="cuda", dtype=tdt), torch.zeros(H, device="cuda", dtype=tdt)
    w = (0.02 * torch.randn((H, vocab), device="cuda", generator=gen)).to(tdt)
    dy, dg, db = torch.empty_like(y), torch.zeros(H, device="cuda"), torch.zeros(H, device="cuda")
    dw, loss = torch.zeros((H, vocab), device="cuda"), torch.zeros(1, device="cuda")
    ws = b.chimera_head_loss(y, tokens, g, be, w, 1.0 / M, dy, dg, db, dw, loss)

    def timed(f, n=5):
        f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            f()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n * 1e3

    emb = timed(lambda: (b.chimera_op_embedding_fwd(tokens, S, wte, wpe, x), b.chimera_op_embedding_bwd(tokens, S, dx, dwte, dwpe)))
    head = timed(lambda: b.chimera_head_loss(y, tokens, g, be, w, 1.0 / M, dy, dg, db, dw, loss, workspace=ws))
    flop = 6.0 * M * H * vocab
    loss.zero_()
    b.chimera_head_loss(y, tokens, g, be, w, 1.0 / M, dy, dg, db, dw, loss, workspace=ws)
    return {"vocab": vocab, "embedding_fwd_bwd_ms": emb, "head_loss_fwd_bwd_ms": head,
            "head_gemm_TFLOP/s": flop / (head * 1e-3) / 1e12, "loss_per_token_at_init": float(loss.item()),
            "ln_vocab": math.log(vocab)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="gpt2-1p3b-n32-bf16", help="workload (default: the largest single-GPU one, 76 TFLOP per iteration)")
    ap.add_argument("--rank", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--no-overlap", action="store_true", help="single stream per stage (analysis only)")
    ap.add_argument("--no-single-stream", action="store_true", help="skip the extra --no-overlap pass that gives context fractions")
    ap.add_argument("--schedule", choices=["direct", "doubling", "halving"], default="direct",
                    help="direct concatenation (the headline workload), forward doubling with recomputation, or backward halving")
    ap.add_argument("--micro-batches", type=int, default=0, help="N (default: the workload's; doubling needs >= 2D)")
    ap.add_argument("--f", type=int, default=1, help="2f pipelines per worker (direct schedule only)")
    ap.add_argument("--edges", action="store_true", help="also time the first stage's embedding and the last stage's head + loss")
    ap.add_argument("--vocab", type=int, default=50304)
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
    D, rank, f = cfg.D, args.rank, args.f
    algo = {"direct": b.DIRECT, "doubling": b.DOUBLING, "halving": b.HALVING}[args.schedule]
    N = args.micro_batches or (2 * cfg.N if algo == b.DOUBLING and cfg.N < 2 * D else cfg.N)
    ops = b.chimera_schedule_pipes(algo, D, N, f, rank)
    need = b.stash_slots_needed_pipes(algo, D, N, f, rank)
    stage_of_pipe = {o.pipe: o.stage for o in ops}
    tdt = torch.float32 if dtype == b.F32 else torch.bfloat16
    stages = {}
    for pipe, stage_id in sorted(stage_of_pipe.items()):
        st = b.Stage(cfg.layers, cfg.hidden, cfg.heads, cfg.seq, cfg.microbatch, dtype, causal=cfg.causal,
                     stash_slots=max(need[pipe], 1), overlap=not args.no_overlap)
        st.set_weights(synth.flatten_params(synth.make_stage_params(cfg.hidden, cfg.layers, stage_id, 0, cfg.dtype)))
        stages[pipe] = st
    doubled = {}
    if algo == b.DOUBLING:
        for pipe in (0, 1):
            doubled[pipe] = b.Stage(cfg.layers, cfg.hidden, cfg.heads, cfg.seq, 2 * cfg.microbatch, dtype, causal=cfg.causal,
                                    keep=False, share_weights_of=stages[pipe], overlap=not args.no_overlap)
    dev = lambda a: torch.from_numpy(a).cuda().to(tdt)
    done = set()
    for o in ops:
        if o.kind == b.OP_F2:               # the pair's inputs side by side; each micro-batch's io aliases its half
            pair = [synth.make_microbatch(cfg.tokens, cfg.hidden, o.mb + j, 0, cfg.dtype) for j in (0, 1)]
            x2 = dev(np.concatenate([pair[0][0], pair[1][0]]))
            doubled[o.pipe].set_io(o.mb, x2, x2)
            for j in (0, 1):
                stages[o.pipe].set_io(o.mb + j, x2[j * cfg.tokens:(j + 1) * cfg.tokens], dev(pair[j][1]))
                done.add(o.mb + j)
    for o in ops:
        if o.mb not in done:
            x, dy = synth.make_microbatch(cfg.tokens, cfg.hidden, o.mb, 0, cfg.dtype)
            stages[o.pipe].set_io(o.mb, dev(x), dev(dy))
            done.add(o.mb)
    b.chimera_worker_bind_pipes([stages.get(p) for p in range(2 * f)])
    if doubled:
        b.chimera_worker_bind_doubling(doubled[0], doubled[1])

    def step():
        for st in stages.values():
            st.zero_grads()
        b.chimera_run_worker_pipes(algo, rank, D, N, f)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    seq_per_s = N * cfg.microbatch * args.steps / elapsed

    out = {
        "metric": "sequences/sec per Chimera worker (1 MI355X) + % bf16 MFMA peak in stage GEMMs",
        "value": seq_per_s, "unit": "sequences/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "host_enqueue_ms_per_step": b.chimera_worker_last_enqueue_ms(), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "schedule": args.schedule, "pipelines_per_worker": 2 * f, "D": D, "N": N, "rank": rank,
                   "blocks_per_stage": cfg.layers, "hidden": cfg.hidden, "heads": cfg.heads, "seq": cfg.seq,
                   "microbatch": cfg.microbatch, "causal": cfg.causal,
                   "stash_slots": {("down" if p % 2 == 0 else "up") + (str(p // 2) if f > 1 else ""): need[p] for p in sorted(stages)},
                   "stash_bytes": int(sum(st.slot_bytes * st.stash_slots for st in stages.values())
                                      + sum(st.slot_bytes for st in doubled.values()))},
    }

    if not args.no_profile:
        # two more iterations, same launches: one with an event pair around every op (F_t, B_t), one
        # with an event pair around every kernel launch (the per-kernel events cost some 20 % of an
        # op's time, so the two are not taken together)
        b.chimera_worker_set_timing(True)
        step()
        torch.cuda.synchronize()
        b.chimera_worker_set_timing(False)
        tm = b.chimera_worker_last_timing()
        b.chimera_profile_reset()
        b.chimera_profile_enable(True)
        step()
        torch.cuda.synchronize()
        b.chimera_profile_enable(False)
        prof = b.chimera_profile_read()
        # dominant kernel by total time (rocprofv3 kernel trace): the weight-gradient GEMM instance
        wg = prof["gemm_wgrad"]
        achieved = wg["work"] / (wg["ms"] * 1e-3) / 1e12 if wg["ms"] else 0.0
        out["roofline"] = {
            "kernel": ("%s (the four weight gradients of a block, dW += X^T dY in fp32, and their bias gradients, per block "
                       "and micro-batch; the figures are those of the first instantiation named)"
                       % b.lib().chimera_op_gemm_group_last_kernel().decode()
                       if dtype == b.BF16 else "gemm_ref_kernel (weight-gradient GEMMs)"),
            "bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
            "traffic": _roofline_traffic(cfg.name) if (not args.no_overlap and algo == b.DIRECT and f == 1 and rank == 0) else None,
            "launches_per_step": wg["launches"], "avg_launch_us": wg["ms"] * 1e3 / max(wg["launches"], 1),
            "flop_per_launch": wg["work"] / max(wg["launches"], 1),
        }
        gemm_classes = ("gemm_fwd", "gemm_dgrad", "gemm_wgrad", "gemm_wgrad_tail")
        gemm_ms = sum(prof[k]["ms"] for k in gemm_classes)
        gemm_flop = sum(prof[k]["work"] for k in gemm_classes)
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
        for name, alg in (("chimera", b.DIRECT), ("1f1b", b.ONE_F_ONE_B), ("gpipe", b.GPIPE)):
            st = b.chimera_schedule_stats(alg, D, N, f_us, b_us)
            proj[name] = {"makespan_ms": st["makespan"] / 1e3,
                          "sequences_per_s_per_pipeline": N * cfg.microbatch / (st["makespan"] * 1e-6),
                          "bubble_frac": st["bubbles"][rank] / st["makespan"], "stash_peak": max(st["stash_peak"])}
        out["pipeline_projection"] = proj
        # Eq. (1) of the paper's performance model with the measured stage times and an assumed link:
        # one xGMI link per neighbour pair (153 GB/s, 5 us latency); words are bytes here
        if algo == b.DIRECT:
            esz = 4 if dtype == b.F32 else 2
            alpha, beta = 5e-6, 1.0 / 153e9
            act = float(cfg.microbatch * cfg.seq * cfg.hidden * esz)
            grad = float(stages[0].grads.numel() * 4)
            model = {}
            for name, alg, ff in (("chimera", b.DIRECT, f), ("1f1b", b.ONE_F_ONE_B, 1), ("gpipe", b.GPIPE, 1)):
                m = b.chimera_model_iteration_time(alg, D, N, ff, 1, out["stage_times"]["F_t_ms"] * 1e-3,
                                                   out["stage_times"]["B_t_ms"] * 1e-3, alpha, beta, act, grad)
                model[name] = {"T_ms": m["T"] * 1e3, "C_f": m["c_f"], "C_b": m["c_b"], "p2p_ms": m["p2p"] * 1e3,
                               "allreduce_ms": m["allreduce"] * 1e3, "unoverlapped_ms": m["unoverlapped"] * 1e3,
                               "sequences_per_s_per_pipeline": N * cfg.microbatch / m["T"]}
            out["model_eq1"] = {"assumed": {"alpha_s": alpha, "beta_s_per_byte": beta, "W": 1}, **model}
            # Section 3.4's selection of (W, D) for this model on P workers at this micro-batch size: stage
            # times, gradient and stash sizes scale with the blocks a stage holds (measured here for
            # cfg.layers of them); memory per stage replica = weights + fp32 gradients + fp32 Adam state.
            if f == 1 and args.schedule == "direct":
                P, minibatch, total_blocks = 32, 512, cfg.layers * D
                per_block = lambda v: v / cfg.layers
                wbytes = stages[0].weights.numel() * esz + stages[0].grads.numel() * 4 * 3
                cands = [dict(D=d, W=P // d, B=cfg.microbatch, f_t=per_block(out["stage_times"]["F_t_ms"] * 1e-3) * total_blocks / d,
                              b_t=per_block(out["stage_times"]["B_t_ms"] * 1e-3) * total_blocks / d, act_words=act,
                              grad_words=per_block(grad) * total_blocks / d, weight_bytes=per_block(wbytes) * total_blocks / d,
                              act_bytes=per_block(stages[0].slot_bytes) * total_blocks / d)
                         for d in (2, 4, 8, 16, 32) if total_blocks % d == 0 and minibatch % ((P // d) * cfg.microbatch) == 0]
                sel = {}
                for name, alg in (("chimera", b.DIRECT), ("1f1b", b.ONE_F_ONE_B), ("gpipe", b.GPIPE)):
                    ev, best = b.chimera_model_select(alg, 1, minibatch, 0.9 * 288e9, alpha, beta, cands)
                    sel[name] = {"best": None if best is None else {"W": cands[best]["W"], "D": cands[best]["D"]},
                                 "candidates": [{"W": c["W"], "D": c["D"], "N": e["N"], "fits": e["fits"], "T_ms": e["T"] * 1e3,
                                                 "sequences_per_s": e["throughput"], "mem_GB": e["mem_bytes"] / 1e9}
                                                for c, e in zip(cands, ev) if e is not None]}
                out["model_select"] = {"assumed": {"workers": P, "minibatch": minibatch, "micro_batch": cfg.microbatch,
                                                   "capacity_bytes": 0.9 * 288e9}, **sel}

    if dtype == b.BF16:
        # what this chip sustains: register-resident MFMA loop on every SIMD, and a streaming copy
        sink = torch.zeros(1, device="cuda")
        src = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        out["measured_ceiling"] = {"mfma_bf16_TFLOP/s": b.chimera_probe_mfma_bf16(sink),
                                   "stream_copy_GB/s": b.chimera_probe_copy(src, dst),
                                   "note": "register-resident 32x32x16 bf16 MFMA loop on all SIMDs; 256 MiB copy, read+write"}
        del src, dst
    if args.edges:
        out["edges"] = _time_edges(cfg, dtype, args.vocab)
    if not args.no_profile and not args.no_overlap and not args.no_single_stream:
        # The same workload with every kernel alone on the chip (one stream per stage): context for the
        # fractions above, whose durations include sharing the chip with the stage's second stream.
        out["single_stream"] = _single_stream(args)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = _cpu_baseline(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
