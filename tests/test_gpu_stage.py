"""GPU parity of a stage and of a whole Chimera worker against the oracle."""
import numpy as np
import pytest

from oracle import block_oracle as bo
from oracle import schedule_oracle as so
from paper_2107_06925_amd import binding as b
from paper_2107_06925_amd import synth
from gpu_util import assert_close, compare_grads, dtype_name, make_stage, to_dev, to_np

pytestmark = pytest.mark.gpu


def _mb(tokens, hidden, g, dtype, seed=0):
    x, dy = synth.make_microbatch(tokens, hidden, g, seed=seed, dtype=dtype_name(dtype))
    return x, dy


STAGE_CASES = [
    # layers hidden heads seq mb dtype causal erf ref qk_gain
    (2, 128, 4, 64, 2, b.F32, True, False, False, 1.0),       # the tiny workload's stage
    (2, 128, 4, 64, 2, b.F32, False, True, False, 20.0),
    (1, 64, 2, 40, 3, b.F32, True, False, False, 20.0),       # ragged sizes
    (2, 128, 4, 64, 2, b.BF16, True, False, True, 1.0),       # bf16 on the plain kernels
    (2, 128, 2, 96, 2, b.BF16, True, False, False, synth.qk_gain_for(128)),     # bf16, matrix-core kernels, d = 64
    (2, 256, 2, 160, 1, b.BF16, False, False, False, synth.qk_gain_for(256)),   # d = 128, bidirectional
    (3, 320, 5, 200, 2, b.BF16, True, True, False, synth.qk_gain_for(320)),     # hidden not a multiple of 128, ragged seq
    (2, 64, 1, 1, 1, b.F32, True, False, False, 1.0),          # degenerate: one token, one head
    (2, 64, 1, 1, 1, b.BF16, True, False, False, 1.0),
    (1, 128, 2, 3, 5, b.BF16, False, False, False, synth.qk_gain_for(128)),     # 15 tokens: fewer rows than any tile
    (1, 128, 1, 129, 1, b.BF16, True, False, False, synth.qk_gain_for(128)),    # d = 128, one row past two attention tiles
]


@pytest.mark.parametrize("case", STAGE_CASES, ids=lambda c: "-".join(str(v)[:6] for v in c))
def test_stage_forward_backward(case):
    import torch
    layers, hidden, heads, seq, mb, dtype, causal, erf, ref, gain = case
    print("stage", case, flush=True)
    st, params = make_stage(layers, hidden, heads, seq, mb, dtype, stage_id=1, causal=causal, gelu_erf=erf,
                            reference_kernels=ref, qk_gain=gain)
    M = seq * mb
    total = None
    for g in range(2):
        x, dy = _mb(M, hidden, g, dtype)
        y, dx = st.set_io(g, to_dev(x, dtype), to_dev(dy, dtype))
        st.fwd(g)
        st.bwd(g)
        torch.cuda.synchronize()
        y64, dx64, gr = bo.stage_pass(x, dy, params, mb, seq, heads, causal, "erf" if erf else "tanh")
        total = bo.add_grads(total, gr)
        assert_close(to_np(y), y64, dtype, "y mb %d" % g)
        assert_close(to_np(dx), dx64, dtype, "dx mb %d" % g)
    compare_grads(st.read_grads(), total, layers, hidden, dtype, "accumulated over 2 micro-batches")
    st.zero_grads()
    assert np.all(st.read_grads() == 0)
    st.close()


def _run_worker(cfg, rank, dtype, layers=None, algo=b.DIRECT, reference_kernels=False, qk_gain=1.0):
    import torch
    D, N = cfg.D, cfg.N
    L = layers or cfg.layers
    need = b.stash_slots_needed(algo, D, N, rank)
    stages, params = [], []
    for pipe, stage_id in ((0, rank), (1, D - 1 - rank)):
        if need[pipe] == 0:
            stages.append(None), params.append(None)
            continue
        st, p = make_stage(L, cfg.hidden, cfg.heads, cfg.seq, cfg.microbatch, dtype, stage_id, causal=cfg.causal,
                           stash_slots=need[pipe], reference_kernels=reference_kernels, qk_gain=qk_gain)
        stages.append(st), params.append(p)
    xs, dys, outs = {}, {}, {}
    for g in range(N):
        pipe = 0 if (algo != b.DIRECT or (g % D) < D // 2) else 1
        x, dy = _mb(cfg.tokens, cfg.hidden, g, dtype)
        xs[g], dys[g] = x, dy
        outs[g] = stages[pipe].set_io(g, to_dev(x, dtype), to_dev(dy, dtype))
    b.chimera_worker_bind(stages[0], stages[1])
    b.chimera_run_worker_algo(algo, rank, D, N)
    torch.cuda.synchronize()
    return stages, params, xs, dys, outs


@pytest.mark.parametrize("rank", [0, 1, 3])
def test_worker_tiny_fp32(rank):
    """The tiny GPT-2-style workload, whole worker: D=4, N=4, 2 blocks per stage."""
    cfg = synth.CONFIGS["tiny-gpt2-f32"]
    stages, params, xs, dys, outs = _run_worker(cfg, rank, b.F32)
    ys, dxs, gd, gu = bo.worker_iteration(rank, cfg.D, cfg.N, params[0], params[1], xs, dys, cfg.microbatch, cfg.seq,
                                          cfg.heads, cfg.causal)
    for g in range(cfg.N):
        assert_close(to_np(outs[g][0]), ys[g], b.F32, "y %d" % g)
        assert_close(to_np(outs[g][1]), dxs[g], b.F32, "dx %d" % g)
    compare_grads(stages[0].read_grads(), gd, cfg.layers, cfg.hidden, b.F32, "down stage")
    compare_grads(stages[1].read_grads(), gu, cfg.layers, cfg.hidden, b.F32, "up stage")
    # the replay left nothing in flight
    assert b.lib().chimera_stage_in_flight(stages[0].handle) == 0
    assert b.lib().chimera_stage_in_flight(stages[1].handle) == 0


def test_worker_bf16_small_and_deterministic():
    """bf16 worker with concatenated units (N = 2D) on the matrix-core kernels;
    two replays give bit-identical gradients (no atomics anywhere)."""
    import torch
    cfg = synth.WorkerConfig("small-bf16", 4, 8, 2, 256, 4, 128, 2, True, "bf16")
    stages, params, xs, dys, outs = _run_worker(cfg, 1, b.BF16, qk_gain=synth.qk_gain_for(256))
    ys, dxs, gd, gu = bo.worker_iteration(1, cfg.D, cfg.N, params[0], params[1], xs, dys, cfg.microbatch, cfg.seq,
                                          cfg.heads, cfg.causal)
    for g in range(cfg.N):
        assert_close(to_np(outs[g][0]), ys[g], b.BF16, "y %d" % g)
        assert_close(to_np(outs[g][1]), dxs[g], b.BF16, "dx %d" % g)
    g0 = [st.read_grads() for st in stages]
    compare_grads(g0[0], gd, cfg.layers, cfg.hidden, b.BF16, "down stage")
    compare_grads(g0[1], gu, cfg.layers, cfg.hidden, b.BF16, "up stage")
    y_first = [outs[g][0].clone() for g in range(cfg.N)]
    for st in stages:
        st.zero_grads()
    b.chimera_run_worker(1, cfg.D, cfg.N)
    torch.cuda.synchronize()
    for st, ref in zip(stages, g0):
        assert np.array_equal(st.read_grads(), ref)
    for g in range(cfg.N):
        assert torch.equal(outs[g][0], y_first[g])
    # the host time of the replay up to its final wait is reported, and is below the whole call's
    import time
    for st in stages:
        st.zero_grads()
    t0 = time.perf_counter()
    b.chimera_run_worker(1, cfg.D, cfg.N)
    whole_ms = (time.perf_counter() - t0) * 1e3
    assert 0.0 < b.chimera_worker_last_enqueue_ms() <= whole_ms


@pytest.mark.parametrize("algo", [b.GPIPE, b.ONE_F_ONE_B])
def test_worker_baseline_schedules(algo):
    """GPipe and 1F1B replay give the same sums (one stage per worker)."""
    cfg = synth.CONFIGS["tiny-gpt2-f32"]
    stages, params, xs, dys, outs = _run_worker(cfg, 1, b.F32, algo=algo)
    total = None
    for g in range(cfg.N):
        y, dx, gr = bo.stage_pass(xs[g], dys[g], params[0], cfg.microbatch, cfg.seq, cfg.heads, cfg.causal)
        total = bo.add_grads(total, gr)
        assert_close(to_np(outs[g][0]), y, b.F32, "y %d" % g)
    compare_grads(stages[0].read_grads(), total, cfg.layers, cfg.hidden, b.F32)


def test_protocol_errors():
    st, _ = make_stage(1, 64, 2, 32, 1, b.F32, 0, stash_slots=1)
    L = b.lib()
    x, dy = _mb(32, 64, 0, b.F32)
    assert L.chimera_fwd(st.handle, 0) == b.ESTATE                 # io not set
    st.set_io(0, to_dev(x, b.F32), to_dev(dy, b.F32))
    st.set_io(1, to_dev(x, b.F32), to_dev(dy, b.F32))
    assert L.chimera_bwd(st.handle, 0) == b.ESTATE                 # backward before forward
    st.fwd(0)
    assert L.chimera_fwd(st.handle, 0) == b.ESTATE                 # forward twice
    assert L.chimera_fwd(st.handle, 1) == b.ESTATE                 # stash full
    assert L.chimera_fwd_slot(st.handle, 1, 5) == b.ENOMEM         # slot beyond the stash
    assert L.chimera_stage_set_option(st.handle, b.OPT_CAUSAL, 0) == b.ESTATE   # after bind
    st.bwd(0)
    assert L.chimera_bwd(st.handle, 0) == b.ESTATE
    st.fwd(1)
    st.bwd(1)
    # a worker whose stage has too few slots is refused before anything runs
    b.chimera_worker_bind(st, None)
    assert L.chimera_run_worker_algo(b.GPIPE, 0, 2, 2) == b.ENOMEM
    assert L.chimera_run_worker(0, 2, 2) == b.ESTATE               # Chimera needs an up stage
    st.close()


def test_deferred_zeroing_of_gradients():
    """chimera_stage_zero_grads defers the fill: the next backward overwrites (matrix-core path)
    or fills first (plain kernels); reading without a backward gives zeros; garbage left in the
    buffer never leaks into the gradients."""
    import torch
    for dtype, ref in ((b.BF16, False), (b.F32, False), (b.BF16, True)):
        L, H, heads, S, B = 2, 128, 2, 64, 2
        gain = synth.qk_gain_for(H) if dtype == b.BF16 else 1.0
        st, params = make_stage(L, H, heads, S, B, dtype, 0, reference_kernels=ref, qk_gain=gain)
        x, dy = _mb(B * S, H, 0, dtype)
        st.set_io(0, to_dev(x, dtype), to_dev(dy, dtype))
        st.grads.fill_(float("nan"))                  # whatever an earlier iteration left behind
        st.zero_grads()
        assert np.all(st.read_grads() == 0.0)         # a reader sees zeros
        st.grads.fill_(float("nan"))
        st.zero_grads()
        st.fwd(0); st.bwd(0)
        st.fwd(0); st.bwd(0)                          # second micro-batch accumulates onto the first
        torch.cuda.synchronize()
        _, _, gr = bo.stage_pass(x, dy, params, B, S, heads, True)
        twice = [{k: 2 * v for k, v in layer.items()} for layer in gr]
        compare_grads(st.read_grads(), twice, L, H, dtype, "dtype %d ref %s" % (dtype, ref))
        st.close()
