"""Parity at the workloads' full sizes, in the launch configuration bench.py times.

The oracle needs about 20 s per micro-batch and stage at these sizes, so the
whole-worker check uses a property that holds at any size: parameter gradients
are linear in the upstream gradients, so with dY = 0 for every micro-batch but
one per stage the accumulated gradients must equal the oracle's for that one
micro-batch, while Y of those micro-batches is unaffected by what the others do.
"""
import numpy as np
import pytest

from oracle import block_oracle as bo
from paper_2107_06925_amd import binding as b
from paper_2107_06925_amd import synth
from gpu_util import assert_close, compare_grads, make_stage, to_dev, to_np

pytestmark = pytest.mark.gpu

_ORACLE = {}


def _oracle_pass(cfg, params, stage_id, g, x, dy):
    """Oracle stage pass of one micro-batch, computed once per (stage, micro-batch) and session
    (the weights depend on the stage id only, the inputs on the micro-batch id only)."""
    key = (cfg.name, stage_id, g)
    if key not in _ORACLE:
        print("oracle: stage %d, micro-batch %d" % (stage_id, g), flush=True)
        _ORACLE[key] = bo.stage_pass(x, dy, params, cfg.microbatch, cfg.seq, cfg.heads, cfg.causal)
    return _ORACLE[key]


def _worker_case(name, rank, gain, tag):
    """One iteration of worker `rank` of the named workload through chimera_run_worker, with the stash
    slots the schedule assigns.  Per stage one micro-batch keeps its dY - one from the middle of the
    stage's backward order, so the overwriting first backward, accumulation after it and (for N > D)
    a later schedule unit all lie on the checked path - and is compared with the oracle: y, dx and
    every parameter gradient.  Micro-batches with dY = 0 must give dX = 0 exactly."""
    import torch
    cfg = synth.CONFIGS[name]
    D, N = cfg.D, cfg.N
    ops = b.chimera_schedule(b.DIRECT, D, N, rank)
    need = b.stash_slots_needed(b.DIRECT, D, N, rank)
    stage_ids = (rank, D - 1 - rank)
    stages, params = [], []
    for pipe, sid in enumerate(stage_ids):
        st, p = make_stage(cfg.layers, cfg.hidden, cfg.heads, cfg.seq, cfg.microbatch, b.BF16, sid, causal=cfg.causal,
                           stash_slots=need[pipe], qk_gain=gain)
        stages.append(st), params.append(p)
    pipe_of = {o.mb: o.pipe for o in ops}
    assert sorted(pipe_of) == list(range(N))
    sampled = {}
    for pipe in (0, 1):
        order = [o.mb for o in ops if o.kind == b.OP_B and o.pipe == pipe]
        assert len(order) == N // 2
        sampled[pipe] = order[len(order) // 2]          # neither the first nor the last backward of the stage
    xs, dys, outs = {}, {}, {}
    for g in range(N):
        keep = sampled[pipe_of[g]] == g
        x, dy = synth.make_microbatch(cfg.tokens, cfg.hidden, g, 0, "bf16")
        if keep:
            xs[g], dys[g] = x, dy
        outs[g] = stages[pipe_of[g]].set_io(g, to_dev(x, b.BF16), to_dev(dy if keep else np.zeros_like(dy), b.BF16))
    b.chimera_worker_bind(stages[0], stages[1])
    for st in stages:
        st.zero_grads()
    b.chimera_run_worker(rank, D, N)
    torch.cuda.synchronize()
    print("%s rank %d: stash slots %s, checked micro-batches %s" % (name, rank, need, sampled), flush=True)
    for pipe, g in sampled.items():
        key = (name, stage_ids[pipe], g, gain)
        if key not in _ORACLE:
            print("oracle: stage %d, micro-batch %d" % (stage_ids[pipe], g), flush=True)
            _ORACLE[key] = bo.stage_pass(xs[g], dys[g], params[pipe], cfg.microbatch, cfg.seq, cfg.heads, cfg.causal)
        y, dx, gr = _ORACLE[key]
        ey = assert_close(to_np(outs[g][0]), y, b.BF16, "y of micro-batch %d" % g)
        ex = assert_close(to_np(outs[g][1]), dx, b.BF16, "dx of micro-batch %d" % g)
        eg = compare_grads(stages[pipe].read_grads(), gr, cfg.layers, cfg.hidden, b.BF16, "stage of pipe %d" % pipe)
        print("%s %s pipe %d micro-batch %d: y %.3e, dx %.3e, worst parameter gradient %.3e" % (name, tag, pipe, g, ey, ex, eg),
              flush=True)
    for g in range(N):
        if sampled[pipe_of[g]] != g:
            assert float(outs[g][1].float().abs().max()) == 0.0, "dx of micro-batch %d (dY = 0)" % g
    for st in stages:
        st.close()


@pytest.mark.parametrize("gained", [False, True], ids=["plain", "peaked-softmax"])
def test_bert48_worker_full_size(gained):
    """BERT-48-like worker exactly as benchmarked: D=4, N=4, rank 0, 12 blocks per stage, hidden 1024,
    16 heads, seq 512, micro-batch 8, bidirectional, bf16 - once with the workload's own weights
    (almost uniform softmax) and once with the Q, K weights scaled so that the scores are peaked."""
    cfg = synth.CONFIGS["bert48-bf16"]
    assert b.stash_slots_needed(b.DIRECT, cfg.D, cfg.N, 0) == (2, 1)
    _worker_case("bert48-bf16", 0, synth.qk_gain_for(cfg.hidden) if gained else 1.0, "gained" if gained else "plain")


# (workload, rank): rank 0 has the smallest stash (D/2+1 slots over its two stages), the middle rank
# D/2-1 the largest (D slots, Table 2 of the paper); the middle rank runs with peaked attention scores.
_GPT2_CASES = [("gpt2-1p3b-bf16", 0), ("gpt2-1p3b-bf16", 3), ("gpt2-1p3b-n32-bf16", 0), ("gpt2-1p3b-n32-bf16", 3),
               ("gpt2-deep-bf16", 0), ("gpt2-deep-bf16", 15)]


@pytest.mark.parametrize("name,rank", _GPT2_CASES, ids=["%s-rank%d" % c for c in _GPT2_CASES])
def test_gpt2_worker_full_size(name, rank):
    """The three GPT-2-like workloads as benchmarked: D=8 N=8 (6 blocks per stage, hidden 1600, 25
    heads, seq 1024, micro-batch 4), D=8 N=32 (four concatenated schedule units, section 3.5 of the
    paper, micro-batch 2) and D=32 N=32 (2 blocks per stage, hidden 2048, head dim 128, seq 2048,
    micro-batch 1); causal, bf16; whole worker through chimera_run_worker."""
    cfg = synth.CONFIGS[name]
    need = b.stash_slots_needed(b.DIRECT, cfg.D, cfg.N, rank)
    middle = rank == cfg.D // 2 - 1
    assert sum(need) == (cfg.D if middle else cfg.D // 2 + 1)
    _worker_case(name, rank, synth.qk_gain_for(cfg.hidden) if middle else 1.0, "peaked" if middle else "plain")


@pytest.mark.parametrize("schedule", ["halving", "doubling"])
def test_bert48_worker_full_size_generalised(schedule):
    """The same worker under backward halving (N=4) and forward doubling with recomputation
    (N=8), as `bench.py --schedule ...` runs them: the doubled forward works on 8192 rows, the
    half backward on 2048.  Same dY = 0 device as above."""
    import torch
    cfg = synth.CONFIGS["bert48-bf16"]
    rank, D = 0, cfg.D
    algo, N = (b.HALVING, 4) if schedule == "halving" else (b.DOUBLING, 8)
    ops = b.chimera_schedule_pipes(algo, D, N, 1, rank)
    need = b.stash_slots_needed_pipes(algo, D, N, 1, rank)
    stages, params, doubled = {}, {}, {}
    for pipe, sid in ((0, rank), (1, D - 1 - rank)):
        stages[pipe], params[pipe] = make_stage(cfg.layers, cfg.hidden, cfg.heads, cfg.seq, cfg.microbatch, b.BF16, sid,
                                                causal=cfg.causal, stash_slots=max(need[pipe], 1))
        if algo == b.DOUBLING:
            doubled[pipe] = b.Stage(cfg.layers, cfg.hidden, cfg.heads, cfg.seq, 2 * cfg.microbatch, b.BF16, causal=cfg.causal,
                                    keep=False, share_weights_of=stages[pipe])
    pipe_of = {}
    for o in ops:
        for g in ((o.mb, o.mb + 1) if o.kind == b.OP_F2 else (o.mb,)):
            pipe_of[g] = o.pipe
    # one micro-batch per stage keeps its dY; for doubling one is the first, one the second of a pair
    sampled = {0: 0, 1: 3} if algo == b.HALVING else {0: 0, 1: max(g for g, p in pipe_of.items() if p == 1)}
    xs, dys, outs = {}, {}, {}
    for g in range(N):
        x, dy = synth.make_microbatch(cfg.tokens, cfg.hidden, g, 0, "bf16")
        xs[g], dys[g] = x, (dy if sampled[pipe_of[g]] == g else np.zeros_like(dy))
    for o in ops:
        if o.kind == b.OP_F2:
            x2 = to_dev(np.concatenate([xs[o.mb], xs[o.mb + 1]]), b.BF16)
            doubled[o.pipe].set_io(o.mb, x2, x2)
            for j in (0, 1):
                outs[o.mb + j] = stages[o.pipe].set_io(o.mb + j, x2[j * cfg.tokens:(j + 1) * cfg.tokens],
                                                       to_dev(dys[o.mb + j], b.BF16))
    for g in range(N):
        if g not in outs:
            outs[g] = stages[pipe_of[g]].set_io(g, to_dev(xs[g], b.BF16), to_dev(dys[g], b.BF16))
    b.chimera_worker_bind_pipes([stages[0], stages[1]])
    if doubled:
        b.chimera_worker_bind_doubling(doubled[0], doubled[1])
    b.chimera_run_worker_pipes(algo, rank, D, N, 1)
    torch.cuda.synchronize()
    for pipe, g in sampled.items():
        y, dx, gr = _oracle_pass(cfg, params[pipe], (rank, D - 1 - rank)[pipe], g, xs[g], dys[g])
        ey = assert_close(to_np(outs[g][0]), y, b.BF16, "y of micro-batch %d" % g)
        ex = assert_close(to_np(outs[g][1]), dx, b.BF16, "dx of micro-batch %d" % g)
        eg = compare_grads(stages[pipe].read_grads(), gr, cfg.layers, cfg.hidden, b.BF16, "stage of pipe %d" % pipe)
        print("%s micro-batch %d: y %.3e, dx %.3e, worst gradient %.3e" % (schedule, g, ey, ex, eg), flush=True)
        if algo == b.DOUBLING:
            # the doubled forward (8192 rows, other tile shapes) wrote the same y as the recomputing forward re-wrote
            pair = g - g % 2
            y2 = doubled[pipe].io[pair][1][(g - pair) * cfg.tokens:(g - pair + 1) * cfg.tokens]
            assert_close(to_np(y2), y, b.BF16, "doubled forward's y of micro-batch %d" % g)
    for st in list(stages.values()) + list(doubled.values()):
        st.close()


@pytest.mark.parametrize("name", ["gpt2-1p3b-bf16", "gpt2-1p3b-n32-bf16", "gpt2-deep-bf16"])
def test_gpt2_shapes_one_block(name):
    """One block at the full token count and width of the GPT-2-like workloads
    (hidden 1600 / 25 heads, and hidden 2048 / head_dim 128 / seq 2048), causal."""
    import torch
    cfg = synth.CONFIGS[name]
    st, params = make_stage(1, cfg.hidden, cfg.heads, cfg.seq, cfg.microbatch, b.BF16, 0, causal=True,
                            qk_gain=synth.qk_gain_for(cfg.hidden))
    x, dy = synth.make_microbatch(cfg.tokens, cfg.hidden, 0, 0, "bf16")
    y, dx = st.set_io(0, to_dev(x, b.BF16), to_dev(dy, b.BF16))
    st.fwd(0)
    st.bwd(0)
    torch.cuda.synchronize()
    y64, dx64, gr = bo.stage_pass(x, dy, params, cfg.microbatch, cfg.seq, cfg.heads, True)
    assert_close(to_np(y), y64, b.BF16, "y")
    assert_close(to_np(dx), dx64, b.BF16, "dx")
    compare_grads(st.read_grads(), gr, 1, cfg.hidden, b.BF16)
    st.close()
