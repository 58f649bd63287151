"""GPU parity of the schedule generalisations (sections 3.5, 3.6): forward doubling with
activation recomputation, backward halving, 2f pipelines - whole worker against the oracle's
op-by-op replay."""
import numpy as np
import pytest

from oracle import block_oracle as bo
from oracle import schedule_oracle as so
from paper_2107_06925_amd import binding as b
from paper_2107_06925_amd import synth
from gpu_util import assert_close, compare_grads, dtype_name, make_stage, to_dev, to_np

pytestmark = pytest.mark.gpu


def _mb(tokens, hidden, g, dtype, seed=0):
    return synth.make_microbatch(tokens, hidden, g, seed=seed, dtype=dtype_name(dtype))


# name, D, N, f, layers, hidden, heads, seq, microbatch, dtype, causal
TINY = ("tiny-f32", 4, 4, 1, 2, 128, 4, 64, 2, b.F32, True)
SMALL_BF16 = ("small-bf16", 4, 4, 1, 2, 256, 4, 128, 2, b.BF16, False)     # several tiles, matrix-core kernels


def _oracle_lists(algo, D, N, f):
    return {b.DIRECT: lambda: so.chimera_schedule(D, N, f), b.DOUBLING: lambda: so.forward_doubling_schedule(D, N),
            b.HALVING: lambda: so.backward_halving_schedule(D, N)}[algo]()


def _run(case, algo, rank, N=None):
    import torch
    name, D, N0, f, L, H, heads, S, B, dtype, causal = case
    N = N or N0
    tokens = B * S
    gain = synth.qk_gain_for(H) if dtype == b.BF16 else 1.0
    ops = _oracle_lists(algo, D, N, f)[rank]
    need = b.stash_slots_needed_pipes(algo, D, N, f, rank)
    stage_of_pipe = {pipe: s for _, pipe, _, s in ops}
    stages, params = {}, {}
    for pipe, s in stage_of_pipe.items():
        st, p = make_stage(L, H, heads, S, B, dtype, s, causal=causal, stash_slots=max(need[pipe], 1), qk_gain=gain)
        stages[pipe], params[pipe] = st, p
    xs, dys, outs = {}, {}, {}
    pipe_of = {}
    for kind, pipe, g, s in ops:
        for gg in ((g, g + 1) if kind == so.F2 else (g,)):
            pipe_of[gg] = pipe
    doubled = {}
    if algo == b.DOUBLING:
        for pipe in (0, 1):
            doubled[pipe] = b.Stage(L, H, heads, S, 2 * B, dtype, causal=causal, keep=False, share_weights_of=stages[pipe])
    pair_io = {}
    for g in range(N):
        x, dy = _mb(tokens, H, g, dtype)
        xs[g], dys[g] = x, dy
    for kind, pipe, g, s in ops:
        if kind == so.F2:
            # the two micro-batches' inputs side by side; the single-micro-batch io aliases the halves
            x2 = to_dev(np.concatenate([xs[g], xs[g + 1]]), dtype)
            y2, _ = doubled[pipe].set_io(g, x2, x2)
            pair_io[g] = y2
            for j, gg in enumerate((g, g + 1)):
                outs[gg] = stages[pipe].set_io(gg, x2[j * tokens:(j + 1) * tokens], to_dev(dys[gg], dtype))
    for g in range(N):
        if g not in outs:
            outs[g] = stages[pipe_of[g]].set_io(g, to_dev(xs[g], dtype), to_dev(dys[g], dtype))
    b.chimera_worker_bind_pipes([stages.get(p) for p in range(2 * f)])
    if algo == b.DOUBLING:
        b.chimera_worker_bind_doubling(doubled[0], doubled[1])
    b.chimera_run_worker_pipes(algo, rank, D, N, f)
    torch.cuda.synchronize()
    ys, dxs, grads = bo.worker_replay(ops, params, xs, dys, B, S, heads, causal)
    for g in range(N):
        assert_close(to_np(outs[g][0]), ys[g], dtype, "y %d" % g)
        assert_close(to_np(outs[g][1]), dxs[g], dtype, "dx %d" % g)
    for g, y2 in pair_io.items():
        assert_close(to_np(y2), np.concatenate([ys[g], ys[g + 1]]), dtype, "doubled forward %d" % g)
    for pipe, st in stages.items():
        compare_grads(st.read_grads(), grads[pipe], L, H, dtype, "pipe %d" % pipe)
        assert b.lib().chimera_stage_in_flight(st.handle) == 0
    return stages, doubled


@pytest.mark.parametrize("rank", [0, 1, 3])
def test_forward_doubling_tiny_fp32(rank):
    print("doubling fp32 rank", rank, flush=True)
    _run(TINY, b.DOUBLING, rank, N=8)


def test_forward_doubling_odd_unit_count():
    print("doubling fp32 K=3", flush=True)
    _run(TINY, b.DOUBLING, 2, N=12)           # one doubled unit and one ordinary unit


def test_forward_doubling_bf16():
    print("doubling bf16", flush=True)
    _run(SMALL_BF16, b.DOUBLING, 0, N=8)


@pytest.mark.parametrize("rank", [0, 2])
def test_backward_halving_tiny_fp32(rank):
    print("halving fp32 rank", rank, flush=True)
    _run(TINY, b.HALVING, rank)


def test_backward_halving_bf16():
    print("halving bf16", flush=True)
    _run(SMALL_BF16, b.HALVING, 1, N=8)


@pytest.mark.parametrize("rank", [0, 3, 5])
def test_four_pipelines_tiny_fp32(rank):
    print("2f fp32 rank", rank, flush=True)
    _run(("tiny-2f", 8, 8, 2, 1, 128, 4, 64, 2, b.F32, True), b.DIRECT, rank)


def test_data_parallel_limit_bf16():
    # f = D/2: every worker holds every ... of the D stages it is given 2f = D of them; no bubbles
    print("2f bf16 f=D/2", flush=True)
    _run(("dp-limit", 4, 4, 2, 1, 256, 4, 128, 2, b.BF16, False), b.DIRECT, 1)


@pytest.mark.parametrize("N,rank", [(1, 0), (3, 1), (2, 3)])
def test_fewer_micro_batches_than_stages(N, rank):
    """Section 3.1: N < D; with N = 1 only the down stage exists on a worker."""
    print("N < D", N, rank, flush=True)
    _run(TINY, b.DIRECT, rank, N=N)


def test_half_backwards_equal_one_backward_bitwise_outputs():
    """dx of the two halves together is bit-identical to dx of the whole backward (same kernels,
    same rows); the gradients agree to rounding (two partial sums instead of one)."""
    import torch
    name, D, N, f, L, H, heads, S, B, dtype, causal = SMALL_BF16
    st, params = make_stage(L, H, heads, S, B, dtype, 0, causal=causal, qk_gain=synth.qk_gain_for(H))
    x, dy = _mb(B * S, H, 0, dtype)
    y, dx = st.set_io(0, to_dev(x, dtype), to_dev(dy, dtype))
    st.fwd(0); st.bwd(0)
    torch.cuda.synchronize()
    dx_whole, g_whole = dx.clone(), st.read_grads()
    st.zero_grads()
    st.fwd(0); st.bwd_half(0, 0); st.bwd_half(0, 1)
    torch.cuda.synchronize()
    assert torch.equal(dx, dx_whole)
    g_halves = st.read_grads()
    assert_close(g_halves, g_whole, b.F32, "gradients of two halves vs one backward")


def test_generalised_protocol_errors():
    name, D, N, f, L, H, heads, S, B, dtype, causal = TINY
    st, _ = make_stage(L, H, heads, S, B, dtype, 0)
    x, dy = _mb(B * S, H, 0, dtype)
    st.set_io(0, to_dev(x, dtype), to_dev(dy, dtype))
    with pytest.raises(b.ChimeraError) as e:
        st.bwd_half(0, 0)                       # no forward yet
    assert e.value.code == b.ESTATE
    st.fwd(0)
    with pytest.raises(b.ChimeraError) as e:
        st.bwd_half(0, 1)                       # second half first
    assert e.value.code == b.ESTATE
    st.bwd_half(0, 0)
    with pytest.raises(b.ChimeraError) as e:
        st.bwd(0)                               # whole backward in the middle of a halved one
    assert e.value.code == b.ESTATE
    st.bwd_half(0, 1)
    assert b.lib().chimera_stage_in_flight(st.handle) == 0
    # forward-only stage: no backward, one scratch slot, smaller stash
    fo = b.Stage(L, H, heads, S, 2 * B, dtype, keep=False, share_weights_of=st)
    assert fo.slot_bytes < 2 * st.slot_bytes * 2
    x2 = to_dev(np.concatenate([x, x]), dtype)
    fo.set_io(0, x2, x2)
    fo.fwd(0)
    fo.fwd(0)                                   # nothing stays in flight
    with pytest.raises(b.ChimeraError) as e:
        fo.bwd(0)
    assert e.value.code == b.ESTATE
    # doubling bind checks
    st_up, _ = make_stage(L, H, heads, S, B, dtype, 3)
    b.chimera_worker_bind(st, st_up)
    with pytest.raises(b.ChimeraError):
        b.chimera_worker_bind_doubling(fo, fo)          # second one is bound to other weights
    odd, _ = make_stage(1, H, heads, S, 3, dtype, 0)
    odd.set_io(0, to_dev(np.zeros((3 * S, H)), dtype), to_dev(np.zeros((3 * S, H)), dtype))
    odd.fwd(0)
    with pytest.raises(b.ChimeraError) as e:
        odd.bwd_half(0, 0)
    assert e.value.code == b.EINVAL
    odd.bwd(0)
