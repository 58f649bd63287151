"""Pins of the performance-model oracle (section 3.4, Eq. (1)); CPU only."""
import math

import pytest

from oracle import perf_model_oracle as pm
from oracle import schedule_oracle as so


def _rabenseifner_by_steps(alpha, beta, words, r):
    """Recursive halving (reduce-scatter) then recursive doubling (allgather): in step j of
    either phase every replica exchanges words / 2^j with one partner."""
    t, steps = 0.0, int(round(math.log2(r)))
    assert 2 ** steps == r
    for phase in range(2):
        for j in range(1, steps + 1):
            t += alpha + beta * words / 2 ** j
    return t


@pytest.mark.parametrize("r", [1, 2, 4, 8, 64])
def test_allreduce_closed_form_matches_step_count(r):
    a, b, L = 3.5e-6, 1.25e-10, 3.0e8
    assert pm.comm_allreduce(a, b, L, r) == pytest.approx(_rabenseifner_by_steps(a, b, L, r), rel=1e-12)


def test_allreduce_bandwidth_term_is_the_lower_bound():
    # 2 (r-1)/r L words leave and enter every replica in any allreduce; the model's bandwidth term is exactly that
    L, r = 1.0e6, 16
    assert pm.comm_allreduce(0.0, 1.0, L, r) == pytest.approx(2 * (r - 1) / r * L)
    assert pm.comm_allreduce(1.0, 0.0, L, r) == pytest.approx(2 * math.log2(r))


def test_backward_time_rule():
    assert pm.backward_time(1.5, False) == 3.0 and pm.backward_time(1.5, True) == 4.5


def test_paper_example_critical_path():
    # section 3.4: N = D = 6, C_f = 6 and C_b = 10; with free communication T is the computation alone
    lists = so.chimera_schedule(6, 6)
    r = pm.iteration_time(lists, 6, 1, 1.0, 2.0, 0.0, 0.0, 0.0, 0.0, replicas_per_group=2)
    assert (r["c_f"], r["c_b"]) == (6, 10)
    assert r["T"] == 26.0 and r["compute"] == 26.0 and r["p2p"] == 0.0 and max(r["unoverlapped"]) == 0.0


@pytest.mark.parametrize("D,N", [(4, 4), (8, 8), (8, 16), (16, 16)])
def test_free_communication_gives_the_makespan(D, N):
    lists = so.chimera_schedule(D, N)
    f_t, b_t = 1.25, 2.75
    r = pm.iteration_time(lists, D, 2, f_t, b_t, 0.0, 0.0, 10.0, 10.0, replicas_per_group=2)
    assert r["T"] == pytest.approx(so.simulate(lists, D, f_t, b_t)["makespan"], rel=1e-12)


def test_p2p_enters_once_per_critical_op():
    lists = so.chimera_schedule(8, 8)
    base = pm.iteration_time(lists, 8, 1, 1.0, 2.0, 0.0, 0.0, 0.0, 0.0, 2)
    withp = pm.iteration_time(lists, 8, 1, 1.0, 2.0, 0.125, 0.0, 0.0, 0.0, 2)
    # alpha only, no gradient traffic (r = 2 but zero words still costs latency): separate the terms
    assert withp["p2p"] == pytest.approx(0.125 * (withp["c_f"] + withp["c_b"]))
    assert withp["T"] - max(withp["unoverlapped"]) == pytest.approx(withp["compute"] + withp["p2p"])
    assert withp["T"] > base["T"]


def test_section_3_2_middle_workers_have_no_bubble_after_their_first_stage():
    # D = N = 4: the outer workers can start the allreduce of their first finished stage inside
    # bubbles, the middle workers cannot (section 3.2)
    lists = so.chimera_schedule(4, 4)
    for costs in ((1, 1), (1, 2)):
        sim = so.simulate(lists, 4, *costs)
        reg = pm.free_regions(lists, sim)
        for w in range(4):
            first_done = reg[w]["stages"][0][1]
            inside = pm._idle_between(reg[w]["idle"], first_done, reg[w]["end"])
            if w in (0, 3):
                assert inside > 0
                assert reg[w]["stages"][0][0] == 3          # the stage with the larger id finishes first
            else:
                assert inside == 0
                assert reg[w]["stages"][0][0] == 2


def test_unoverlapped_accounting():
    region = dict(stages=[(5, 10.0), (0, 20.0)], idle=[(2.0, 3.0), (12.0, 14.0), (16.0, 17.0), (20.0, 23.0)], end=20.0)
    # eager: first allreduce (cost 4) uses 3 idle units before the second stage is done, 1 is left;
    # then 1 + 4 against a tail of 3 leaves 2
    assert pm.unoverlapped(region, 23.0, 4.0, True) == pytest.approx(2.0)
    # not eager: 8 against the tail of 3
    assert pm.unoverlapped(region, 23.0, 4.0, False) == pytest.approx(5.0)
    # plenty of room
    assert pm.unoverlapped(region, 23.0, 1.0, True) == 0.0
    # idle time before a stage is complete never counts
    assert pm.unoverlapped(dict(stages=[(1, 9.0)], idle=[(0.0, 8.0)], end=9.0), 9.0, 2.0, True) == 2.0


def test_eager_launch_never_hurts_and_model_is_monotone():
    lists = so.chimera_schedule(8, 8)
    args = dict(D=8, W=4, f_t=1.0, b_t=2.0, act_words=1.0e6, grad_words=5.0e7, replicas_per_group=2)
    prev = None
    for beta in (0.0, 1e-9, 1e-8, 1e-7):
        e = pm.iteration_time(lists, alpha=1e-5, beta=beta, eager=True, **args)
        n = pm.iteration_time(lists, alpha=1e-5, beta=beta, eager=False, **args)
        assert e["T"] <= n["T"] + 1e-12
        if prev is not None:
            assert e["T"] >= prev
        prev = e["T"]
    # the slowest worker decides
    assert e["T"] == pytest.approx(e["compute"] + e["p2p"] + max(e["unoverlapped"]))


def test_chimera_beats_one_directional_schedules_in_the_model():
    # same stage time, same messages: fewer bubbles give the smaller T (the paper's selection logic)
    D = N = 8
    kw = dict(D=D, W=1, f_t=1.0, b_t=2.0, alpha=1e-3, beta=0.0, act_words=0.0, grad_words=0.0)
    chim = pm.iteration_time(so.chimera_schedule(D, N), replicas_per_group=2, **kw)["T"]
    dapple = pm.iteration_time(so.one_f_one_b_schedule(D, N), replicas_per_group=1, **kw)["T"]
    gpipe = pm.iteration_time(so.gpipe_schedule(D, N), replicas_per_group=1, **kw)["T"]
    assert chim < dapple <= gpipe


# ---------------------------------------------------------------- configuration selection (section 3.4)

def _cand(D, W, B, f_t=1.0, **kw):
    c = dict(D=D, W=W, B=B, f_t=f_t, b_t=None, recompute=False, act_words=0.0, grad_words=0.0,
             weight_bytes=10.0, act_bytes=1.0)
    c.update(kw)
    return c


@pytest.mark.parametrize("D", [4, 8, 16])
def test_worker_memory_matches_table_2(D):
    """Table 2: Chimera keeps 2 M_theta and between (D/2+1) M_a and D M_a; GPipe M_theta and N M_a;
    1F1B (DAPPLE) M_theta and between M_a and D M_a.  N = D micro-batches."""
    m_theta, m_a = 1000.0, 7.0
    lists, _, per_worker = pm.schedule_for("chimera", D, D)
    mem = pm.worker_memory(lists, D, per_worker, m_theta, m_a)
    assert min(mem) == 2 * m_theta + (D // 2 + 1) * m_a and max(mem) == 2 * m_theta + D * m_a
    lists, _, per_worker = pm.schedule_for("gpipe", D, D)
    assert set(pm.worker_memory(lists, D, per_worker, m_theta, m_a)) == {m_theta + D * m_a}
    lists, _, per_worker = pm.schedule_for("1f1b", D, D)
    mem = pm.worker_memory(lists, D, per_worker, m_theta, m_a)
    assert min(mem) == m_theta + m_a and max(mem) == m_theta + D * m_a


def test_selection_takes_the_largest_micro_batch_that_fits():
    """Greedy rule of section 3.4: per (W, D) the largest B that fits is taken even when a smaller
    one models faster; B = 8 does not fit here (2*10 + 4*8 = 52 > 40), B = 4 does (36)."""
    cands = [_cand(4, 2, 1, f_t=0.9, act_bytes=1.0), _cand(4, 2, 2, f_t=1.9, act_bytes=2.0),
             _cand(4, 2, 4, f_t=4.4, act_bytes=4.0), _cand(4, 2, 8, f_t=7.0, act_bytes=8.0)]
    evals, best = pm.select_configuration("chimera", 1, 64, 40.0, 0.0, 0.0, cands)
    assert [e["fits"] for e in evals] == [True, True, True, False]
    assert [e["chosen"] for e in evals] == [False, False, True, False]
    assert best == 2
    assert evals[0]["throughput"] > evals[2]["throughput"]          # the smaller B would have modelled faster
    assert evals[2]["mem_bytes"] == 2 * 10.0 + 4 * 4.0 and evals[2]["N"] == 8


def test_selection_closed_form_without_communication():
    """alpha = beta = 0, F_t proportional to B / D (a stage holds 1/D of the layers): with N = D the
    iteration takes F_t (C_f + 2 C_b) with C_f = D, C_b = 2D - 2 (section 3.4's example: 6 and 10),
    so time per sample is t0 (5D - 4) / (D^2 W) for P = W D workers: the deepest pipeline whose N
    still equals D wins here."""
    t0, P, minibatch = 1.0, 16, 64
    cands = []
    for D in (2, 4, 8):
        W = P // D
        B = minibatch // (W * D)                                   # N = D
        cands.append(_cand(D, W, B, f_t=t0 * B / D))
    evals, best = pm.select_configuration("chimera", 1, minibatch, 1e9, 0.0, 0.0, cands)
    for c, e in zip(cands, evals):
        D = c["D"]
        assert e["N"] == D and (e["c_f"], e["c_b"]) == (D, 2 * D - 2)
        assert e["T"] == pytest.approx(c["f_t"] * (D + 2 * (2 * D - 2)))
        assert e["throughput"] == pytest.approx(minibatch / e["T"])
    per_sample = [e["T"] / minibatch for e in evals]
    assert best == per_sample.index(min(per_sample))


def test_selection_skips_what_does_not_divide_or_fit():
    cands = [_cand(4, 3, 2), _cand(4, 2, 4, weight_bytes=1e6), _cand(4, 2, 2)]
    evals, best = pm.select_configuration("chimera", 1, 32, 100.0, 0.0, 0.0, cands)
    assert evals[0] is None                                          # 32 % (3*2) != 0
    assert evals[1]["fits"] is False
    assert best == 2
    evals, best = pm.select_configuration("chimera", 1, 32, 1.0, 0.0, 0.0, cands)
    assert best is None


def test_selection_evaluations_are_eq_1():
    c = _cand(4, 2, 2, f_t=3.0, b_t=5.3, act_words=1e6, grad_words=3e8)
    evals, _ = pm.select_configuration("chimera", 1, 32, 1e12, 5e-6, 1e-9, [c], eager=True)
    lists = so.chimera_schedule(4, 8)
    ref = pm.iteration_time(lists, 4, 2, 3.0, 5.3, 5e-6, 1e-9, 1e6, 3e8, 2, True)
    assert evals[0]["T"] == ref["T"] and evals[0]["N"] == 8
    # recomputation changes only the modelled backward time
    c2 = _cand(4, 2, 2, f_t=3.0, recompute=True)
    e2, _ = pm.select_configuration("1f1b", 1, 32, 1e12, 0.0, 0.0, [c2])
    assert e2[0]["T"] == pytest.approx(pm.iteration_time(so.one_f_one_b_schedule(4, 8), 4, 2, 3.0, 9.0, 0, 0, 0, 0, 1)["T"])
