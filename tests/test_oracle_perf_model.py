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
