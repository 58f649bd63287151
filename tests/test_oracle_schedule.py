"""Pins of the schedule oracle against what the Chimera paper fixes (CPU only)."""
import os

import pytest

from oracle import schedule_oracle as so

HERE = os.path.dirname(os.path.abspath(__file__))
EVEN_D = [2, 4, 6, 8, 10, 12, 16, 32, 64]


def _pins():
    out = []
    with open(os.path.join(HERE, "golden", "paper_schedule_pins.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                out.append((line[0],) + tuple(int(v) for v in line[1:]))
    return out


@pytest.mark.parametrize("pin", _pins(), ids=lambda p: "-".join(map(str, p)))
def test_paper_pins(pin):
    key, D, N, cf, cb, want = pin
    lists = so.chimera_schedule(D, N)
    r = so.simulate(lists, D, cf, cb)
    if key in ("bubbles_per_worker", "bubble_time"):
        assert r["bubbles"] == [want] * D
    elif key == "critical_cf":
        assert r["critical"][0] == want
    elif key == "critical_cb":
        assert r["critical"][1] == want
    elif key == "stash_min":
        assert min(r["stash_peak"]) == want
        # the paper: the minimum sits on the first and the last worker
        assert r["stash_peak"][0] == want and r["stash_peak"][-1] == want
    elif key == "stash_max":
        assert max(r["stash_peak"]) == want
    elif key.startswith("last_bwd_of_last_stage_P"):
        w = int(key[-1])
        last = [g for kind, pipe, g, s in lists[w] if kind == so.B and s == D - 1][-1]
        assert last == want
    else:
        raise AssertionError(key)


@pytest.mark.parametrize("D", EVEN_D)
@pytest.mark.parametrize("K", [1, 2, 4])
def test_chimera_structure_and_formulas(D, K):
    N = K * D
    lists = so.chimera_schedule(D, N)
    assert so.check_valid(lists, D, N, stages_per_worker=2)
    for w, ops in enumerate(lists):
        assert len(ops) == 2 * N
        # worker w holds stage w (down) and stage D-1-w (up): section 3.1
        assert {(pipe, s) for _, pipe, _, s in ops} == {(so.DOWN, w), (so.UP, D - 1 - w)}
        # N/2 micro-batches per pipeline
        assert sum(1 for k, p, _, _ in ops if k == so.F and p == so.DOWN) == N // 2
        assert sum(1 for k, p, _, _ in ops if k == so.F and p == so.UP) == N // 2
    r = so.simulate(lists, D, 1, 1)
    # Table 2: bubble ratio (D-2)/(2N+D-2) <=> D-2 idle slots in a makespan of 2N+D-2
    assert r["makespan"] == 2 * N + D - 2
    assert r["bubbles"] == [D - 2] * D
    # Table 2: activations in [(D/2+1) M_a, D M_a]
    assert min(r["stash_peak"]) == (D // 2 + 1 if D > 2 else 2)
    assert max(r["stash_peak"]) == D
    # ASAP replay never finishes later than the slot grid it came from
    grid = so.chimera_grid(D, N)
    assert max(max(row) for row in grid) + 1 == 2 * N + D - 2


@pytest.mark.parametrize("D", EVEN_D)
def test_chimera_b_equals_2f(D):
    """Section 2: with backward = 2 forward and N = D the ratio is (D-2)/(3N/2+D-2)."""
    N = D
    r = so.simulate(so.chimera_schedule(D, N), D, 1, 2)
    assert r["makespan"] == 3 * N + 2 * (D - 2)
    assert r["bubbles"] == [2 * (D - 2)] * D
    cf, cb = r["critical"]
    assert cf * 1 + cb * 2 == r["makespan"]


@pytest.mark.parametrize("D", EVEN_D)
def test_merge_is_conflict_free_and_slot_exact(D):
    """Section 3.1: at most one micro-batch per slot and worker for even D."""
    grid = so.chimera_grid(D, 2 * D)       # would raise on a conflict
    for w, row in enumerate(grid):
        assert len(row) == 4 * D
    # unit-cost ASAP replay starts every op no later than its grid slot
    lists = so.chimera_schedule(D, 2 * D)
    r = so.simulate(lists, D)
    for w, row in enumerate(grid):
        slots = sorted(row)
        for i, t in enumerate(slots):
            assert r["start"][w][i] <= t


def test_odd_depth_conflicts():
    """The same overlay with an odd D does put two ops into one cell."""
    table = so._pipeline_table(5, 2)
    cells = set()
    clash = False
    for pipe in (0, 1):
        for (kind, m, s), t in table.items():
            w = s if pipe == 0 else 4 - s
            clash |= (w, t) in cells
            cells.add((w, t))
    assert clash
    with pytest.raises(ValueError):
        so.chimera_schedule(5, 5)
    with pytest.raises(ValueError):
        so.chimera_schedule(4, 6)


def test_d4_worked_example():
    """D = N = 4 (figure 3 / section 3.2): down carries {0,1}, up carries {2,3}."""
    lists = so.chimera_schedule(4, 4)
    txt = [" ".join("FB"[k] + str(g) + "du"[p] for k, p, g, s in ops) for ops in lists]
    assert txt == [
        "F0d F1d F2u B2u F3u B3u B0d B1d",
        "F0d F2u F1d F3u B2u B0d B3u B1d",
        "F2u F0d F3u F1d B0d B2u B1d B3u",
        "F2u F3u F0d B0d F1d B1d B2u B3u",
    ]
    # mirror symmetry of the two pipelines: worker w and worker D-1-w swap roles
    for w in range(4):
        a = [(k, p, g % 2) for k, p, g, s in lists[w]]
        b = [(k, 1 - p, g % 2) for k, p, g, s in lists[3 - w]]
        assert a == b


@pytest.mark.parametrize("D,N", [(1, 3), (2, 2), (4, 4), (4, 16), (8, 8), (8, 32), (5, 7), (32, 32)])
def test_baselines(D, N):
    """Section 2: GPipe and DAPPLE (1F1B) both have 2(D-1) bubbles; Table 2 memory."""
    for make, peak in ((so.gpipe_schedule, [N] * D),
                       (so.one_f_one_b_schedule, [min(D - s, N) for s in range(D)])):
        lists = make(D, N)
        so.check_valid(lists, D, N, stages_per_worker=1)
        r = so.simulate(lists, D, 1, 1)
        assert r["bubbles"] == [2 * (D - 1)] * D
        assert r["makespan"] == 2 * (N + D - 1)        # ratio (D-1)/(N+D-1)
        assert r["stash_peak"] == peak
        r2 = so.simulate(lists, D, 1, 2)
        assert r2["makespan"] == 3 * (N + D - 1)


def test_chimera_halves_bubbles():
    for D in EVEN_D[1:]:
        c = so.simulate(so.chimera_schedule(D, D), D)["bubbles"][0]
        b = so.simulate(so.one_f_one_b_schedule(D, D), D)["bubbles"][0]
        assert c == D - 2 and b == 2 * (D - 1) and c < b / 2 + 1e-9 <= b


def test_simulator_detects_broken_order():
    """A planted mistake (backward listed before its forward) is caught."""
    lists = so.chimera_schedule(4, 4)
    bad = [list(ops) for ops in lists]
    bad[3][2], bad[3][3] = bad[3][3], bad[3][2]     # B0d before F0d on the last stage
    with pytest.raises(AssertionError):
        so.check_valid(bad, 4, 4, 2)


# ------------------------------------------------- generalisations (sections 3.5, 3.6)
def _gen_pins():
    out = []
    with open(os.path.join(HERE, "golden", "paper_generalisation_pins.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                out.append((line[0],) + tuple(int(v) for v in line[1:]))
    return out


def _idle_before_first_backward(lists, r, w):
    """Idle slots of worker w before its first backward chunk starts (unit slots)."""
    first_b = next(i for i, op in enumerate(lists[w]) if op[0] not in (so.F, so.F2))
    return r["start"][w][first_b] - first_b


@pytest.mark.parametrize("pin", _gen_pins(), ids=lambda p: "-".join(map(str, p)))
def test_paper_generalisation_pins(pin):
    key, D, N, f, want = pin
    if key.endswith("_2f"):
        lists = so.chimera_schedule(D, N, f)
        r = so.simulate(lists, D, 1, 1)
        if key == "bubbles_2f":
            assert r["bubbles"] == [want] * D
            # Table 3's ratio (D-2f)/(2fN+D-2f) is bubbles / makespan
            assert r["bubbles"][0] * (2 * f * N + D - 2 * f) == (D - 2 * f) * r["makespan"]
        elif key == "stash_min_2f":
            assert min(r["stash_peak"]) == want
        else:
            assert max(r["stash_peak"]) == want
    elif key.startswith("worker_down1_stage"):
        assert so.worker_of(D, f, 2, int(key[len("worker_down1_stage"):])) == want
    else:
        doubling = key.endswith("doubling")
        lists = so.forward_doubling_schedule(D, N) if doubling else so.backward_halving_schedule(D, N)
        r = so.simulate(lists, D, 1, 1, cost_f2=1, cost_bh=1)
        if key.startswith("bubbles_fwd_part"):
            for w in range(D):
                assert _idle_before_first_backward(lists, r, w) == want
                assert r["bubbles"][w] - want == D // 2 - 1
        else:
            assert r["bubbles"] == [want] * D


@pytest.mark.parametrize("D,f", [(4, 1), (4, 2), (8, 2), (8, 4), (12, 2), (12, 3), (12, 6), (16, 2), (16, 4), (32, 8)])
@pytest.mark.parametrize("K", [1, 2, 3])
def test_2f_structure(D, f, K):
    N = K * D
    lists = so.chimera_schedule(D, N, f)
    assert so.check_valid(lists, D, N, stages_per_worker=2 * f)
    n = D // (2 * f)
    for w, ops in enumerate(lists):
        assert len(ops) == 2 * N
        held = {(pipe, s) for _, pipe, _, s in ops}
        assert held == {(pipe, s) for pipe in range(2 * f) for s in range(D) if so.worker_of(D, f, pipe, s) == w}
        assert len(held) == 2 * f
        for pipe in range(2 * f):
            assert sum(1 for k, p, _, _ in ops if k == so.F and p == pipe) == K * n
    # every pipeline visits every worker exactly once, the up pipeline in the reverse order of its down pipeline
    for i in range(f):
        down = [so.worker_of(D, f, 2 * i, s) for s in range(D)]
        up = [so.worker_of(D, f, 2 * i + 1, s) for s in range(D)]
        assert sorted(down) == list(range(D)) and up == down[::-1]
        assert down[0] == i * (D // f)
    r = so.simulate(lists, D, 1, 1)
    assert r["makespan"] == 2 * N + D // f - 2
    assert r["bubbles"] == [D // f - 2] * D
    assert min(r["stash_peak"]) == D - D // (2 * f) + 1 and max(r["stash_peak"]) == D


def test_2f_rejects_bad_f():
    for D, f in [(8, 3), (8, 0), (12, 4), (6, 2)]:
        with pytest.raises(ValueError):
            so.chimera_schedule(D, D, f)


def test_f1_is_the_bidirectional_schedule():
    for D in (2, 4, 8):
        assert so.chimera_schedule(D, 2 * D, 1) == so.chimera_schedule(D, 2 * D)


@pytest.mark.parametrize("D", [2, 4, 6, 8, 16, 32])
@pytest.mark.parametrize("K", [2, 3, 4, 5])
def test_forward_doubling_structure(D, K):
    N = K * D
    lists = so.forward_doubling_schedule(D, N)
    # every micro-batch: forward exactly once per stage (alone or in a pair), backward exactly once per stage
    fwd, bwd = set(), set()
    for w, ops in enumerate(lists):
        assert {s for _, _, _, s in ops} == {w, D - 1 - w}
        for kind, pipe, g, s in ops:
            assert s == (w if pipe == so.DOWN else D - 1 - w)
            if kind == so.F2:
                assert g % 2 == 0
                for gg in (g, g + 1):
                    assert (gg, s) not in fwd
                    fwd.add((gg, s))
            elif kind == so.F:
                assert (g, s) not in fwd
                fwd.add((g, s))
            else:
                assert kind == so.B and (g, s) in fwd and (g, s) not in bwd
                bwd.add((g, s))
    want = {(g, s) for g in range(N) for s in range(D)}
    assert fwd == want and bwd == want
    r = so.simulate(lists, D, 1, 1, cost_f2=1)
    # whole doubled units (1 slot per doubled forward, 1 per backward): 3D busy slots per unit
    if K % 2 == 0:
        assert r["bubbles"] == [D - 2] * D
        assert r["makespan"] == 3 * N // 2 + D - 2
        # twice the activations of the basic schedule when nothing is recomputed (section 3.5)
        base = so.simulate(so.chimera_schedule(D, D), D)["stash_peak"]
        assert r["stash_peak"] == [2 * p for p in base]


@pytest.mark.parametrize("D", [2, 4, 6, 8, 16])
@pytest.mark.parametrize("K", [1, 2, 3])
def test_backward_halving_structure(D, K):
    N = K * D
    lists = so.backward_halving_schedule(D, N)
    base = so.chimera_schedule(D, N)
    for ops, bops in zip(lists, base):
        # same forwards in the same order; each backward replaced by its two halves, in order
        assert [op for op in ops if op[0] == so.F] == [op for op in bops if op[0] == so.F]
        halves = [(op[0], op[2], op[3]) for op in ops if op[0] != so.F]
        assert halves == [(h, g, s) for kind, _, g, s in bops if kind == so.B for h in (so.BH0, so.BH1)]
    r = so.simulate(lists, D, 1, 1, cost_bh=1)
    assert r["bubbles"] == [D - 2] * D
    # no more activations than the basic schedule (section 3.5)
    assert r["stash_peak"] == so.simulate(base, D)["stash_peak"]


def test_halving_with_true_costs_matches_direct():
    # a half backward costing half a backward: the replay is never slower than the direct schedule
    for D in (4, 8):
        direct = so.simulate(so.chimera_schedule(D, D), D, 2, 4)["makespan"]
        halved = so.simulate(so.backward_halving_schedule(D, D), D, 2, 4, cost_bh=2)["makespan"]
        assert halved <= direct


@pytest.mark.parametrize("D", [2, 4, 6, 8, 16])
def test_fewer_micro_batches_than_stages(D):
    """Section 3.1: N < D micro-batches are split as evenly as possible between the two
    pipelines; N = 1 is one micro-batch on a single pipeline."""
    for N in range(1, D):
        lists = so.chimera_schedule(D, N)
        n_down = sum(1 for k, p, _, _ in lists[0] if k == so.F and p == so.DOWN)
        n_up = sum(1 for k, p, _, _ in lists[0] if k == so.F and p == so.UP)
        assert n_down + n_up == N and 0 <= n_down - n_up <= 1
        assert so.check_valid(lists, D, N, stages_per_worker=1 if N == 1 else 2)
        for w, ops in enumerate(lists):
            assert len(ops) == 2 * N
            for kind, pipe, g, s in ops:
                assert s == (w if pipe == so.DOWN else D - 1 - w)
                assert (g < n_down) == (pipe == so.DOWN)
        r = so.simulate(lists, D, 1, 1)
        # one pipeline with n micro-batches under 1F1B ends at 2(D-1) + 2n; the longer one decides
        assert r["makespan"] == 2 * (D - 1) + 2 * n_down
        # it is the N = D schedule with the surplus micro-batches left out: same slots for the rest
        full = so.simulate(so.chimera_schedule(D, D), D, 1, 1)
        assert r["makespan"] <= full["makespan"]
    # a single micro-batch walks down and back: 2D slots, every worker idle for all but two of them
    r = so.simulate(so.chimera_schedule(D, 1), D, 1, 1)
    assert r["makespan"] == 2 * D and r["bubbles"] == [2 * D - 2] * D
    with pytest.raises(ValueError):
        so.chimera_schedule(D, D + 1)
