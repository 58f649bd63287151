"""Schedule oracle: Chimera's bidirectional pipeline schedule, plus GPipe and 1F1B.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
tests, the smoke check and the bench's cpu_baseline leg compare the product
against.  It shares no code with the HIP/C++ library and the product never
imports it.

What it follows (Chimera paper, Li & Hoefler, SC'21):

* Section 3.1 "Bidirectional Pipelines": D stages (D even), N micro-batches
  per worker and iteration.  The down pipeline maps stage s to worker s, the
  up pipeline maps stage s to worker D-1-s.  The micro-batches are split
  equally between the two pipelines, each pipeline runs them with the 1F1B
  strategy, and the two time tables are overlaid; with D even no slot of any
  worker receives two micro-batches.
* Section 3.1, last paragraph: with fewer micro-batches than stages the N
  micro-batches are divided between the two pipelines as evenly as possible
  (N = 1: one micro-batch on one pipeline).
* Section 3.5 "Scale to More Micro-Batches", direct concatenation: the table
  for D micro-batches is a basic unit; K = N/D units are chained so that the
  forwards of unit k+1 drop into the trailing bubbles of unit k.
* Section 2 "Bubbles in the pipeline" and Table 2: GPipe injects all N
  forwards and then runs all backwards; DAPPLE is 1F1B with a flush.
* Section 3.4: the critical path counts C_f, C_b.
* Section 3.5, forward doubling and backward halving: the order of the basic
  unit is kept, but every forward carries two micro-batches (doubling) or every
  backward is cut into two halves of a micro-batch (halving), so that one
  forward and one backward chunk cost about the same; a backward chunk only
  waits for the same chunk at the next stage.  The paper's figure for it is
  missing from the text; the reading here (basic-unit order, chunk-granular
  backward dependencies, as-soon-as-possible replay) reproduces the number the
  text does give: D-2 bubbles in all, D/2-1 among the forwards and D/2-1 among
  the backwards.
* Section 3.6 and Table 3, 2f pipelines: f down and f up pipelines, each with
  D/(2f) micro-batches per unit under 1F1B; down pipeline i puts stage 0 on
  worker i*(D/f) and the following stages on the following workers (cyclically);
  up pipeline i uses the reverse order of down pipeline i.

The paper has no listing for the merge; it describes it with a (missing)
figure.  The construction here fills an explicit worker x slot grid:

  1. One pipeline with n = D/2 micro-batches under 1F1B.  In 1F1B's steady
     state every stage alternates one forward and one backward, so one
     micro-batch enters every second slot: local micro-batch m starts its
     forward at stage 0 in slot 2m, moves one stage per slot, turns round at
     the last stage (its backward there takes the very next slot) and moves
     back one stage per slot.  `one_f_one_b_order` gives the textbook 1F1B
     order of every stage; `_pipeline_table` asserts that the table it fills
     has exactly that order on every stage.
  2. The up pipeline is the same table with worker = D-1-stage.
  3. Both are written into one grid; writing into an occupied cell raises.
  4. Unit k is written 2*D slots after unit k-1 (each worker is busy 2*D slots
     per unit, so this is the seamless chaining the paper describes for equal
     forward and backward cost).

A worker's op list is its grid row read left to right.  Only this ORDER is the
schedule the runtime consumes; start times under any cost model come from
`simulate`, which replays the orders as-soon-as-possible under the data
dependencies.

Micro-batch numbering (the paper fixes it only for D = N = 4, section 3.2:
worker 0 finishes the last stage's gradients with micro-batch 3, worker 3 with
micro-batch 1): inside unit k the down pipeline carries global ids
k*D + 0 .. k*D + D/2-1 and the up pipeline k*D + D/2 .. k*D + D-1.
Parity unpinned by the paper: the numbering across units (K > 1) and the
number of intermediate bubbles of direct concatenation when a backward costs
two forwards.
"""

F, B = 0, 1          # op kind: forward / backward of one micro-batch
F2 = 2               # forward of the two micro-batches g and g+1 together (forward doubling)
BH0, BH1 = 3, 4      # backward of the first / second half of micro-batch g (backward halving)
DOWN, UP = 0, 1      # pipeline; with 2f pipelines: pipe = 2*i (down pipeline i) or 2*i+1 (up pipeline i)


def one_f_one_b_order(D, n, s):
    """Textbook 1F1B order of stage s in a D-stage pipeline with n micro-batches.

    A stage keeps at most D-s micro-batches in flight: it runs forwards until
    that many are in flight (or none are left), then alternates one backward
    and one forward, and drains the remaining backwards at the end.
    Returns a list of (kind, local_micro_batch).
    """
    order = []
    warm = min(D - s, n)
    nf = nb = 0
    for _ in range(warm):
        order.append((F, nf))
        nf += 1
    while nb < n:
        order.append((B, nb))
        nb += 1
        if nf < n:
            order.append((F, nf))
            nf += 1
    return order


def _pipeline_table(D, n):
    """Slots of one pipeline: {(kind, m, s): slot} for n micro-batches, D stages."""
    slot = {}
    for m in range(n):
        t = 2 * m                      # one injection per forward+backward pair
        for s in range(D):             # forward sweep, one stage per slot
            slot[(F, m, s)] = t
            t += 1
        for s in range(D - 1, -1, -1):  # backward sweep starts right away
            slot[(B, m, s)] = t
            t += 1
    # the table must be a 1F1B schedule on every stage
    for s in range(D):
        ops = sorted((t, kind, m) for (kind, m, ss), t in slot.items() if ss == s)
        assert len({t for t, _, _ in ops}) == len(ops), "two ops in one slot"
        got = [(kind, m) for _, kind, m in ops]
        assert got == one_f_one_b_order(D, n, s), (D, n, s, got)
    return slot


def worker_of(D, f, pipe, s):
    """Worker that holds stage s of pipeline `pipe` (section 3.1; section 3.6 for f > 1)."""
    first = (pipe // 2) * (D // f)              # worker of stage 0 of the down pipeline
    if pipe % 2 == DOWN:
        return (first + s) % D
    return (first + D - 1 - s) % D              # the down pipeline's order, reversed


def chimera_grid(D, N, f=1):
    """Overlay of all pipelines and units: list over workers of {slot: op}.

    op = (kind, pipe, global_micro_batch, stage).  f down and f up pipelines;
    inside a unit the pipelines take consecutive blocks of D/(2f) micro-batch
    ids in the order down 0 .. down f-1, up 0 .. up f-1.
    """
    if D < 2 or D % 2:
        raise ValueError("Chimera needs an even number of stages")
    if N < D:
        return _partial_unit_grid(D, N, f)
    if N % D:
        raise ValueError("N must be a multiple of D, or smaller than D")
    if f < 1 or (D // 2) % f:
        raise ValueError("f must divide D/2")
    n = D // (2 * f)
    table = _pipeline_table(D, n)
    grid = [dict() for _ in range(D)]
    for k in range(N // D):
        for i in range(f):
            for direction in (DOWN, UP):
                pipe = 2 * i + direction
                block = i if direction == DOWN else f + i
                for (kind, m, s), t in table.items():
                    w = worker_of(D, f, pipe, s)
                    g = k * D + block * n + m
                    cell = 2 * D * k + t
                    if cell in grid[w]:
                        raise AssertionError("merge conflict on worker %d slot %d" % (w, cell))
                    grid[w][cell] = (kind, pipe, g, s)
    return grid


def _partial_unit_grid(D, N, f):
    """Fewer micro-batches than stages (section 3.1): the N micro-batches are split between
    the two pipelines as evenly as possible (the down pipeline takes the extra one; N = 1
    runs on the down pipeline alone), each pipeline runs its share under 1F1B, and the
    tables are overlaid as before.  Ids: down 0 .. n_down-1, up n_down .. N-1."""
    if N < 1:
        raise ValueError("N must be positive")
    if f != 1:
        raise ValueError("N < D is defined for the two-pipeline scheme")
    n_down = (N + 1) // 2
    grid = [dict() for _ in range(D)]
    for pipe, n, first in ((DOWN, n_down, 0), (UP, N - n_down, n_down)):
        if n == 0:
            continue
        for (kind, m, s), t in _pipeline_table(D, n).items():
            w = worker_of(D, 1, pipe, s)
            if t in grid[w]:
                raise AssertionError("merge conflict on worker %d slot %d" % (w, t))
            grid[w][t] = (kind, pipe, first + m, s)
    return grid


def chimera_schedule(D, N, f=1):
    """Per-worker op lists [(kind, pipe, mb, stage), ...] in execution order."""
    return [[row[t] for t in sorted(row)] for row in chimera_grid(D, N, f)]


def forward_doubling_schedule(D, N):
    """Section 3.5, forward doubling: units of 2D micro-batches.

    The order is that of the direct schedule for N/2 "double" micro-batches;
    the forward of double micro-batch j becomes one forward over micro-batches
    2j and 2j+1, its backward becomes the backward of 2j followed by that of
    2j+1 (each with recomputation when the runtime drops the activations).
    If N/D is odd the last D micro-batches form an ordinary basic unit.
    """
    if N < 2 * D or N % D:
        raise ValueError("forward doubling needs N = K*D with K >= 2")
    K = N // D
    lists = [[] for _ in range(D)]
    doubled = chimera_schedule(D, (K // 2) * D)
    for w, ops in enumerate(doubled):
        for kind, pipe, j, st in ops:
            if kind == F:
                lists[w].append((F2, pipe, 2 * j, st))
            else:
                lists[w] += [(B, pipe, 2 * j, st), (B, pipe, 2 * j + 1, st)]
    if K % 2:
        rest = chimera_schedule(D, D)
        for w, ops in enumerate(rest):
            lists[w] += [(kind, pipe, (K - 1) * D + g, st) for kind, pipe, g, st in ops]
    return lists


def backward_halving_schedule(D, N):
    """Section 3.5, backward halving: the same schedule as forward doubling, but
    a forward keeps one micro-batch and a backward is cut into two halves."""
    if N < D or N % D:
        raise ValueError("N must be a positive multiple of D")
    lists = []
    for ops in chimera_schedule(D, N):
        l = []
        for kind, pipe, g, st in ops:
            if kind == F:
                l.append((F, pipe, g, st))
            else:
                l += [(BH0, pipe, g, st), (BH1, pipe, g, st)]
        lists.append(l)
    return lists


def gpipe_schedule(D, N):
    """GPipe: every worker runs all N forwards, then all N backwards."""
    if D < 1 or N < 1:
        raise ValueError("bad D or N")
    return [[(F, DOWN, g, s) for g in range(N)] + [(B, DOWN, g, s) for g in range(N)]
            for s in range(D)]


def one_f_one_b_schedule(D, N):
    """1F1B with a flush per iteration (DAPPLE's schedule)."""
    if D < 1 or N < 1:
        raise ValueError("bad D or N")
    return [[(kind, DOWN, g, s) for kind, g in one_f_one_b_order(D, N, s)]
            for s in range(D)]


def simulate(lists, D, cost_f=1, cost_b=1, cost_f2=None, cost_bh=None):
    """ASAP replay of per-worker op lists under the pipeline's data dependencies.

    Dependencies of a micro-batch g: forward at stage s needs forward at s-1;
    backward at the last stage needs the forward there; backward at stage s
    needs backward at s+1.  A doubled forward (F2, micro-batches g and g+1)
    chains like a forward; the backward of g or g+1 at the last stage needs it.
    A half backward chains with the same half at the next stage.  A worker
    runs its list strictly in order, one op at a time.  cost_f2 (default
    cost_b) and cost_bh (default cost_f) price the doubled forward and the half
    backward.  Returns a dict with
      start[w][i], finish[w][i]   per op,
      makespan,
      bubbles[w]   = makespan - busy time of worker w,
      stash_peak[w] = max over time of the micro-batches whose activations the
                      worker holds (forward +1, doubled forward +2, backward
                      -1, half backward -1/2; no recomputation assumed),
      critical     = (C_f, C_b): forwards and backwards on the chain of ops
                     that fixes the makespan (section 3.4).
    """
    W = len(lists)
    cost = {F: cost_f, B: cost_b, F2: cost_b if cost_f2 is None else cost_f2,
            BH0: cost_f if cost_bh is None else cost_bh, BH1: cost_f if cost_bh is None else cost_bh}
    live_change = {F: 2, F2: 4, B: -2, BH0: -1, BH1: -1}      # in half micro-batches
    where = {}
    for w, ops in enumerate(lists):
        for i, (kind, pipe, g, s) in enumerate(ops):
            key = (kind, g, s)
            assert key not in where, "op listed twice: %r" % (key,)
            where[key] = (w, i)

    def dependency(kind, g, s):
        if kind in (F, F2):
            return (kind, g, s - 1) if s > 0 else None
        if s < D - 1:
            return (kind, g, s + 1)
        if (F, g, s) in where:
            return (F, g, s)
        return (F2, g - g % 2, s)                # the doubled forward that carried g

    start = [[None] * len(ops) for ops in lists]
    finish = [[None] * len(ops) for ops in lists]
    pred = {}
    nxt = [0] * W
    left = sum(len(ops) for ops in lists)
    while left:
        moved = False
        for w in range(W):
            while nxt[w] < len(lists[w]):
                i = nxt[w]
                kind, pipe, g, s = lists[w][i]
                t_worker = finish[w][i - 1] if i else 0
                dep = dependency(kind, g, s)
                if dep is None:
                    t_dep = 0
                else:
                    if dep not in where:
                        raise AssertionError("missing op %r" % (dep,))
                    dw, di = where[dep]
                    if finish[dw][di] is None:
                        break
                    t_dep = finish[dw][di]
                t0 = max(t_worker, t_dep)
                start[w][i] = t0
                finish[w][i] = t0 + cost[kind]
                # the op that this one actually waited for (data dependency
                # first when both end at the same time)
                if dep is not None and t_dep == t0:
                    pred[(w, i)] = where[dep]
                elif i and t_worker == t0:
                    pred[(w, i)] = (w, i - 1)
                else:
                    pred[(w, i)] = None
                nxt[w] += 1
                left -= 1
                moved = True
        if not moved:
            raise AssertionError("schedule deadlocks")

    makespan = max(fin[-1] for fin in finish if fin)
    bubbles, peaks = [], []
    for w, ops in enumerate(lists):
        busy = sum(cost[k] for k, _, _, _ in ops)
        bubbles.append(makespan - busy)
        live = peak = 0
        for kind, _, _, _ in ops:
            live += live_change[kind]
            assert live >= 0, "backward before forward"
            peak = max(peak, live)
        peaks.append(peak // 2 if peak % 2 == 0 else peak / 2)

    # critical path: walk back from the op that ends last (lowest worker wins ties)
    end = min((w for w in range(W) if finish[w] and finish[w][-1] == makespan))
    node = (end, len(lists[end]) - 1)
    cf = cb = 0
    while node is not None:
        w, i = node
        if lists[w][i][0] in (F, F2):
            cf += 1
        else:
            cb += 1
        node = pred[node]
    return dict(start=start, finish=finish, makespan=makespan, bubbles=bubbles,
                stash_peak=peaks, critical=(cf, cb))


def check_valid(lists, D, N, stages_per_worker):
    """Structural validity of a schedule; raises AssertionError when violated.

    Every (kind, micro-batch, stage) appears exactly once in the whole
    pipeline, every worker holds exactly `stages_per_worker` distinct stages,
    every forward precedes its backward on the same worker, and the replay
    does not deadlock (every dependency can be honoured in list order).
    """
    seen = set()
    for w, ops in enumerate(lists):
        stages = {s for _, _, _, s in ops}
        assert len(stages) == stages_per_worker, (w, stages)
        pos = {}
        for i, (kind, pipe, g, s) in enumerate(ops):
            assert (kind, g, s) not in seen
            seen.add((kind, g, s))
            pos[(kind, g, s)] = i
        for (kind, g, s), i in pos.items():
            if kind == B:
                assert (F, g, s) in pos and pos[(F, g, s)] < i
    assert seen == {(k, g, s) for k in (F, B) for g in range(N) for s in range(D)}
    simulate(lists, D)
    return True
