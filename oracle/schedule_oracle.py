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
* Section 3.5 "Scale to More Micro-Batches", direct concatenation: the table
  for D micro-batches is a basic unit; K = N/D units are chained so that the
  forwards of unit k+1 drop into the trailing bubbles of unit k.
* Section 2 "Bubbles in the pipeline" and Table 2: GPipe injects all N
  forwards and then runs all backwards; DAPPLE is 1F1B with a flush.
* Section 3.4: the critical path counts C_f, C_b.

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

F, B = 0, 1          # op kind
DOWN, UP = 0, 1      # pipeline


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


def chimera_grid(D, N):
    """Overlay of all pipelines and units: list over workers of {slot: op}.

    op = (kind, pipe, global_micro_batch, stage).
    """
    if D < 2 or D % 2:
        raise ValueError("Chimera needs an even number of stages")
    if N < D or N % D:
        raise ValueError("N must be a positive multiple of D")
    n = D // 2
    table = _pipeline_table(D, n)
    grid = [dict() for _ in range(D)]
    for k in range(N // D):
        for pipe in (DOWN, UP):
            for (kind, m, s), t in table.items():
                w = s if pipe == DOWN else D - 1 - s
                g = k * D + (m if pipe == DOWN else n + m)
                cell = 2 * D * k + t
                if cell in grid[w]:
                    raise AssertionError("merge conflict on worker %d slot %d" % (w, cell))
                grid[w][cell] = (kind, pipe, g, s)
    return grid


def chimera_schedule(D, N):
    """Per-worker op lists [(kind, pipe, mb, stage), ...] in execution order."""
    return [[row[t] for t in sorted(row)] for row in chimera_grid(D, N)]


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


def simulate(lists, D, cost_f=1, cost_b=1):
    """ASAP replay of per-worker op lists under the pipeline's data dependencies.

    Dependencies of a micro-batch g: forward at stage s needs forward at s-1;
    backward at the last stage needs the forward there; backward at stage s
    needs backward at s+1.  A worker runs its list strictly in order, one op at
    a time.  Returns a dict with
      start[w][i], finish[w][i]   per op,
      makespan,
      bubbles[w]   = makespan - busy time of worker w,
      stash_peak[w] = max over time of (#forwards - #backwards) run so far,
      critical     = (C_f, C_b): forwards and backwards on the chain of ops
                     that fixes the makespan (section 3.4).
    """
    W = len(lists)
    cost = {F: cost_f, B: cost_b}
    where = {}
    for w, ops in enumerate(lists):
        for i, (kind, pipe, g, s) in enumerate(ops):
            key = (kind, g, s)
            assert key not in where, "op listed twice: %r" % (key,)
            where[key] = (w, i)

    def dependency(kind, g, s):
        if kind == F:
            return (F, g, s - 1) if s > 0 else None
        return (B, g, s + 1) if s < D - 1 else (F, g, s)

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
            live += 1 if kind == F else -1
            assert live >= 0, "backward before forward"
            peak = max(peak, live)
        peaks.append(peak)

    # critical path: walk back from the op that ends last (lowest worker wins ties)
    end = min((w for w in range(W) if finish[w] and finish[w][-1] == makespan))
    node = (end, len(lists[end]) - 1)
    cf = cb = 0
    while node is not None:
        w, i = node
        if lists[w][i][0] == F:
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
