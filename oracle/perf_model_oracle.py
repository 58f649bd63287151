"""Performance-model oracle: predicted time of one training iteration.

TEST INFRASTRUCTURE ONLY.  Plain, slow reference that the tests compare the
library's model against.  It shares no code with the C++ library and the
product never imports it.

What it follows (Chimera paper, Li & Hoefler, SC'21, section 3.4
"Configuration Selection Based on Performance Modelling", Eq. (1)):

    T = (F_t + Comm_p2p) C_f + (B_t + Comm_p2p) C_b + max_i Comm_unoverlapped(i)

* F_t: measured forward time of one stage and micro-batch; B_t = 2 F_t, or 3 F_t
  with activation recomputation, when it is not measured itself.
* C_f, C_b: forwards and backwards on the critical path of the schedule.
* Comm_p2p = alpha + beta L for a message of L words (latency-bandwidth model).
* Comm_allreduce = 2 log2(r) alpha + 2 (r-1) beta L / r over r stage replicas
  (Rabenseifner's algorithm).
* Comm_unoverlapped(i): the part of worker i's gradient synchronisation that its
  free regions cannot hide (section 3.2: the allreduce of a stage is launched as
  soon as the stage's gradients are complete and proceeds in the bubbles).

Readings (the figure that draws the free regions is not in the text):

* The timeline is the as-soon-as-possible replay of the schedule with every
  forward costing F_t + Comm_p2p and every backward B_t + Comm_p2p; its makespan
  is the first two terms of Eq. (1) by the definition of the critical path.
* A worker's free regions are its idle intervals.  The allreduce of a stage can
  use the idle time after that stage's last backward; allreduces of one worker
  run one after the other in the order their stages complete; what is left
  when the iteration's computation ends (the makespan) is unoverlapped.
  Without eager launch every allreduce starts after the worker's last op.
* r = (stage replicas per pipeline group) x W: 2 f W for Chimera, W for the
  one-directional baselines.

Pinned by the tests: Rabenseifner's closed form against a step-by-step count
of recursive halving + doubling; T with free communication equals the
simulator's makespan (26 forward units for N = D = 6 with C_f = 6, C_b = 10,
section 3.4); section 3.2's remark that for D = 4 the middle workers have no
bubble between the completion of their first stage and the end of their
computation while the outer workers do.  PARITY UNPINNED by the paper: which
idle interval serves which replica (regions (a), (b), (c) of the missing
figure); the rule above is this file's reading.

Configuration selection (section 3.4, first and last paragraphs; section 4.3):
for every candidate (W, D) the micro-batch size is the largest one whose
memory fits the device (greedy), and among those the configuration with the
smallest modelled time per sample wins.  Memory of a worker (section 3.1 and
Table 2): the stage replicas it keeps (2f for Chimera, one otherwise), M_theta
each, plus M_a per micro-batch whose activations it holds at the worst moment
of the schedule.  Pinned by the tests against Table 2's intervals
([(D/2+1) M_a, D M_a] with 2 M_theta for Chimera, N M_a for GPipe, [M_a, D M_a]
for 1F1B) and on hand-built candidate sets; the candidate sets, the tie rule
(first candidate wins) and N = mini-batch / (W B) are this file's reading.
"""
import math

from . import schedule_oracle as so


def backward_time(f_t, recompute):
    """Section 3.4: a backward is modelled as two forwards, three with recomputation."""
    return (3.0 if recompute else 2.0) * f_t


def comm_p2p(alpha, beta, words):
    return alpha + beta * words


def comm_allreduce(alpha, beta, words, r):
    """Rabenseifner's allreduce over r replicas (section 3.4)."""
    if r < 1:
        raise ValueError("r must be >= 1")
    if r == 1:
        return 0.0
    return 2.0 * math.log2(r) * alpha + 2.0 * (r - 1) * beta * words / r


def free_regions(lists, sim):
    """Per worker: [(stage, time its gradients are complete)] sorted by time, the
    worker's idle intervals [(t0, t1)] up to the makespan, and the end of its last op."""
    out = []
    for w, ops in enumerate(lists):
        done = {}
        for (kind, pipe, g, s), fin in zip(ops, sim["finish"][w]):
            if kind not in (so.F, so.F2):
                done[s] = fin                        # ops are in time order: the last one stays
        idle, t = [], 0
        for a, b in zip(sim["start"][w], sim["finish"][w]):
            if a > t:
                idle.append((t, a))
            t = b
        if t < sim["makespan"]:
            idle.append((t, sim["makespan"]))
        out.append(dict(stages=sorted(done.items(), key=lambda kv: (kv[1], kv[0])), idle=idle, end=t))
    return out


def _idle_between(idle, t0, t1):
    return sum(max(0.0, min(b, t1) - max(a, t0)) for a, b in idle)


def unoverlapped(region, makespan, allreduce_cost, eager):
    """Allreduce time of one worker that its free regions cannot hide."""
    stages = region["stages"]
    if not eager:
        return max(0.0, len(stages) * allreduce_cost - _idle_between(region["idle"], region["end"], makespan))
    pending = 0.0
    for j, (_, t_done) in enumerate(stages):
        t_next = stages[j + 1][1] if j + 1 < len(stages) else makespan
        pending += allreduce_cost
        pending = max(0.0, pending - _idle_between(region["idle"], t_done, t_next))
    return pending


def iteration_time(lists, D, W, f_t, b_t, alpha, beta, act_words, grad_words, replicas_per_group, eager=True):
    """Eq. (1) for the schedule `lists` (per-worker op lists of the schedule oracle).

    act_words: size of one stage boundary message; grad_words: gradients of one stage;
    replicas_per_group: workers that hold the same stage inside one pipeline group
    (2f for Chimera, 1 for GPipe / 1F1B).  Returns a dict with T and its parts.
    """
    p2p = comm_p2p(alpha, beta, act_words)
    sim = so.simulate(lists, D, f_t + p2p, b_t + p2p)
    c_f, c_b = sim["critical"]
    compute = (f_t + p2p) * c_f + (b_t + p2p) * c_b
    assert abs(compute - sim["makespan"]) <= 1e-9 * max(1.0, compute), "critical path does not add up to the makespan"
    ar = comm_allreduce(alpha, beta, grad_words, replicas_per_group * W)
    regions = free_regions(lists, sim)
    rest = [unoverlapped(r, sim["makespan"], ar, eager) for r in regions]
    return dict(T=compute + max(rest), compute=f_t * c_f + b_t * c_b, p2p=(c_f + c_b) * p2p, c_f=c_f, c_b=c_b,
                allreduce=ar, unoverlapped=rest, comm_p2p=p2p)


def schedule_for(algo, D, N, f=1):
    """(op lists, stage replicas per pipeline group, stage replicas per worker) of a named schedule."""
    if algo == "chimera":
        return so.chimera_schedule(D, N, f), 2 * f, 2 * f
    if algo == "gpipe":
        return so.gpipe_schedule(D, N), 1, 1
    if algo == "1f1b":
        return so.one_f_one_b_schedule(D, N), 1, 1
    raise ValueError("unknown schedule %r" % (algo,))


def worker_memory(lists, D, replicas_on_worker, weight_bytes, act_bytes):
    """Bytes each worker needs (section 3.1, Table 2): its stage replicas and the
    activations of the micro-batches it holds at the worst moment."""
    peaks = so.simulate(lists, D, 1, 1)["stash_peak"]
    return [replicas_on_worker * weight_bytes + p * act_bytes for p in peaks]


def select_configuration(algo, f, minibatch, capacity_bytes, alpha, beta, candidates, eager=True):
    """Section 3.4: greedy micro-batch size per (W, D), then the best modelled throughput.

    candidates: dicts with D, W, B, f_t, b_t (None: modelled from f_t), recompute,
    act_words, grad_words, weight_bytes (M_theta of one stage replica), act_bytes
    (M_a of one stage and micro-batch).  Returns (evaluations, best index or None);
    an evaluation is None for a candidate whose W*B does not divide the mini-batch
    or whose schedule does not exist, else a dict N, mem_bytes, fits, T, throughput,
    c_f, c_b, chosen (largest fitting B of its (W, D)).
    """
    evals = []
    for c in candidates:
        per_iter = c["W"] * c["B"]
        if per_iter < 1 or minibatch % per_iter or minibatch // per_iter < 1:
            evals.append(None)
            continue
        N = minibatch // per_iter
        try:
            lists, per_group, per_worker = schedule_for(algo, c["D"], N, f)
        except ValueError:
            evals.append(None)
            continue
        mem = max(worker_memory(lists, c["D"], per_worker, c["weight_bytes"], c["act_bytes"]))
        b_t = backward_time(c["f_t"], c.get("recompute", False)) if c.get("b_t") is None else c["b_t"]
        r = iteration_time(lists, c["D"], c["W"], c["f_t"], b_t, alpha, beta, c["act_words"], c["grad_words"],
                           per_group, eager)
        evals.append(dict(N=N, mem_bytes=mem, fits=mem <= capacity_bytes, T=r["T"], throughput=minibatch / r["T"],
                          c_f=r["c_f"], c_b=r["c_b"], chosen=False))
    best = None
    for i, (c, e) in enumerate(zip(candidates, evals)):
        if e is None or not e["fits"]:
            continue
        bigger = any(e2 is not None and e2["fits"] and (c2["D"], c2["W"]) == (c["D"], c["W"]) and c2["B"] > c["B"]
                     for c2, e2 in zip(candidates, evals))
        if bigger:
            continue
        e["chosen"] = True
        if best is None or e["throughput"] > evals[best]["throughput"]:
            best = i
    return evals, best
