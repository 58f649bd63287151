// Pipeline schedules for one training iteration: Chimera's bidirectional
// schedule with direct concatenation (sections 3.1 and 3.5) and the GPipe and
// 1F1B baselines (section 2), plus an as-soon-as-possible replay of all D
// workers that yields start times, bubbles, stash peaks and the critical path
// counts C_f, C_b of section 3.4.  Host code only.
//
// Chimera in closed form.  With n = D/2 micro-batches per pipeline and unit,
// a micro-batch enters its pipeline every second time slot (the 1F1B steady
// state), advances one stage per slot, and turns round at the last stage:
//     forward  of local micro-batch m at stage s:  slot = s + 2m
//     backward of local micro-batch m at stage s:  slot = (2D-1-s) + 2m
// Unit k is shifted by 2D slots.  The down pipeline puts stage s on worker s,
// the up pipeline on worker D-1-s; because D-1 is odd the two pipelines use
// slots of opposite parity on any worker, or the same parity in disjoint
// ranges, so sorting a worker's ops by slot gives a total order.
//
// 2f pipelines (section 3.6, Table 3): f down and f up pipelines with n = D/(2f)
// micro-batches each per unit, all injected in lockstep with the same two slot
// formulas; down pipeline i holds stage s on worker (i D/f + s) mod D, up pipeline
// i on worker (i D/f + D-1-s) mod D.
//
// Forward doubling and backward halving (section 3.5) keep the order of the
// direct schedule: doubling reads it for N/2 double micro-batches and turns the
// forward of double j into one forward over micro-batches 2j and 2j+1 and its
// backward into the backwards of 2j and 2j+1; halving cuts every backward into
// its two halves.  Backward chunks depend on the same chunk of the next stage only.
//
// Performance model (section 3.4, Eq. (1)) at the end of the file.
#include "internal.h"

#include <algorithm>
#include <cmath>
#include <utility>
#include <vector>

namespace chimera {

namespace {

struct Keyed { int64_t slot; Op op; };

int build_chimera(int D, int N, int f, std::vector<std::vector<Op>>& lists) {
    if (D < 2 || (D & 1)) return fail(CHIMERA_EINVAL, "Chimera needs an even number of stages, got D=%d", D);
    if (N > D && N % D) return fail(CHIMERA_EINVAL, "N=%d must be a multiple of D=%d, or smaller than D", N, D);
    if (f < 1 || (D / 2) % f) return fail(CHIMERA_EINVAL, "f=%d must divide D/2=%d", f, D / 2);
    // Fewer micro-batches than stages (section 3.1): one partial unit, the micro-batches split
    // between the two pipelines as evenly as possible (the down pipeline takes the odd one).
    const bool partial = N < D;
    if (partial && f != 1) return fail(CHIMERA_EINVAL, "N < D is defined for two pipelines (f=1)");
    const int n_full = D / (2 * f), K = partial ? 1 : N / D, span = D / f;
    const int n_down = (N + 1) / 2;
    lists.assign(D, {});
    for (int w = 0; w < D; ++w) {
        std::vector<Keyed> ops;
        ops.reserve(2 * N);
        for (int k = 0; k < K; ++k)
            for (int pipe = 0; pipe < 2 * f; ++pipe) {
                const int i = pipe >> 1, up = pipe & 1;
                // stage of this pipeline that worker w holds
                const int s = up ? ((i * span + D - 1 - w) % D + D) % D : ((w - i * span) % D + D) % D;
                const int block = up ? f + i : i;           // which n ids of the unit this pipeline carries
                const int n = partial ? (up ? N - n_down : n_down) : n_full;
                const int first = partial ? (up ? n_down : 0) : k * D + block * n_full;
                for (int m = 0; m < n; ++m) {
                    const int g = first + m;
                    const int64_t base = (int64_t)2 * D * k + 2 * m;
                    Op fw{}; fw.kind = CHIMERA_OP_F; fw.pipe = pipe; fw.mb = g; fw.stage = s;
                    Op bw = fw; bw.kind = CHIMERA_OP_B;
                    ops.push_back({base + s, fw});
                    ops.push_back({base + (2 * D - 1 - s), bw});
                }
            }
        std::sort(ops.begin(), ops.end(), [](const Keyed& a, const Keyed& b) { return a.slot < b.slot; });
        for (size_t i = 1; i < ops.size(); ++i)
            if (ops[i].slot == ops[i - 1].slot)
                return fail(CHIMERA_EINVAL, "internal: slot conflict on worker %d", w);
        for (auto& k : ops) lists[w].push_back(k.op);
    }
    return CHIMERA_OK;
}

int build_doubling(int D, int N, std::vector<std::vector<Op>>& lists) {
    if (D < 2 || (D & 1)) return fail(CHIMERA_EINVAL, "Chimera needs an even number of stages, got D=%d", D);
    if (N < 2 * D || N % D) return fail(CHIMERA_EINVAL, "forward doubling needs N=%d to be K*D with K >= 2 (D=%d)", N, D);
    const int K = N / D;
    std::vector<std::vector<Op>> doubles, rest;
    int rc = build_chimera(D, (K / 2) * D, 1, doubles);
    if (rc) return rc;
    if (K & 1) { rc = build_chimera(D, D, 1, rest); if (rc) return rc; }
    lists.assign(D, {});
    for (int w = 0; w < D; ++w) {
        for (const Op& o : doubles[w]) {
            Op a = o;
            a.mb = 2 * o.mb;
            if (o.kind == CHIMERA_OP_F) { a.kind = CHIMERA_OP_F2; lists[w].push_back(a); }
            else { lists[w].push_back(a); a.mb += 1; lists[w].push_back(a); }
        }
        if (K & 1)
            for (const Op& o : rest[w]) { Op a = o; a.mb += (K - 1) * D; lists[w].push_back(a); }
    }
    return CHIMERA_OK;
}

int build_halving(int D, int N, std::vector<std::vector<Op>>& lists) {
    std::vector<std::vector<Op>> direct;
    int rc = build_chimera(D, N, 1, direct);
    if (rc) return rc;
    lists.assign(D, {});
    for (int w = 0; w < D; ++w)
        for (const Op& o : direct[w]) {
            if (o.kind == CHIMERA_OP_F) { lists[w].push_back(o); continue; }
            Op a = o;
            a.kind = CHIMERA_OP_BH0; lists[w].push_back(a);
            a.kind = CHIMERA_OP_BH1; lists[w].push_back(a);
        }
    return CHIMERA_OK;
}

int build_gpipe(int D, int N, std::vector<std::vector<Op>>& lists) {
    lists.assign(D, {});
    for (int s = 0; s < D; ++s) {
        for (int g = 0; g < N; ++g) { Op o{}; o.kind = 0; o.mb = g; o.stage = s; lists[s].push_back(o); }
        for (int g = 0; g < N; ++g) { Op o{}; o.kind = 1; o.mb = g; o.stage = s; lists[s].push_back(o); }
    }
    return CHIMERA_OK;
}

// 1F1B: stage s keeps at most D-s micro-batches in flight.
int build_1f1b(int D, int N, std::vector<std::vector<Op>>& lists) {
    lists.assign(D, {});
    for (int s = 0; s < D; ++s) {
        int nf = 0, nb = 0;
        auto push = [&](int kind, int g) { Op o{}; o.kind = kind; o.mb = g; o.stage = s; lists[s].push_back(o); };
        const int warm = std::min(D - s, N);
        while (nf < warm) push(0, nf++);
        while (nb < N) {
            push(1, nb++);
            if (nf < N) push(0, nf++);
        }
    }
    return CHIMERA_OK;
}

}  // namespace

int build_schedule(int algo, int D, int N, int f, std::vector<std::vector<Op>>& lists) {
    if (D < 1 || N < 1) return fail(CHIMERA_EINVAL, "D=%d and N=%d must be positive", D, N);
    if ((int64_t)D * N > (int64_t)1 << 26) return fail(CHIMERA_EINVAL, "D*N too large");
    if (algo != CHIMERA_DIRECT && f != 1) return fail(CHIMERA_EINVAL, "f=%d: only the direct Chimera schedule has 2f pipelines", f);
    switch (algo) {
        case CHIMERA_DIRECT: return build_chimera(D, N, f, lists);
        case CHIMERA_GPIPE: return build_gpipe(D, N, lists);
        case CHIMERA_1F1B: return build_1f1b(D, N, lists);
        case CHIMERA_DOUBLING: return build_doubling(D, N, lists);
        case CHIMERA_HALVING: return build_halving(D, N, lists);
        default: return fail(CHIMERA_EINVAL, "unknown schedule algorithm %d", algo);
    }
}
int build_schedule(int algo, int D, int N, std::vector<std::vector<Op>>& lists) { return build_schedule(algo, D, N, 1, lists); }

// ASAP replay.  done[kind][g*D + s] hold finish times (-1 = not yet run).  cost[kind] for
// the five op kinds.  T = int64_t (slot counts) or double (seconds, for the performance model).
namespace {
inline bool is_forward(int kind) { return kind == CHIMERA_OP_F || kind == CHIMERA_OP_F2; }
}

template <typename T>
int replay_costs(const std::vector<std::vector<Op>>& lists, int D, int N, const T (&cost)[CHIMERA_OP_KINDS],
                 std::vector<std::vector<T>>& start, std::vector<std::vector<T>>& fin, ReplayStatsT<T>* stats) {
    const int W = (int)lists.size();
    std::vector<T> done[CHIMERA_OP_KINDS];
    struct Ref { int w, i; };
    std::vector<Ref> where[CHIMERA_OP_KINDS];
    for (int k = 0; k < CHIMERA_OP_KINDS; ++k) {
        done[k].assign((size_t)N * D, (T)-1);
        where[k].assign((size_t)N * D, Ref{-1, -1});
    }
    for (int w = 0; w < W; ++w)
        for (int i = 0; i < (int)lists[w].size(); ++i) {
            const Op& o = lists[w][i];
            if (o.kind < 0 || o.kind >= CHIMERA_OP_KINDS || o.mb < 0 || o.mb >= N || o.stage < 0 || o.stage >= D)
                return fail(CHIMERA_EINVAL, "internal: malformed op");
            where[o.kind][(size_t)o.mb * D + o.stage] = Ref{w, i};
        }
    start.assign(W, {});
    fin.assign(W, {});
    std::vector<std::vector<Ref>> pred(W);
    for (int w = 0; w < W; ++w) {
        start[w].assign(lists[w].size(), (T)-1);
        fin[w].assign(lists[w].size(), (T)-1);
        pred[w].assign(lists[w].size(), Ref{-1, -1});
    }
    std::vector<int> next(W, 0);
    size_t left = 0;
    for (auto& l : lists) left += l.size();
    while (left) {
        bool moved = false;
        for (int w = 0; w < W; ++w) {
            while (next[w] < (int)lists[w].size()) {
                const int i = next[w];
                const Op& o = lists[w][i];
                const T t_worker = i ? fin[w][i - 1] : (T)0;
                // dependency (kind, micro-batch, stage)
                int dk = -1, dg = o.mb, ds = 0;
                if (is_forward(o.kind)) { if (o.stage > 0) { dk = o.kind; ds = o.stage - 1; } }
                else if (o.stage < D - 1) { dk = o.kind; ds = o.stage + 1; }
                else {
                    ds = o.stage;
                    if (where[CHIMERA_OP_F][(size_t)o.mb * D + ds].w >= 0) dk = CHIMERA_OP_F;
                    else { dk = CHIMERA_OP_F2; dg = o.mb - (o.mb & 1); }      // the doubled forward that carried it
                }
                T t_dep = 0;
                if (dk >= 0) {
                    if (where[dk][(size_t)dg * D + ds].w < 0) return fail(CHIMERA_EINVAL, "internal: op without producer");
                    t_dep = done[dk][(size_t)dg * D + ds];
                    if (t_dep < 0) break;        // producer has not run yet
                }
                const T t0 = std::max(t_worker, t_dep);
                start[w][i] = t0;
                fin[w][i] = t0 + cost[o.kind];
                done[o.kind][(size_t)o.mb * D + o.stage] = fin[w][i];
                if (dk >= 0 && t_dep == t0) pred[w][i] = where[dk][(size_t)dg * D + ds];
                else if (i && t_worker == t0) pred[w][i] = Ref{w, i - 1};
                ++next[w];
                --left;
                moved = true;
            }
        }
        if (!moved) return fail(CHIMERA_EINVAL, "internal: schedule deadlocks");
    }
    if (!stats) return CHIMERA_OK;
    T makespan = 0;
    for (int w = 0; w < W; ++w)
        if (!fin[w].empty()) makespan = std::max(makespan, fin[w].back());
    stats->makespan = makespan;
    stats->bubbles.assign(W, 0);
    stats->stash_peak_halves.assign(W, 0);
    static const int live_change[CHIMERA_OP_KINDS] = {2, -2, 4, -1, -1};      // in half micro-batches
    for (int w = 0; w < W; ++w) {
        T busy = 0;
        int live = 0, peak = 0;
        for (const Op& o : lists[w]) {
            busy += cost[o.kind];
            live += live_change[o.kind];
            peak = std::max(peak, live);
        }
        stats->bubbles[w] = makespan - busy;
        stats->stash_peak_halves[w] = peak;
    }
    // critical path: back from the op that ends last (lowest worker on ties),
    // following the data dependency when it and the worker's previous op end together
    Ref node{-1, -1};
    for (int w = 0; w < W && node.w < 0; ++w)
        if (!fin[w].empty() && fin[w].back() == makespan) node = Ref{w, (int)lists[w].size() - 1};
    stats->cf = stats->cb = 0;
    while (node.w >= 0) {
        if (is_forward(lists[node.w][node.i].kind)) ++stats->cf; else ++stats->cb;
        node = pred[node.w][node.i];
    }
    return CHIMERA_OK;
}

int replay(const std::vector<std::vector<Op>>& lists, int D, int N, int64_t cost_f, int64_t cost_b,
           std::vector<std::vector<int64_t>>& start, ReplayStats* stats) {
    // a doubled forward is priced like a backward chunk and a half backward like a forward (section 3.5)
    const int64_t cost[CHIMERA_OP_KINDS] = {cost_f, cost_b, cost_b, cost_f, cost_f};
    std::vector<std::vector<int64_t>> fin;
    ReplayStatsT<int64_t> st;
    int rc = replay_costs<int64_t>(lists, D, N, cost, start, fin, stats ? &st : nullptr);
    if (rc || !stats) return rc;
    stats->makespan = st.makespan; stats->bubbles = st.bubbles; stats->cf = st.cf; stats->cb = st.cb;
    stats->stash_peak.assign(st.stash_peak_halves.size(), 0);
    for (size_t w = 0; w < st.stash_peak_halves.size(); ++w) stats->stash_peak[w] = (st.stash_peak_halves[w] + 1) / 2;
    return CHIMERA_OK;
}

// Stash slots (lowest free slot of the op's pipeline at its forward), unit-cost
// start times and the "gradients of this stage are complete" flag.  A doubled
// forward keeps no activations (slot -1); the backwards that follow it recompute
// into whatever slot is free when they run (slot -1 as well).
int annotate(std::vector<std::vector<Op>>& lists, int D, int N) {
    std::vector<std::vector<int64_t>> start;
    int rc = replay(lists, D, N, 1, 1, start, nullptr);
    if (rc) return rc;
    for (size_t w = 0; w < lists.size(); ++w) {
        int pipes = 0;
        for (const Op& o : lists[w]) pipes = std::max(pipes, o.pipe + 1);
        std::vector<std::vector<char>> used(pipes);
        std::vector<int> slot_of(N, -1);
        std::vector<int> last_b(pipes, -1);
        for (size_t i = 0; i < lists[w].size(); ++i) {
            Op& o = lists[w][i];
            o.start = (int32_t)start[w][i];
            o.last_of_stage = 0;
            auto& u = used[o.pipe];
            if (o.kind == CHIMERA_OP_F) {
                size_t s = 0;
                while (s < u.size() && u[s]) ++s;
                if (s == u.size()) u.push_back(0);
                u[s] = 1;
                slot_of[o.mb] = (int)s;
                o.slot = (int32_t)s;
            } else if (o.kind == CHIMERA_OP_F2) {
                o.slot = -1;
            } else {
                o.slot = slot_of[o.mb];
                if (o.slot >= 0 && o.kind != CHIMERA_OP_BH0) u[o.slot] = 0;      // the first half keeps the slot
                last_b[o.pipe] = (int)i;
            }
        }
        for (int p = 0; p < pipes; ++p)
            if (last_b[p] >= 0) lists[w][last_b[p]].last_of_stage = 1;
    }
    return CHIMERA_OK;
}

// ------------------------------------------------------------ performance model
// Section 3.4.  The timeline is the ASAP replay with every forward costing F_t + Comm_p2p
// and every backward B_t + Comm_p2p (its makespan is the first two terms of Eq. (1)).  A
// worker's free regions are its idle intervals; the allreduce of a stage may use the idle
// time after that stage's last backward, the allreduces of a worker run one after the
// other in the order their stages complete, and what is left at the makespan is
// Comm_unoverlapped(i).  Without eager launch all of them start after the worker's last op.
namespace {

double idle_between(const std::vector<std::pair<double, double>>& idle, double t0, double t1) {
    double sum = 0;
    for (const auto& iv : idle) sum += std::max(0.0, std::min(iv.second, t1) - std::max(iv.first, t0));
    return sum;
}

}  // namespace

int model_iteration(int algo, int D, int N, int f, int W, double f_t, double b_t, double alpha, double beta,
                    double act_words, double grad_words, int eager, ModelResult* out) {
    if (W < 1) return fail(CHIMERA_EINVAL, "W=%d must be positive", W);
    if (!(f_t > 0) || !(b_t > 0) || alpha < 0 || beta < 0 || act_words < 0 || grad_words < 0)
        return fail(CHIMERA_EINVAL, "times must be positive, communication parameters non-negative");
    if (algo == CHIMERA_DOUBLING || algo == CHIMERA_HALVING) return fail(CHIMERA_EINVAL, "the model covers whole-micro-batch schedules");
    std::vector<std::vector<Op>> lists;
    int rc = build_schedule(algo, D, N, f, lists);
    if (rc) return rc;
    const double p2p = alpha + beta * act_words;
    const double cost[CHIMERA_OP_KINDS] = {f_t + p2p, b_t + p2p, b_t + p2p, f_t + p2p, f_t + p2p};
    std::vector<std::vector<double>> start, fin;
    ReplayStatsT<double> st;
    rc = replay_costs<double>(lists, D, N, cost, start, fin, &st);
    if (rc) return rc;
    const int r = (algo == CHIMERA_DIRECT ? 2 * f : 1) * W;          // replicas of one stage
    const double ar = r <= 1 ? 0.0 : 2.0 * std::log2((double)r) * alpha + 2.0 * (r - 1) * beta * grad_words / r;
    double worst = 0;
    for (int w = 0; w < D; ++w) {
        // completion time of every stage this worker holds, in completion order
        std::vector<std::pair<double, int>> stages;
        for (size_t i = 0; i < lists[w].size(); ++i) {
            const Op& o = lists[w][i];
            if (is_forward(o.kind)) continue;
            bool seen = false;
            for (auto& sd : stages) if (sd.second == o.stage) { sd.first = fin[w][i]; seen = true; }
            if (!seen) stages.push_back({fin[w][i], o.stage});
        }
        std::sort(stages.begin(), stages.end());
        std::vector<std::pair<double, double>> idle;
        double t = 0;
        for (size_t i = 0; i < lists[w].size(); ++i) {
            if (start[w][i] > t) idle.push_back({t, start[w][i]});
            t = fin[w][i];
        }
        if (t < st.makespan) idle.push_back({t, st.makespan});
        double pending = 0;
        if (!eager) {
            pending = std::max(0.0, stages.size() * ar - idle_between(idle, t, st.makespan));
        } else {
            for (size_t j = 0; j < stages.size(); ++j) {
                const double t_next = j + 1 < stages.size() ? stages[j + 1].first : st.makespan;
                pending += ar;
                pending = std::max(0.0, pending - idle_between(idle, stages[j].first, t_next));
            }
        }
        worst = std::max(worst, pending);
    }
    out->c_f = st.cf; out->c_b = st.cb;
    out->compute = f_t * st.cf + b_t * st.cb;
    out->p2p = (st.cf + st.cb) * p2p;
    out->allreduce = ar;
    out->unoverlapped = worst;
    out->T = (f_t + p2p) * st.cf + (b_t + p2p) * st.cb + worst;
    return CHIMERA_OK;
}

}  // namespace chimera

using namespace chimera;

extern "C" int chimera_schedule(int algo, int D, int N, int rank, chimera_op* h_out, size_t cap,
                                size_t* h_count) {
    std::vector<std::vector<Op>> lists;
    int rc = build_schedule(algo, D, N, lists);
    if (rc) return rc;
    if (rank < 0 || rank >= D) return fail(CHIMERA_EINVAL, "rank %d outside [0,%d)", rank, D);
    rc = annotate(lists, D, N);
    if (rc) return rc;
    const auto& l = lists[rank];
    if (h_count) *h_count = l.size();
    if (cap && !h_out) return fail(CHIMERA_EINVAL, "h_out is NULL");
    const size_t n = std::min(cap, l.size());
    for (size_t i = 0; i < n; ++i) h_out[i] = l[i];
    if (cap < l.size() && cap) return fail(CHIMERA_ENOMEM, "op list has %zu entries, capacity %zu", l.size(), cap);
    return CHIMERA_OK;
}

extern "C" int chimera_schedule_stats(int algo, int D, int N, int cost_f, int cost_b, int64_t* h_makespan,
                                      int64_t* h_bubbles, int32_t* h_stash_peak, int32_t* h_critical) {
    if (cost_f < 1 || cost_b < 1) return fail(CHIMERA_EINVAL, "costs must be >= 1");
    std::vector<std::vector<Op>> lists;
    int rc = build_schedule(algo, D, N, lists);
    if (rc) return rc;
    std::vector<std::vector<int64_t>> start;
    ReplayStats st;
    rc = replay(lists, D, N, cost_f, cost_b, start, &st);
    if (rc) return rc;
    if (h_makespan) *h_makespan = st.makespan;
    for (int w = 0; w < D; ++w) {
        if (h_bubbles) h_bubbles[w] = st.bubbles[w];
        if (h_stash_peak) h_stash_peak[w] = st.stash_peak[w];
    }
    if (h_critical) { h_critical[0] = st.cf; h_critical[1] = st.cb; }
    return CHIMERA_OK;
}

extern "C" int chimera_schedule_pipes(int algo, int D, int N, int f, int rank, chimera_op* h_out, size_t cap,
                                      size_t* h_count) {
    std::vector<std::vector<Op>> lists;
    int rc = build_schedule(algo, D, N, f, lists);
    if (rc) return rc;
    if (rank < 0 || rank >= D) return fail(CHIMERA_EINVAL, "rank %d outside [0,%d)", rank, D);
    rc = annotate(lists, D, N);
    if (rc) return rc;
    const auto& l = lists[rank];
    if (h_count) *h_count = l.size();
    if (cap && !h_out) return fail(CHIMERA_EINVAL, "h_out is NULL");
    const size_t n = std::min(cap, l.size());
    for (size_t i = 0; i < n; ++i) h_out[i] = l[i];
    if (cap < l.size() && cap) return fail(CHIMERA_ENOMEM, "op list has %zu entries, capacity %zu", l.size(), cap);
    return CHIMERA_OK;
}

extern "C" int chimera_schedule_stats_costs(int algo, int D, int N, int f, const int64_t* h_cost, int64_t* h_makespan,
                                            int64_t* h_bubbles, int32_t* h_stash_peak_halves, int32_t* h_critical) {
    if (!h_cost) return fail(CHIMERA_EINVAL, "h_cost is NULL");
    int64_t cost[CHIMERA_OP_KINDS];
    for (int k = 0; k < CHIMERA_OP_KINDS; ++k) {
        if (h_cost[k] < 1) return fail(CHIMERA_EINVAL, "costs must be >= 1");
        cost[k] = h_cost[k];
    }
    std::vector<std::vector<Op>> lists;
    int rc = build_schedule(algo, D, N, f, lists);
    if (rc) return rc;
    std::vector<std::vector<int64_t>> start, fin;
    ReplayStatsT<int64_t> st;
    rc = replay_costs<int64_t>(lists, D, N, cost, start, fin, &st);
    if (rc) return rc;
    if (h_makespan) *h_makespan = st.makespan;
    for (int w = 0; w < D; ++w) {
        if (h_bubbles) h_bubbles[w] = st.bubbles[w];
        if (h_stash_peak_halves) h_stash_peak_halves[w] = st.stash_peak_halves[w];
    }
    if (h_critical) { h_critical[0] = st.cf; h_critical[1] = st.cb; }
    return CHIMERA_OK;
}

extern "C" int chimera_pipe_worker(int D, int f, int pipe, int stage) {
    if (D < 2 || (D & 1) || f < 1 || (D / 2) % f) return fail(CHIMERA_EINVAL, "D=%d must be even and f=%d divide D/2", D, f);
    if (pipe < 0 || pipe >= 2 * f || stage < 0 || stage >= D) return fail(CHIMERA_EINVAL, "pipe %d or stage %d out of range", pipe, stage);
    const int first = (pipe >> 1) * (D / f);
    return (pipe & 1) ? (first + D - 1 - stage) % D : (first + stage) % D;
}

extern "C" int chimera_model_iteration_time(int algo, int D, int N, int f, int W, double f_t, double b_t, double alpha,
                                            double beta, double act_words, double grad_words, int eager,
                                            double* h_out) {
    if (!h_out) return fail(CHIMERA_EINVAL, "h_out is NULL");
    ModelResult r{};
    int rc = model_iteration(algo, D, N, f, W, f_t, b_t, alpha, beta, act_words, grad_words, eager, &r);
    if (rc) return rc;
    h_out[0] = r.T; h_out[1] = r.compute; h_out[2] = r.p2p; h_out[3] = r.allreduce; h_out[4] = r.unoverlapped;
    h_out[5] = r.c_f; h_out[6] = r.c_b;
    return CHIMERA_OK;
}

extern "C" int chimera_model_select(int algo, int f, int64_t minibatch, double capacity_bytes, double alpha, double beta,
                                    int eager, int count, const chimera_candidate* h_cand,
                                    chimera_candidate_eval* h_eval, int* h_best) {
    if (count < 1 || !h_cand || !h_eval || !h_best) return fail(CHIMERA_EINVAL, "count must be positive and the arrays non-NULL");
    if (minibatch < 1 || capacity_bytes < 0 || alpha < 0 || beta < 0) return fail(CHIMERA_EINVAL, "mini-batch must be positive, capacity and communication parameters non-negative");
    if (algo != CHIMERA_DIRECT && algo != CHIMERA_GPIPE && algo != CHIMERA_1F1B) return fail(CHIMERA_EINVAL, "the model covers whole-micro-batch schedules");
    for (int i = 0; i < count; ++i) {
        const chimera_candidate& c = h_cand[i];
        if (!(c.f_t > 0) || c.act_words < 0 || c.grad_words < 0 || c.weight_bytes < 0 || c.act_bytes < 0 || c.D < 1 || c.W < 1 || c.B < 1)
            return fail(CHIMERA_EINVAL, "candidate %d: D, W, B and f_t must be positive, sizes non-negative", i);
    }
    const int replicas = algo == CHIMERA_DIRECT ? 2 * f : 1;        // stage replicas a worker keeps
    for (int i = 0; i < count; ++i) {
        const chimera_candidate& c = h_cand[i];
        chimera_candidate_eval& e = h_eval[i];
        e = chimera_candidate_eval{};
        const int64_t per_iter = (int64_t)c.W * c.B;
        if (minibatch % per_iter || minibatch / per_iter > (int64_t)1 << 20) continue;
        const int N = (int)(minibatch / per_iter);
        std::vector<std::vector<Op>> lists;
        if (build_schedule(algo, c.D, N, f, lists)) continue;                 // e.g. odd D for Chimera
        const int64_t unit[CHIMERA_OP_KINDS] = {1, 1, 1, 1, 1};
        std::vector<std::vector<int64_t>> start, fin;
        ReplayStatsT<int64_t> st;
        if (replay_costs<int64_t>(lists, c.D, N, unit, start, fin, &st)) continue;
        int peak = 0;
        for (int32_t h : st.stash_peak_halves) peak = std::max(peak, (int)h);
        const double b_t = c.b_t > 0 ? c.b_t : (c.recompute ? 3.0 : 2.0) * c.f_t;
        ModelResult r{};
        if (model_iteration(algo, c.D, N, f, c.W, c.f_t, b_t, alpha, beta, c.act_words, c.grad_words, eager, &r)) continue;
        e.valid = 1; e.N = N; e.c_f = r.c_f; e.c_b = r.c_b;
        e.mem_bytes = replicas * c.weight_bytes + 0.5 * peak * c.act_bytes;
        e.fits = e.mem_bytes <= capacity_bytes;
        e.T = r.T;
        e.throughput = (double)minibatch / r.T;
    }
    int best = -1;
    for (int i = 0; i < count; ++i) {
        if (!h_eval[i].valid || !h_eval[i].fits) continue;
        bool bigger = false;
        for (int j = 0; j < count; ++j)
            bigger = bigger || (h_eval[j].valid && h_eval[j].fits && h_cand[j].D == h_cand[i].D && h_cand[j].W == h_cand[i].W &&
                                h_cand[j].B > h_cand[i].B);
        if (bigger) continue;
        h_eval[i].chosen = 1;
        if (best < 0 || h_eval[i].throughput > h_eval[best].throughput) best = i;
    }
    *h_best = best;
    return CHIMERA_OK;
}
