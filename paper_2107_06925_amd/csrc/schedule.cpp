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
#include "internal.h"

#include <algorithm>
#include <vector>

namespace chimera {

namespace {

struct Keyed { int64_t slot; Op op; };

int build_chimera(int D, int N, std::vector<std::vector<Op>>& lists) {
    if (D < 2 || (D & 1)) return fail(CHIMERA_EINVAL, "Chimera needs an even number of stages, got D=%d", D);
    if (N < D || N % D) return fail(CHIMERA_EINVAL, "N=%d must be a positive multiple of D=%d", N, D);
    const int n = D / 2, K = N / D;
    lists.assign(D, {});
    for (int w = 0; w < D; ++w) {
        std::vector<Keyed> ops;
        ops.reserve(2 * N);
        for (int k = 0; k < K; ++k)
            for (int pipe = 0; pipe < 2; ++pipe) {
                const int s = pipe == 0 ? w : D - 1 - w;
                for (int m = 0; m < n; ++m) {
                    const int g = k * D + (pipe == 0 ? m : n + m);
                    const int64_t base = (int64_t)2 * D * k + 2 * m;
                    Op f{}; f.kind = 0; f.pipe = pipe; f.mb = g; f.stage = s;
                    Op b = f; b.kind = 1;
                    ops.push_back({base + s, f});
                    ops.push_back({base + (2 * D - 1 - s), b});
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

int build_schedule(int algo, int D, int N, std::vector<std::vector<Op>>& lists) {
    if (D < 1 || N < 1) return fail(CHIMERA_EINVAL, "D=%d and N=%d must be positive", D, N);
    if ((int64_t)D * N > (int64_t)1 << 26) return fail(CHIMERA_EINVAL, "D*N too large");
    switch (algo) {
        case CHIMERA_DIRECT: return build_chimera(D, N, lists);
        case CHIMERA_GPIPE: return build_gpipe(D, N, lists);
        case CHIMERA_1F1B: return build_1f1b(D, N, lists);
        default: return fail(CHIMERA_EINVAL, "unknown schedule algorithm %d", algo);
    }
}

// ASAP replay.  done_f / done_b [g*D + s] hold finish times (-1 = not yet run).
int replay(const std::vector<std::vector<Op>>& lists, int D, int N, int64_t cost_f, int64_t cost_b,
           std::vector<std::vector<int64_t>>& start, ReplayStats* stats) {
    const int W = (int)lists.size();
    std::vector<int64_t> done[2];
    done[0].assign((size_t)N * D, -1);
    done[1].assign((size_t)N * D, -1);
    struct Ref { int w, i; };
    std::vector<Ref> where[2];
    where[0].assign((size_t)N * D, Ref{-1, -1});
    where[1].assign((size_t)N * D, Ref{-1, -1});
    for (int w = 0; w < W; ++w)
        for (int i = 0; i < (int)lists[w].size(); ++i) {
            const Op& o = lists[w][i];
            where[o.kind][(size_t)o.mb * D + o.stage] = Ref{w, i};
        }
    start.assign(W, {});
    std::vector<std::vector<int64_t>> fin(W);
    std::vector<std::vector<Ref>> pred(W);
    for (int w = 0; w < W; ++w) {
        start[w].assign(lists[w].size(), -1);
        fin[w].assign(lists[w].size(), -1);
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
                const int64_t t_worker = i ? fin[w][i - 1] : 0;
                int dk = -1, ds = 0;             // dependency (kind, stage) of the same micro-batch
                if (o.kind == 0) { if (o.stage > 0) { dk = 0; ds = o.stage - 1; } }
                else if (o.stage < D - 1) { dk = 1; ds = o.stage + 1; }
                else { dk = 0; ds = o.stage; }
                int64_t t_dep = 0;
                if (dk >= 0) {
                    t_dep = done[dk][(size_t)o.mb * D + ds];
                    if (t_dep < 0) break;        // producer has not run yet
                }
                const int64_t t0 = std::max(t_worker, t_dep);
                start[w][i] = t0;
                fin[w][i] = t0 + (o.kind == 0 ? cost_f : cost_b);
                done[o.kind][(size_t)o.mb * D + o.stage] = fin[w][i];
                if (dk >= 0 && t_dep == t0) pred[w][i] = where[dk][(size_t)o.mb * D + ds];
                else if (i && t_worker == t0) pred[w][i] = Ref{w, i - 1};
                ++next[w];
                --left;
                moved = true;
            }
        }
        if (!moved) return fail(CHIMERA_EINVAL, "internal: schedule deadlocks");
    }
    if (!stats) return CHIMERA_OK;
    int64_t makespan = 0;
    for (int w = 0; w < W; ++w)
        if (!fin[w].empty()) makespan = std::max(makespan, fin[w].back());
    stats->makespan = makespan;
    stats->bubbles.assign(W, 0);
    stats->stash_peak.assign(W, 0);
    for (int w = 0; w < W; ++w) {
        int64_t busy = 0;
        int live = 0, peak = 0;
        for (const Op& o : lists[w]) {
            busy += o.kind == 0 ? cost_f : cost_b;
            live += o.kind == 0 ? 1 : -1;
            peak = std::max(peak, live);
        }
        stats->bubbles[w] = makespan - busy;
        stats->stash_peak[w] = peak;
    }
    // critical path: back from the op that ends last (lowest worker on ties),
    // following the data dependency when it and the worker's previous op end together
    Ref node{-1, -1};
    for (int w = 0; w < W && node.w < 0; ++w)
        if (!fin[w].empty() && fin[w].back() == makespan) node = Ref{w, (int)lists[w].size() - 1};
    stats->cf = stats->cb = 0;
    while (node.w >= 0) {
        if (lists[node.w][node.i].kind == 0) ++stats->cf; else ++stats->cb;
        node = pred[node.w][node.i];
    }
    return CHIMERA_OK;
}

// Stash slots (lowest free slot of the op's stage at its forward), unit-cost
// start times and the "gradients of this stage are complete" flag.
int annotate(std::vector<std::vector<Op>>& lists, int D, int N) {
    std::vector<std::vector<int64_t>> start;
    int rc = replay(lists, D, N, 1, 1, start, nullptr);
    if (rc) return rc;
    for (size_t w = 0; w < lists.size(); ++w) {
        std::vector<char> used[2];
        std::vector<int> slot_of(N, -1);
        int last_b[2] = {-1, -1};
        for (size_t i = 0; i < lists[w].size(); ++i) {
            Op& o = lists[w][i];
            o.start = (int32_t)start[w][i];
            o.last_of_stage = 0;
            auto& u = used[o.pipe];
            if (o.kind == 0) {
                size_t s = 0;
                while (s < u.size() && u[s]) ++s;
                if (s == u.size()) u.push_back(0);
                u[s] = 1;
                slot_of[o.mb] = (int)s;
                o.slot = (int32_t)s;
            } else {
                o.slot = slot_of[o.mb];
                u[o.slot] = 0;
                last_b[o.pipe] = (int)i;
            }
        }
        for (int p = 0; p < 2; ++p)
            if (last_b[p] >= 0) lists[w][last_b[p]].last_of_stage = 1;
    }
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
