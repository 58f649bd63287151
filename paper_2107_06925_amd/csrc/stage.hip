// Stage runtime and C ABI: a stage of L Transformer blocks (forward, backward
// with in-place float gradient accumulation), its activation stash, and the
// replay of a worker's op list (section 3.1: worker i runs stage i of the down
// pipeline and stage D-1-i of the up pipeline in the merged 1F1B order).
#include <chrono>
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <unordered_map>
#include <vector>

#include "internal.h"

namespace chimera {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

static inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

// Optional per-kernel-class timing: a HIP event pair around every launch of a
// class on the stage's stream, summed after the stream has been waited for.
enum ProfClass { PC_GEMM_FWD, PC_GEMM_DGRAD, PC_GEMM_WGRAD, PC_ATTN_FWD, PC_ATTN_BWD, PC_LN_FWD, PC_LN_BWD, PC_COLSUM, PC_GEMM_WGRAD_TAIL, PC_COUNT };
struct ProfRec { hipEvent_t a, b; int cls; double work; };
struct Profiler {
    bool on = false;
    std::vector<ProfRec> recs;
    double ms[PC_COUNT] = {}, work[PC_COUNT] = {};
    long long launches[PC_COUNT] = {};
} g_prof;

struct ProfScope {
    hipStream_t s; bool live = false; ProfRec r{};
    ProfScope(int cls, double work, hipStream_t stream) : s(stream) {
        if (!g_prof.on) return;
        if (hipEventCreate(&r.a) != hipSuccess) return;
        if (hipEventCreate(&r.b) != hipSuccess) { (void)hipEventDestroy(r.a); return; }
        r.cls = cls; r.work = work; live = true;
        (void)hipEventRecord(r.a, s);
    }
    ~ProfScope() {
        if (!live) return;
        (void)hipEventRecord(r.b, s);
        g_prof.recs.push_back(r);
    }
};

// Folds finished event pairs into the totals; the stream(s) must be idle.
static void prof_collect() {
    for (ProfRec& r : g_prof.recs) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, r.a, r.b) == hipSuccess) {
            g_prof.ms[r.cls] += t; g_prof.work[r.cls] += r.work; ++g_prof.launches[r.cls];
        }
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    g_prof.recs.clear();
}

}  // namespace chimera

using namespace chimera;

struct chimera_stage {
    int L, H, heads, S, B, dtype;
    int M, d;
    size_t esz;
    int causal = 1, gelu_erf = 0, kernels = 0, overlap = 1, keep = 1;
    bool bound = false;
    // rows (tokens) and sequences the running op works on: the whole micro-batch, or one half
    // of it in a half backward
    int vM = 0, vB = 0;

    // parameter offsets (elements) inside one block and block size
    size_t o_ln1_g, o_ln1_b, o_w_qkv, o_b_qkv, o_w_o, o_b_o, o_ln2_g, o_ln2_b, o_w_fc1, o_b_fc1, o_w_fc2, o_b_fc2;
    size_t layer_params;

    // stash layout (bytes) inside one block of one slot
    size_t s_mean1, s_rstd1, s_h1, s_qkv, s_ctx, s_lse, s_x1, s_mean2, s_rstd2, s_h2, s_u, s_g, s_y;
    size_t layer_stash, slot_bytes;

    // workspace layout (bytes)
    size_t w_dy[2], w_dyf[2], w_dx1f, w_du[2], w_dh, w_dx1[2], w_dctx, w_dqkv[2], w_delta, w_scratch, w_scratch2, w_lnpart, lnpart_floats, ws_bytes;

    const char* weights = nullptr;
    float* grads = nullptr;
    char* stash = nullptr;
    char* ws = nullptr;
    int slots = 0;
    hipStream_t stream = nullptr;
    // Weight and bias gradients run on a second stream beside the chain of input
    // gradients: they are off the critical path of a backward and fill the CUs that
    // the chain's smaller kernels leave idle.  Gradient buffers are only ever
    // touched by that stream (or by the main one with the side stream idle).
    hipStream_t side = nullptr;
    hipEvent_t ev_ready[4] = {};      // main -> side: dy, du, dx1, dqkv of the current block are written
    hipEvent_t ev_side[2] = {};       // side -> main: the side work of a block (by parity) is done
    bool have_side = false;

    struct IO { const void* x; void* y; const void* dy; void* dx; };
    std::unordered_map<int, IO> io;
    std::unordered_map<int, int> in_flight;   // micro-batch -> slot
    std::unordered_map<int, int> halves_done; // micro-batch -> halves of its backward already run
    // chimera_stage_zero_grads only notes that the gradients are to be read as zero: the next
    // backward then WRITES every gradient instead of accumulating (no fill pass, no read of the
    // old values); anything else that looks at the buffer first performs the fill.
    bool grads_pending_zero = false;
    std::vector<char> slot_used;

    const char* W(int l, size_t off) const { return weights + ((size_t)l * layer_params + off) * esz; }
    float* G(int l, size_t off) const { return grads + (size_t)l * layer_params + off; }
    char* ST(int slot, int l, size_t off) const { return stash + (size_t)slot * slot_bytes + (size_t)l * layer_stash + off; }
};

namespace {

void layout(chimera_stage* st) {
    const size_t H = st->H, M = st->M, e = st->esz;
    size_t o = 0;
    auto take = [&](size_t n) { size_t r = o; o += n; return r; };
    st->o_ln1_g = take(H); st->o_ln1_b = take(H);
    st->o_w_qkv = take(H * 3 * H); st->o_b_qkv = take(3 * H);
    st->o_w_o = take(H * H); st->o_b_o = take(H);
    st->o_ln2_g = take(H); st->o_ln2_b = take(H);
    st->o_w_fc1 = take(H * 4 * H); st->o_b_fc1 = take(4 * H);
    st->o_w_fc2 = take(4 * H * H); st->o_b_fc2 = take(H);
    st->layer_params = o;

    size_t b = 0;
    auto takeb = [&](size_t bytes) { size_t r = b; b += align_up(bytes); return r; };
    st->s_mean1 = takeb(M * 4); st->s_rstd1 = takeb(M * 4);
    st->s_h1 = takeb(M * H * e);
    st->s_qkv = takeb(M * 3 * H * e);
    st->s_ctx = takeb(M * H * e);
    st->s_lse = takeb((size_t)st->B * st->heads * st->S * 4);
    const size_t re = 4;                      // the residual stream between blocks is float in every dtype
    st->s_x1 = takeb(M * H * re);
    st->s_mean2 = takeb(M * 4); st->s_rstd2 = takeb(M * 4);
    st->s_h2 = takeb(M * H * e);
    st->s_u = takeb(M * 4 * H * e);
    st->s_g = takeb(M * 4 * H * e);
    st->s_y = takeb(M * H * re);
    st->layer_stash = b;
    // a forward-only stage keeps nothing: two block areas serve as scratch in turn
    st->slot_bytes = b * (st->keep ? st->L : std::min(st->L, 2));

    b = 0;
    st->w_dy[0] = takeb(M * H * e); st->w_dy[1] = takeb(M * H * e);
    st->w_dyf[0] = takeb(M * H * 4); st->w_dyf[1] = takeb(M * H * 4);
    st->w_dx1f = takeb(M * H * 4);
    st->w_du[0] = takeb(M * 4 * H * e); st->w_du[1] = takeb(M * 4 * H * e);
    st->w_dh = takeb(M * H * e);
    st->w_dx1[0] = takeb(M * H * e); st->w_dx1[1] = takeb(M * H * e);
    st->w_dctx = takeb(M * H * e);
    st->w_dqkv[0] = takeb(M * 3 * H * e); st->w_dqkv[1] = takeb(M * 3 * H * e);
    st->w_delta = takeb((size_t)st->B * st->heads * st->S * 4);
    const size_t sc = std::max(colsum_scratch_floats((int)M, (int)(4 * H)), layernorm_bwd_scratch_floats((int)M, (int)H));
    st->w_scratch = takeb(sc * 4);
    st->w_scratch2 = takeb(sc * 4);
    // partial sums of every LayerNorm backward of a stage pass, reduced by one launch at its end
    st->lnpart_floats = layernorm_bwd_scratch_floats((int)M, (int)H);
    st->w_lnpart = takeb(st->lnpart_floats * 4 * 2 * st->L);
    st->ws_bytes = b;
}

#define TRY(expr) do { int rc__ = (expr); if (rc__) return rc__; } while (0)

int gemm(chimera_stage* st, const GemmArgs& g, int cls, hipStream_t stream) {
    ProfScope prof(cls, 2.0 * g.m * g.n * g.k, stream);
    if (st->dtype == CHIMERA_BF16 && st->kernels == 0 && gemm_mfma_supports(g)) return gemm_mfma_bf16(g, stream);
    return gemm_reference(st->dtype, g, stream);
}

// C[m,n] = X[m,k] W[k,n] (+ epilogue); W stored [in, out].
int linear_fwd(chimera_stage* st, int m, int n, int k, const void* x, const void* w, const void* bias, const void* r,
               void* c, void* c2, int epi, int r_f32 = 0, int c_f32 = 0) {
    GemmArgs g{};
    g.m = m; g.n = n; g.k = k;
    g.a = x; g.lda = k; g.a_kc = 1;
    g.b = w; g.ldb = n; g.b_kc = 0;
    g.bias = bias; g.r = r; g.c = c; g.c2 = c2; g.epilogue = epi; g.gelu_erf = st->gelu_erf;
    g.r_f32 = r_f32; g.c_f32 = c_f32;
    return gemm(st, g, PC_GEMM_FWD, st->stream);
}
// dX[m,k] = dY[m,n] W^T, W stored [k, n]: contraction over n, contiguous in both.
int linear_dgrad(chimera_stage* st, int m, int n, int k, const void* dy, const void* w, const void* r, void* dx, int epi) {
    GemmArgs g{};
    g.m = m; g.n = k; g.k = n;
    g.a = dy; g.lda = n; g.a_kc = 1;
    g.b = w; g.ldb = n; g.b_kc = 1;
    g.r = r; g.c = dx; g.epilogue = epi; g.gelu_erf = st->gelu_erf;
    return gemm(st, g, PC_GEMM_DGRAD, st->stream);
}
// dW[k,n] += X[m,k]^T dY[m,n]: contraction over the tokens.
GemmArgs wgrad_args(int m, int n, int k, const void* x, const void* dy, float* dw) {
    GemmArgs g{};
    g.m = k; g.n = n; g.k = m;
    g.a = x; g.lda = k; g.a_kc = 0;
    g.b = dy; g.ldb = n; g.b_kc = 0;
    g.c = dw; g.epilogue = EPI_ACCUM_F32;
    return g;
}
int linear_wgrad(chimera_stage* st, int m, int n, int k, const void* x, const void* dy, float* dw, hipStream_t stream) {
    return gemm(st, wgrad_args(m, n, k, x, dy, dw), PC_GEMM_WGRAD, stream);
}
// the four weight gradients of one block as one launch (bf16 matrix-core path only)
bool wgrad_group_ok(const chimera_stage* st, const GemmArgs (&g)[4]) {
    return st->dtype == CHIMERA_BF16 && st->kernels == 0 && gemm_mfma_group_supports(4, g);
}
// One or two launches (the second takes the last row bands of one product on smaller tiles),
// each timed as a class of its own so that a class is one kernel.
int wgrad_group(chimera_stage* st, const GemmArgs (&g)[4], float* const (&db)[4], int overwrite, hipStream_t stream) {
    GemmGroupPlan plan;
    TRY(gemm_mfma_group_plan(4, g, &plan));
    double flop = 0;
    for (int i = 0; i < plan.count; ++i) flop += 2.0 * plan.head[i].m * plan.head[i].n * plan.head[i].k;
    {
        ProfScope prof(PC_GEMM_WGRAD, flop, stream);
        TRY(gemm_mfma_group_launch_head(plan, db, overwrite, stream));
    }
    if (!plan.has_tail) return CHIMERA_OK;
    ProfScope prof(PC_GEMM_WGRAD_TAIL, 2.0 * plan.tail.m * plan.tail.n * plan.tail.k, stream);
    return gemm_mfma_group_launch_tail(plan, overwrite, stream);
}

// Performs a zeroing that chimera_stage_zero_grads deferred.
int flush_pending_zero(chimera_stage* st) {
    if (!st->grads_pending_zero) return CHIMERA_OK;
    st->grads_pending_zero = false;
    return fill_zero_f32(st->grads, st->layer_params * st->L, st->stream);
}

int attn_args(chimera_stage* st, AttnArgs& a) {
    a.batch = st->vB; a.seq = st->S; a.heads = st->heads; a.head_dim = st->d; a.causal = st->causal;
    return 0;
}


// useful attention flop: 4 S^2 d per (sequence, head) forward (x 1/2 causal, exactly (S+1)/(2S)), 2x that backward
double attn_flop(const chimera_stage* st) {
    const double c = st->causal ? (st->S + 1.0) / (2.0 * st->S) : 1.0;
    return 4.0 * st->vM * (double)st->S * st->H * c;
}
int st_attn_fwd(chimera_stage* st, const AttnArgs& a) {
    ProfScope prof(PC_ATTN_FWD, attn_flop(st), st->stream);
    if (st->dtype == CHIMERA_BF16 && st->kernels == 0 && attention_mfma_supports(a)) return attention_fwd_mfma(a, st->stream);
    return attention_fwd_reference(st->dtype, a, st->stream);
}
int st_attn_bwd(chimera_stage* st, const AttnArgs& a) {
    ProfScope prof(PC_ATTN_BWD, 2.0 * attn_flop(st), st->stream);
    if (st->dtype == CHIMERA_BF16 && st->kernels == 0 && attention_mfma_supports(a)) return attention_bwd_mfma(a, st->stream);
    return attention_bwd_reference(st->dtype, a, st->stream);
}
// algorithmic bytes of the row-wise kernels: every operand once, at the width it is stored in
int st_ln_fwd(chimera_stage* st, const void* x, int x_f32, const void* g, const void* b, void* y, float* mean, float* rstd) {
    ProfScope prof(PC_LN_FWD, (double)st->vM * st->H * ((x_f32 ? 4 : st->esz) + st->esz), st->stream);
    return layernorm_fwd(st->dtype, st->vM, st->H, x, x_f32, g, b, y, mean, rstd, st->stream);
}
int st_ln_bwd(chimera_stage* st, const void* dy, const void* x, int x_f32, const float* mean, const float* rstd,
              const void* g, const void* res, int res_f32, void* dx_lo, float* dx_hi, float* dg, float* db, float* scratch,
              int overwrite) {
    const double bytes = st->esz + (x_f32 ? 4 : st->esz) + (res_f32 ? 4 : st->esz) + (dx_lo ? st->esz : 0) + (dx_hi ? 4 : 0);
    ProfScope prof(PC_LN_BWD, (double)st->vM * st->H * bytes, st->stream);
    return layernorm_bwd(st->dtype, st->vM, st->H, dy, x, x_f32, mean, rstd, g, res, res_f32, dx_lo, dx_hi, dg, db, scratch,
                         overwrite, st->stream);
}
int st_colsum(chimera_stage* st, int cols, const void* x, float* out, float* scratch, hipStream_t stream) {
    ProfScope prof(PC_COLSUM, (double)st->vM * cols * st->esz, stream);
    return colsum(st->dtype, st->vM, cols, x, out, scratch, stream);
}

#define HIP_TRY(expr) do { hipError_t e__ = (expr); if (e__ != hipSuccess) return fail(CHIMERA_EDEVICE, "%s: %s", #expr, hipGetErrorString(e__)); } while (0)

// side stream waits until the main stream has reached this point
int fork_to_side(chimera_stage* st, int which) {
    if (!st->have_side) return CHIMERA_OK;
    HIP_TRY(hipEventRecord(st->ev_ready[which], st->stream));
    HIP_TRY(hipStreamWaitEvent(st->side, st->ev_ready[which], 0));
    return CHIMERA_OK;
}

// Inside a bf16 stage the residual stream (x -> x1 -> y of every block) stays in
// float: a bf16 stream would be re-rounded at each of the 2L residual additions and
// that random walk, not the matrix products, would dominate the stage's error.
// Only the stage's own input and output are in the stage dtype.
int stage_forward(chimera_stage* st, const chimera_stage::IO& io, int slot) {
    const int M = st->M, H = st->H, L = st->L;
    st->vM = st->M; st->vB = st->B;
    const int wide = st->dtype == CHIMERA_BF16;       // float stream differs from the stage dtype
    for (int l = 0; l < L; ++l) {
        // block area of the stash: one per block, or two used in turn when nothing is kept
        const int la = st->keep ? l : (l & 1), lp = st->keep ? l - 1 : ((l - 1) & 1);
        const void* x = l == 0 ? io.x : st->ST(slot, lp, st->s_y);
        const int x_f32 = wide && l > 0;
        void* y = l == L - 1 ? io.y : st->ST(slot, la, st->s_y);
        const int y_f32 = wide && l < L - 1;
        void* h1 = st->ST(slot, la, st->s_h1);
        void* qkv = st->ST(slot, la, st->s_qkv);
        void* ctx = st->ST(slot, la, st->s_ctx);
        void* x1 = st->ST(slot, la, st->s_x1);
        void* h2 = st->ST(slot, la, st->s_h2);
        void* u = st->ST(slot, la, st->s_u);
        void* g = st->ST(slot, la, st->s_g);
        TRY(st_ln_fwd(st, x, x_f32, st->W(l, st->o_ln1_g), st->W(l, st->o_ln1_b), h1, (float*)st->ST(slot, la, st->s_mean1),
                      (float*)st->ST(slot, la, st->s_rstd1)));
        TRY(linear_fwd(st, M, 3 * H, H, h1, st->W(l, st->o_w_qkv), st->W(l, st->o_b_qkv), nullptr, qkv, nullptr, EPI_BIAS));
        AttnArgs a{};
        attn_args(st, a);
        a.qkv = qkv; a.ctx = ctx; a.lse = (float*)st->ST(slot, la, st->s_lse);
        TRY(st_attn_fwd(st, a));
        TRY(linear_fwd(st, M, H, H, ctx, st->W(l, st->o_w_o), st->W(l, st->o_b_o), x, x1, nullptr, EPI_BIAS_RESIDUAL, x_f32, wide));
        TRY(st_ln_fwd(st, x1, wide, st->W(l, st->o_ln2_g), st->W(l, st->o_ln2_b), h2, (float*)st->ST(slot, la, st->s_mean2),
                      (float*)st->ST(slot, la, st->s_rstd2)));
        TRY(linear_fwd(st, M, 4 * H, H, h2, st->W(l, st->o_w_fc1), st->W(l, st->o_b_fc1), nullptr, u, g, EPI_BIAS_GELU));
        TRY(linear_fwd(st, M, H, 4 * H, g, st->W(l, st->o_w_fc2), st->W(l, st->o_b_fc2), x1, y, nullptr, EPI_BIAS_RESIDUAL, wide, y_f32));
    }
    return CHIMERA_OK;
}

// The gradient of the residual stream is float as well (dy -> dx1 -> dx); each
// LayerNorm backward also writes a copy in the stage dtype, which is what the
// matrix-core products and the bias sums read.
// Rows [row0, row0 + rows) of the micro-batch (whole sequences): the whole of it, or one
// half in a half backward (section 3.5, backward halving).  Every operation of a block acts
// within one sequence, so a part of the rows is an independent backward over the same stash.
int stage_backward(chimera_stage* st, const chimera_stage::IO& io_full, int slot, int row0, int rows) {
    const int M = rows, H = st->H, L = st->L;
    st->vM = rows; st->vB = rows / st->S;
    const size_t e = st->esz, r0 = (size_t)row0;
    auto shift = [&](const void* p, size_t cols, size_t bytes) { return (const void*)((const char*)p + r0 * cols * bytes); };
    chimera_stage::IO io = io_full;
    io.x = shift(io_full.x, H, e); io.dy = shift(io_full.dy, H, e); io.dx = (void*)shift(io_full.dx, H, e);
    const int wide = st->dtype == CHIMERA_BF16;
    // First backward after a deferred zeroing: every gradient is written, not accumulated -
    // possible when all parameter gradients of a block come from kernels that can overwrite
    // (the grouped launch and the LayerNorm reductions); otherwise the fill happens now.
    int fresh = 0;
    if (st->grads_pending_zero) {
        const GemmArgs probe[4] = {wgrad_args(M, H, 4 * H, io.x, io.x, st->grads), wgrad_args(M, 4 * H, H, io.x, io.x, st->grads),
                                   wgrad_args(M, H, H, io.x, io.x, st->grads), wgrad_args(M, 3 * H, H, io.x, io.x, st->grads)};
        if (wgrad_group_ok(st, probe)) { fresh = 1; st->grads_pending_zero = false; }
        else TRY(flush_pending_zero(st));
    }
    float* lnpart = (float*)(st->ws + st->w_lnpart);
    float* scratch2 = (float*)(st->ws + (st->have_side ? st->w_scratch2 : st->w_scratch));
    hipStream_t gs = st->have_side ? st->side : st->stream;       // stream of the parameter gradients
    void* dh = st->ws + st->w_dh;
    float* dx1f = wide ? (float*)(st->ws + st->w_dx1f) : nullptr;
    void* dctx = st->ws + st->w_dctx;
    const void* dy = io.dy;           // stage dtype: operand of the products
    const void* dyr = io.dy;          // what the residual path adds (float inside a bf16 stage)
    int dyr_f32 = 0;
    for (int l = L - 1; l >= 0; --l) {
        const int par = l & 1;
        // du, dx1, dqkv and the dy ping-pong alternate between two buffers by block parity, so
        // before this block overwrites a buffer the side stream must be done with the block
        // two above, which read it
        if (st->have_side && l + 2 <= L - 1) HIP_TRY(hipStreamWaitEvent(st->stream, st->ev_side[par], 0));
        void* du = st->ws + st->w_du[par];
        void* dx1 = st->ws + st->w_dx1[par];
        void* dqkv = st->ws + st->w_dqkv[par];
        const void* x = l == 0 ? io.x : shift(st->ST(slot, l - 1, st->s_y), H, 4);
        const int x_f32 = wide && l > 0;
        void* dx = l == 0 ? io.dx : (void*)(st->ws + st->w_dy[par]);
        float* dxf = (wide && l > 0) ? (float*)(st->ws + st->w_dyf[par]) : nullptr;
        const void* h1 = shift(st->ST(slot, l, st->s_h1), H, e);
        const void* qkv = shift(st->ST(slot, l, st->s_qkv), 3 * H, e);
        const void* ctx = shift(st->ST(slot, l, st->s_ctx), H, e);
        const void* x1 = shift(st->ST(slot, l, st->s_x1), H, 4);
        const void* h2 = shift(st->ST(slot, l, st->s_h2), H, e);
        const void* u = shift(st->ST(slot, l, st->s_u), 4 * H, e);
        const void* g = shift(st->ST(slot, l, st->s_g), 4 * H, e);
        const float* mean1 = (const float*)shift(st->ST(slot, l, st->s_mean1), 1, 4);
        const float* rstd1 = (const float*)shift(st->ST(slot, l, st->s_rstd1), 1, 4);
        const float* mean2 = (const float*)shift(st->ST(slot, l, st->s_mean2), 1, 4);
        const float* rstd2 = (const float*)shift(st->ST(slot, l, st->s_rstd2), 1, 4);
        float* lse = (float*)shift(st->ST(slot, l, st->s_lse), st->heads, 4);       // [sequence, head, position]: heads floats per token
        // With the matrix-core kernels the block's four weight gradients go out as one launch,
        // once the last of their operands (dqkv) exists; otherwise each follows its operands.
        const GemmArgs wg[4] = {wgrad_args(M, H, 4 * H, g, dy, st->G(l, st->o_w_fc2)),
                                wgrad_args(M, 4 * H, H, h2, du, st->G(l, st->o_w_fc1)),
                                wgrad_args(M, H, H, ctx, dx1, st->G(l, st->o_w_o)),
                                wgrad_args(M, 3 * H, H, h1, dqkv, st->G(l, st->o_w_qkv))};
        const bool grouped = wgrad_group_ok(st, wg);
        if (fresh && !grouped) return fail(CHIMERA_ESTATE, "internal: overwrite mode needs the grouped weight gradients");
        // y = x1 + g W2 + b2
        if (!grouped) {
            TRY(fork_to_side(st, 0));
            TRY(st_colsum(st, H, dy, st->G(l, st->o_b_fc2), scratch2, gs));
            TRY(linear_wgrad(st, M, H, 4 * H, g, dy, st->G(l, st->o_w_fc2), gs));
        }
        TRY(linear_dgrad(st, M, H, 4 * H, dy, st->W(l, st->o_w_fc2), u, du, EPI_DGELU));       // du = dg * GeLU'(u)
        // u = h2 W1 + b1
        if (!grouped) {
            TRY(fork_to_side(st, 1));
            TRY(st_colsum(st, 4 * H, du, st->G(l, st->o_b_fc1), scratch2, gs));
            TRY(linear_wgrad(st, M, 4 * H, H, h2, du, st->G(l, st->o_w_fc1), gs));
        }
        TRY(linear_dgrad(st, M, 4 * H, H, du, st->W(l, st->o_w_fc1), nullptr, dh, EPI_NONE));
        TRY(st_ln_bwd(st, dh, x1, wide, mean2, rstd2,
                      st->W(l, st->o_ln2_g), dyr, dyr_f32, dx1, dx1f, nullptr, nullptr, lnpart + (size_t)(2 * l + 1) * st->lnpart_floats, fresh));
        // x1 = x + ctx Wo + bo
        if (!grouped) {
            TRY(fork_to_side(st, 2));
            TRY(st_colsum(st, H, dx1, st->G(l, st->o_b_o), scratch2, gs));
            TRY(linear_wgrad(st, M, H, H, ctx, dx1, st->G(l, st->o_w_o), gs));
        }
        TRY(linear_dgrad(st, M, H, H, dx1, st->W(l, st->o_w_o), nullptr, dctx, EPI_NONE));
        AttnArgs a{};
        attn_args(st, a);
        a.qkv = qkv; a.ctx = (void*)ctx; a.lse = lse;
        a.dctx = dctx; a.dqkv = dqkv; a.delta = (float*)(st->ws + st->w_delta);
        TRY(st_attn_bwd(st, a));
        // qkv = h1 Wqkv + bqkv
        TRY(fork_to_side(st, 3));
        if (grouped) {
            // the bias gradients (column sums of dy, du, dx1, dqkv) come out of the same launch
            float* const db[4] = {st->G(l, st->o_b_fc2), st->G(l, st->o_b_fc1), st->G(l, st->o_b_o), st->G(l, st->o_b_qkv)};
            TRY(wgrad_group(st, wg, db, fresh, gs));
        } else {
            TRY(st_colsum(st, 3 * H, dqkv, st->G(l, st->o_b_qkv), scratch2, gs));
            TRY(linear_wgrad(st, M, 3 * H, H, h1, dqkv, st->G(l, st->o_w_qkv), gs));
        }
        if (st->have_side) HIP_TRY(hipEventRecord(st->ev_side[par], st->side));
        TRY(linear_dgrad(st, M, 3 * H, H, dqkv, st->W(l, st->o_w_qkv), nullptr, dh, EPI_NONE));
        // dx goes into the buffer that the block above read its dy from, also on the side stream
        if (st->have_side && l + 1 <= L - 1) HIP_TRY(hipStreamWaitEvent(st->stream, st->ev_side[(l + 1) & 1], 0));
        TRY(st_ln_bwd(st, dh, x, x_f32, mean1, rstd1,
                      st->W(l, st->o_ln1_g), wide ? (const void*)dx1f : (const void*)dx1, wide, dx, dxf,
                      nullptr, nullptr, lnpart + (size_t)(2 * l) * st->lnpart_floats, fresh));
        dy = dx;
        dyr = dxf ? (const void*)dxf : (const void*)dx;
        dyr_f32 = dxf != nullptr;
    }
    // dgamma, dbeta of all 2L LayerNorms from their partial sums, in one launch
    {
        const LnGradOffsets off{{st->o_ln1_g, st->o_ln2_g}, {st->o_ln1_b, st->o_ln2_b}};
        ProfScope prof(PC_LN_BWD, 0.0, st->stream);
        TRY(layernorm_bwd_reduce(st->dtype, M, H, 2 * L, lnpart, st->lnpart_floats, st->grads, st->layer_params, off, fresh, st->stream));
    }
    // the stash slot, the workspace and the gradient buffers are free for the next op only
    // once the side stream has drained
    if (st->have_side) {
        HIP_TRY(hipStreamWaitEvent(st->stream, st->ev_side[0], 0));
        if (L > 1) HIP_TRY(hipStreamWaitEvent(st->stream, st->ev_side[1], 0));
    }
    return CHIMERA_OK;
}

struct Worker {
    std::vector<chimera_stage*> pipes;        // stage of pipeline p (2f of them; 0 = down, 1 = up)
    chimera_stage* fwd2[2] = {nullptr, nullptr};   // forward-only stages at twice the micro-batch (forward doubling)
    int timing = 0;
    double fwd_ms = 0, bwd_ms = 0;
    int nf = 0, nb = 0;
    double enqueue_ms = 0;                    // host time of the last replay up to its final wait
} g_worker;

}  // namespace

// ----------------------------------------------------------------------- ABI
extern "C" {

const char* chimera_last_error(void) { return g_err; }

chimera_stage* chimera_stage_create(int layers, int hidden, int heads, int seq, int microbatch, int dtype) {
    if (layers < 1 || hidden < 1 || heads < 1 || seq < 1 || microbatch < 1) {
        fail(CHIMERA_EINVAL, "stage sizes must be positive");
        return nullptr;
    }
    if (dtype != CHIMERA_F32 && dtype != CHIMERA_BF16) { fail(CHIMERA_EINVAL, "unknown dtype %d", dtype); return nullptr; }
    if (hidden % heads) { fail(CHIMERA_EINVAL, "hidden=%d is not a multiple of heads=%d", hidden, heads); return nullptr; }
    if (hidden % 8) { fail(CHIMERA_EINVAL, "hidden=%d must be a multiple of 8", hidden); return nullptr; }
    if ((int64_t)seq * microbatch > (1 << 24) || hidden > 4096) { fail(CHIMERA_EINVAL, "stage too large"); return nullptr; }
    chimera_stage* st = new (std::nothrow) chimera_stage();
    if (!st) { fail(CHIMERA_ENOMEM, "out of host memory"); return nullptr; }
    st->L = layers; st->H = hidden; st->heads = heads; st->S = seq; st->B = microbatch; st->dtype = dtype;
    st->M = seq * microbatch; st->d = hidden / heads;
    st->esz = dtype == CHIMERA_F32 ? 4 : 2;
    layout(st);
    return st;
}

int chimera_stage_set_option(chimera_stage* st, int key, int value) {
    if (!st) return fail(CHIMERA_EINVAL, "stage is NULL");
    if (st->bound) return fail(CHIMERA_ESTATE, "options can only be set before chimera_stage_bind");
    switch (key) {
        case CHIMERA_OPT_CAUSAL: if (value != 0 && value != 1) break; st->causal = value; return CHIMERA_OK;
        case CHIMERA_OPT_GELU: if (value != 0 && value != 1) break; st->gelu_erf = value; return CHIMERA_OK;
        case CHIMERA_OPT_KERNELS: if (value != 0 && value != 1) break; st->kernels = value; return CHIMERA_OK;
        case CHIMERA_OPT_OVERLAP: if (value != 0 && value != 1) break; st->overlap = value; return CHIMERA_OK;
        case CHIMERA_OPT_KEEP: if (value != 0 && value != 1) break; st->keep = value; layout(st); return CHIMERA_OK;
        default: return fail(CHIMERA_EINVAL, "unknown option %d", key);
    }
    return fail(CHIMERA_EINVAL, "bad value %d for option %d", value, key);
}

static void drop_side(chimera_stage* st) {
    if (!st->have_side) return;
    (void)hipStreamSynchronize(st->side);
    for (hipEvent_t& e : st->ev_ready) (void)hipEventDestroy(e);
    for (hipEvent_t& e : st->ev_side) (void)hipEventDestroy(e);
    (void)hipStreamDestroy(st->side);
    st->have_side = false;
}

void chimera_stage_destroy(chimera_stage* st) {
    if (!st) return;
    for (chimera_stage*& p : g_worker.pipes) if (p == st) p = nullptr;
    for (chimera_stage*& p : g_worker.fwd2) if (p == st) p = nullptr;
    drop_side(st);
    delete st;
}

size_t chimera_stage_weight_bytes(const chimera_stage* st) { return st ? st->layer_params * st->L * st->esz : 0; }
size_t chimera_stage_grad_bytes(const chimera_stage* st) { return st ? st->layer_params * st->L * sizeof(float) : 0; }
size_t chimera_stage_stash_slot_bytes(const chimera_stage* st) { return st ? st->slot_bytes : 0; }
size_t chimera_stage_workspace_bytes(const chimera_stage* st) { return st ? st->ws_bytes : 0; }

int chimera_stage_bind(chimera_stage* st, const void* d_weights, float* d_grads, void* d_stash, int stash_slots,
                       void* d_workspace, void* hip_stream) {
    if (!st) return fail(CHIMERA_EINVAL, "stage is NULL");
    if (!d_weights || !d_grads || !d_stash || !d_workspace) return fail(CHIMERA_EINVAL, "a device buffer is NULL");
    if (stash_slots < 1) return fail(CHIMERA_EINVAL, "stash_slots=%d must be positive", stash_slots);
    if (((uintptr_t)d_weights | (uintptr_t)d_grads | (uintptr_t)d_stash | (uintptr_t)d_workspace) & 255)
        return fail(CHIMERA_EINVAL, "device buffers must be 256-byte aligned");
    if (!st->in_flight.empty()) return fail(CHIMERA_ESTATE, "cannot rebind with micro-batches in flight");
    st->weights = (const char*)d_weights; st->grads = d_grads; st->stash = (char*)d_stash; st->ws = (char*)d_workspace;
    st->slots = stash_slots; st->stream = (hipStream_t)hip_stream;
    st->grads_pending_zero = false;
    st->slot_used.assign(stash_slots, 0);
    drop_side(st);
    if (st->overlap) {
        // default priority on purpose; non-blocking so that it never syncs with the NULL stream implicitly
        if (hipStreamCreateWithFlags(&st->side, hipStreamNonBlocking) != hipSuccess)
            return fail(CHIMERA_EDEVICE, "cannot create the side stream");
        bool ok = true;
        for (hipEvent_t& e : st->ev_ready) ok = ok && hipEventCreateWithFlags(&e, hipEventDisableTiming) == hipSuccess;
        for (hipEvent_t& e : st->ev_side) ok = ok && hipEventCreateWithFlags(&e, hipEventDisableTiming) == hipSuccess;
        if (!ok) return fail(CHIMERA_EDEVICE, "cannot create events");
        st->have_side = true;
    }
    st->bound = true;
    return CHIMERA_OK;
}

int chimera_stage_set_io(chimera_stage* st, int mb, const void* d_x_in, void* d_y_out, const void* d_dy_in,
                         void* d_dx_out) {
    if (!st) return fail(CHIMERA_EINVAL, "stage is NULL");
    if (mb < 0) return fail(CHIMERA_EINVAL, "micro-batch id %d is negative", mb);
    if (!d_x_in || !d_y_out || !d_dy_in || !d_dx_out) return fail(CHIMERA_EINVAL, "an io buffer is NULL");
    if (((uintptr_t)d_x_in | (uintptr_t)d_y_out | (uintptr_t)d_dy_in | (uintptr_t)d_dx_out) & 15)
        return fail(CHIMERA_EINVAL, "io buffers must be 16-byte aligned");
    if (st->in_flight.count(mb)) return fail(CHIMERA_ESTATE, "micro-batch %d is in flight", mb);
    st->io[mb] = chimera_stage::IO{d_x_in, d_y_out, d_dy_in, d_dx_out};
    return CHIMERA_OK;
}

int chimera_fwd_slot(chimera_stage* st, int mb, int slot) {
    if (!st) return fail(CHIMERA_EINVAL, "stage is NULL");
    if (!st->bound) return fail(CHIMERA_ESTATE, "stage is not bound");
    auto it = st->io.find(mb);
    if (it == st->io.end()) return fail(CHIMERA_ESTATE, "io of micro-batch %d not set", mb);
    if (st->in_flight.count(mb)) return fail(CHIMERA_ESTATE, "forward of micro-batch %d already done", mb);
    if (!st->keep) {
        // nothing is kept: the one scratch slot is free again as soon as the kernels are enqueued
        if (slot > 0) return fail(CHIMERA_ENOMEM, "a forward-only stage has a single scratch slot");
        return stage_forward(st, it->second, 0);
    }
    if (slot < 0) {
        slot = 0;
        while (slot < st->slots && st->slot_used[slot]) ++slot;
        if (slot == st->slots) return fail(CHIMERA_ESTATE, "no free stash slot (%d bound)", st->slots);
    } else if (slot >= st->slots) {
        return fail(CHIMERA_ENOMEM, "stash slot %d requested, %d bound", slot, st->slots);
    } else if (st->slot_used[slot]) {
        return fail(CHIMERA_ESTATE, "stash slot %d is taken", slot);
    }
    int rc = stage_forward(st, it->second, slot);
    if (rc) return rc;
    st->slot_used[slot] = 1;
    st->in_flight[mb] = slot;
    return CHIMERA_OK;
}

int chimera_fwd(chimera_stage* st, int mb) { return chimera_fwd_slot(st, mb, -1); }

int chimera_bwd(chimera_stage* st, int mb) {
    if (!st) return fail(CHIMERA_EINVAL, "stage is NULL");
    if (!st->bound) return fail(CHIMERA_ESTATE, "stage is not bound");
    auto fl = st->in_flight.find(mb);
    if (fl == st->in_flight.end()) return fail(CHIMERA_ESTATE, "backward of micro-batch %d without its forward", mb);
    if (st->halves_done.count(mb)) return fail(CHIMERA_ESTATE, "micro-batch %d is half-way through a halved backward", mb);
    int rc = stage_backward(st, st->io[mb], fl->second, 0, st->M);
    if (rc) return rc;
    st->slot_used[fl->second] = 0;
    st->in_flight.erase(fl);
    return CHIMERA_OK;
}

int chimera_bwd_half(chimera_stage* st, int mb, int half) {
    if (!st) return fail(CHIMERA_EINVAL, "stage is NULL");
    if (!st->bound) return fail(CHIMERA_ESTATE, "stage is not bound");
    if (half != 0 && half != 1) return fail(CHIMERA_EINVAL, "half=%d must be 0 or 1", half);
    if (st->B % 2) return fail(CHIMERA_EINVAL, "a micro-batch of %d sequences cannot be halved", st->B);
    auto fl = st->in_flight.find(mb);
    if (fl == st->in_flight.end()) return fail(CHIMERA_ESTATE, "backward of micro-batch %d without its forward", mb);
    const int done = st->halves_done.count(mb) ? st->halves_done[mb] : 0;
    if (done != half) return fail(CHIMERA_ESTATE, "half %d of micro-batch %d out of order", half, mb);
    int rc = stage_backward(st, st->io[mb], fl->second, half * (st->M / 2), st->M / 2);
    if (rc) return rc;
    if (half == 0) { st->halves_done[mb] = 1; return CHIMERA_OK; }
    st->halves_done.erase(mb);
    st->slot_used[fl->second] = 0;
    st->in_flight.erase(fl);
    return CHIMERA_OK;
}

int chimera_stage_in_flight(const chimera_stage* st) { return st ? (int)st->in_flight.size() : 0; }

int chimera_stage_zero_grads(chimera_stage* st) {
    if (!st) return fail(CHIMERA_EINVAL, "stage is NULL");
    if (!st->bound) return fail(CHIMERA_ESTATE, "stage is not bound");
    st->grads_pending_zero = true;           // performed by the next backward (as overwriting) or reader
    return CHIMERA_OK;
}

int chimera_stage_read_grads(chimera_stage* st, float* h_dst, size_t bytes) {
    if (!st || !h_dst) return fail(CHIMERA_EINVAL, "NULL argument");
    if (!st->bound) return fail(CHIMERA_ESTATE, "stage is not bound");
    if (bytes < chimera_stage_grad_bytes(st)) return fail(CHIMERA_ENOMEM, "destination holds %zu bytes, need %zu", bytes, chimera_stage_grad_bytes(st));
    TRY(flush_pending_zero(st));
    hipError_t e = hipMemcpyAsync(h_dst, st->grads, chimera_stage_grad_bytes(st), hipMemcpyDeviceToHost, st->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(st->stream);
    if (e != hipSuccess) return fail(CHIMERA_EDEVICE, "gradient readback: %s", hipGetErrorString(e));
    return CHIMERA_OK;
}

int chimera_worker_bind_pipes(chimera_stage* const* h_stages, int count) {
    if (!h_stages || count < 1 || count > 64) return fail(CHIMERA_EINVAL, "1..64 stages expected");
    for (int i = 0; i < count; ++i) {
        if (!h_stages[i]) { if (i == 0) return fail(CHIMERA_EINVAL, "stage of pipeline 0 is NULL"); continue; }
        if (!h_stages[i]->bound) return fail(CHIMERA_ESTATE, "stages must be bound first");
        if (!h_stages[i]->keep) return fail(CHIMERA_EINVAL, "a forward-only stage cannot serve a pipeline");
        for (int j = 0; j < i; ++j)
            if (h_stages[j] == h_stages[i]) return fail(CHIMERA_EINVAL, "the stages of a worker must differ");
    }
    g_worker.pipes.assign(h_stages, h_stages + count);
    g_worker.fwd2[0] = g_worker.fwd2[1] = nullptr;
    return CHIMERA_OK;
}

int chimera_worker_bind(chimera_stage* down_stage, chimera_stage* up_stage) {
    if (!down_stage) return fail(CHIMERA_EINVAL, "down stage is NULL");
    if (down_stage == up_stage) return fail(CHIMERA_EINVAL, "down and up stage must differ");
    chimera_stage* both[2] = {down_stage, up_stage};
    return chimera_worker_bind_pipes(both, 2);
}

int chimera_worker_bind_doubling(chimera_stage* down2, chimera_stage* up2) {
    Worker& wk = g_worker;
    if (wk.pipes.size() != 2 || !wk.pipes[0] || !wk.pipes[1]) return fail(CHIMERA_ESTATE, "bind the worker's two stages first");
    chimera_stage* two[2] = {down2, up2};
    for (int p = 0; p < 2; ++p) {
        const chimera_stage* a = wk.pipes[p];
        const chimera_stage* b = two[p];
        if (!b) return fail(CHIMERA_EINVAL, "doubled stage is NULL");
        if (!b->bound) return fail(CHIMERA_ESTATE, "stages must be bound first");
        if (b->keep) return fail(CHIMERA_EINVAL, "the doubled stage must be forward-only (CHIMERA_OPT_KEEP = 0)");
        if (b->L != a->L || b->H != a->H || b->heads != a->heads || b->S != a->S || b->dtype != a->dtype || b->B != 2 * a->B ||
            b->causal != a->causal || b->gelu_erf != a->gelu_erf)
            return fail(CHIMERA_EINVAL, "the doubled stage must have the pipeline stage's shape at twice the micro-batch");
        if (b->weights != a->weights) return fail(CHIMERA_EINVAL, "the doubled stage must be bound to the same weights");
    }
    wk.fwd2[0] = down2; wk.fwd2[1] = up2;
    return CHIMERA_OK;
}

int chimera_worker_set_timing(int on) { g_worker.timing = on ? 1 : 0; return CHIMERA_OK; }

int chimera_run_worker_pipes(int algo, int rank, int D, int N, int f) {
    Worker& wk = g_worker;
    if (wk.pipes.empty() || !wk.pipes[0]) return fail(CHIMERA_ESTATE, "no worker bound");
    const auto t_start = std::chrono::steady_clock::now();
    std::vector<std::vector<Op>> lists;
    TRY(build_schedule(algo, D, N, f, lists));
    if (rank < 0 || rank >= D) return fail(CHIMERA_EINVAL, "rank %d outside [0,%d)", rank, D);
    TRY(annotate(lists, D, N));
    const std::vector<Op>& ops = lists[rank];
    const int pipes = (int)wk.pipes.size();
    std::vector<int> need(pipes, 0);
    bool recompute = false;
    for (const Op& o : ops) {
        if (o.pipe >= pipes || !wk.pipes[o.pipe]) return fail(CHIMERA_ESTATE, "schedule uses pipeline %d but no stage is bound for it", o.pipe);
        need[o.pipe] = std::max(need[o.pipe], o.slot + 1);
        if (o.kind == CHIMERA_OP_F2) recompute = true;
    }
    for (int p = 0; p < pipes; ++p) {
        chimera_stage* st = wk.pipes[p];
        if (!st || (!need[p] && !recompute)) continue;
        // a backward after a doubled forward recomputes into one more slot
        const int slots = need[p] + (recompute ? 1 : 0);
        if (st->slots < slots) return fail(CHIMERA_ENOMEM, "stage of pipeline %d bound with %d stash slots, schedule needs %d", p, st->slots, slots);
        if (!st->in_flight.empty()) return fail(CHIMERA_ESTATE, "stage of pipeline %d has micro-batches in flight", p);
    }
    for (const Op& o : ops) {
        chimera_stage* st = wk.pipes[o.pipe];
        if (o.kind == CHIMERA_OP_F2) {
            if (o.pipe > 1 || !wk.fwd2[o.pipe]) return fail(CHIMERA_ESTATE, "forward doubling needs chimera_worker_bind_doubling");
            if (!wk.fwd2[o.pipe]->io.count(o.mb)) return fail(CHIMERA_ESTATE, "io of micro-batches %d,%d not set on the doubled stage", o.mb, o.mb + 1);
        } else if (!st->io.count(o.mb)) {
            return fail(CHIMERA_ESTATE, "io of micro-batch %d not set on the stage of pipeline %d", o.mb, o.pipe);
        }
        if ((o.kind == CHIMERA_OP_BH0 || o.kind == CHIMERA_OP_BH1) && (st->B % 2))
            return fail(CHIMERA_EINVAL, "a micro-batch of %d sequences cannot be halved", st->B);
    }
    std::vector<hipEvent_t> ev;
    if (wk.timing) {
        ev.resize(ops.size() * 2);
        for (auto& e : ev)
            if (hipEventCreate(&e) != hipSuccess) return fail(CHIMERA_EDEVICE, "hipEventCreate failed");
    }
    int rc = CHIMERA_OK;
    for (size_t i = 0; i < ops.size() && !rc; ++i) {
        const Op& o = ops[i];
        chimera_stage* st = wk.pipes[o.pipe];
        if (wk.timing) (void)hipEventRecord(ev[2 * i], st->stream);
        switch (o.kind) {
            case CHIMERA_OP_F: rc = chimera_fwd_slot(st, o.mb, o.slot); break;
            case CHIMERA_OP_F2: rc = chimera_fwd_slot(wk.fwd2[o.pipe], o.mb, 0); break;
            case CHIMERA_OP_B:
                // after a doubled forward nothing was kept: run the forward again, then the backward
                if (!st->in_flight.count(o.mb)) rc = chimera_fwd_slot(st, o.mb, -1);
                if (!rc) rc = chimera_bwd(st, o.mb);
                break;
            case CHIMERA_OP_BH0: rc = chimera_bwd_half(st, o.mb, 0); break;
            case CHIMERA_OP_BH1: rc = chimera_bwd_half(st, o.mb, 1); break;
            default: rc = fail(CHIMERA_EINVAL, "unknown op kind %d", o.kind);
        }
        if (wk.timing) (void)hipEventRecord(ev[2 * i + 1], st->stream);
    }
    wk.enqueue_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t_start).count();
    // one wait per distinct stream
    hipError_t e = hipSuccess;
    std::vector<hipStream_t> waited;
    auto wait = [&](chimera_stage* st) {
        if (!st || e != hipSuccess) return;
        for (hipStream_t s : waited) if (s == st->stream) return;
        waited.push_back(st->stream);
        e = hipStreamSynchronize(st->stream);
    };
    for (chimera_stage* st : wk.pipes) wait(st);
    for (chimera_stage* st : wk.fwd2) wait(st);
    if (wk.timing) {
        wk.fwd_ms = wk.bwd_ms = 0; wk.nf = wk.nb = 0;
        for (size_t i = 0; i < ops.size(); ++i) {
            float ms = 0.f;
            if (!rc && e == hipSuccess && hipEventElapsedTime(&ms, ev[2 * i], ev[2 * i + 1]) == hipSuccess) {
                if (ops[i].kind == CHIMERA_OP_F || ops[i].kind == CHIMERA_OP_F2) { wk.fwd_ms += ms; ++wk.nf; } else { wk.bwd_ms += ms; ++wk.nb; }
            }
            (void)hipEventDestroy(ev[2 * i]);
            (void)hipEventDestroy(ev[2 * i + 1]);
        }
    }
    if (rc) return rc;
    if (e != hipSuccess) return fail(CHIMERA_EDEVICE, "worker replay: %s", hipGetErrorString(e));
    return CHIMERA_OK;
}

int chimera_run_worker_algo(int algo, int rank, int D, int N) { return chimera_run_worker_pipes(algo, rank, D, N, 1); }

int chimera_run_worker(int rank, int D, int N) { return chimera_run_worker_pipes(CHIMERA_DIRECT, rank, D, N, 1); }

int chimera_worker_last_timing(double* h_fwd_ms, double* h_bwd_ms, int* h_nf, int* h_nb) {
    if (h_fwd_ms) *h_fwd_ms = g_worker.fwd_ms;
    if (h_bwd_ms) *h_bwd_ms = g_worker.bwd_ms;
    if (h_nf) *h_nf = g_worker.nf;
    if (h_nb) *h_nb = g_worker.nb;
    return CHIMERA_OK;
}

int chimera_worker_last_enqueue_ms(double* h_ms) {
    if (!h_ms) return fail(CHIMERA_EINVAL, "h_ms is NULL");
    *h_ms = g_worker.enqueue_ms;
    return CHIMERA_OK;
}

int chimera_profile_enable(int on) {
    if (!g_prof.recs.empty()) prof_collect();
    g_prof.on = on != 0;
    return CHIMERA_OK;
}

int chimera_profile_reset(void) {
    prof_collect();
    for (int c = 0; c < PC_COUNT; ++c) { g_prof.ms[c] = 0; g_prof.work[c] = 0; g_prof.launches[c] = 0; }
    return CHIMERA_OK;
}

int chimera_profile_read(int cls, double* h_ms, long long* h_launches, double* h_work) {
    if (cls < 0 || cls >= PC_COUNT) return fail(CHIMERA_EINVAL, "profile class %d outside [0,%d)", cls, (int)PC_COUNT);
    prof_collect();
    if (h_ms) *h_ms = g_prof.ms[cls];
    if (h_launches) *h_launches = g_prof.launches[cls];
    if (h_work) *h_work = g_prof.work[cls];
    return CHIMERA_OK;
}

// ------------------------------------------------------------ single operators
int chimera_op_gemm(int dtype, int impl, int epilogue, int gelu_kind, int m, int n, int k, const void* d_a, int lda,
                    int a_kc, const void* d_b, int ldb, int b_kc, const void* d_bias, const void* d_r, void* d_c,
                    void* d_c2, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
    if (!d_a || !d_b || !d_c) return fail(CHIMERA_EINVAL, "NULL operand");
    if (m < 1 || n < 1 || k < 1) return fail(CHIMERA_EINVAL, "gemm sizes must be positive");
    if ((k % 8) || (n % 8) || (lda % 8) || (ldb % 8)) return fail(CHIMERA_EINVAL, "k, n, lda, ldb must be multiples of 8");
    if (!a_kc && (m % 8)) return fail(CHIMERA_EINVAL, "m must be a multiple of 8 when A is stored [k, m]");
    if (lda < (a_kc ? k : m) || ldb < (b_kc ? k : n)) return fail(CHIMERA_EINVAL, "leading dimension too small");
    if (epilogue < EPI_NONE || epilogue > EPI_ACCUM_F32) return fail(CHIMERA_EINVAL, "unknown epilogue %d", epilogue);
    if ((epilogue == EPI_BIAS || epilogue == EPI_BIAS_GELU || epilogue == EPI_BIAS_RESIDUAL) && !d_bias)
        return fail(CHIMERA_EINVAL, "epilogue %d needs a bias", epilogue);
    if ((epilogue == EPI_BIAS_RESIDUAL || epilogue == EPI_DGELU) && !d_r) return fail(CHIMERA_EINVAL, "epilogue %d needs R", epilogue);
    if (epilogue == EPI_BIAS_GELU && !d_c2) return fail(CHIMERA_EINVAL, "epilogue %d needs C2", epilogue);
    GemmArgs g{};
    g.m = m; g.n = n; g.k = k; g.a = d_a; g.lda = lda; g.a_kc = a_kc ? 1 : 0; g.b = d_b; g.ldb = ldb; g.b_kc = b_kc ? 1 : 0;
    g.bias = d_bias; g.r = d_r; g.c = d_c; g.c2 = d_c2; g.epilogue = epilogue; g.gelu_erf = gelu_kind ? 1 : 0;
    g.ws = d_workspace; g.ws_bytes = d_workspace ? workspace_bytes : 0;
    if (impl == 0 && dtype == CHIMERA_BF16 && gemm_mfma_supports(g)) return gemm_mfma_bf16(g, hip_stream);
    return gemm_reference(dtype, g, hip_stream);
}

size_t chimera_op_gemm_workspace_bytes(int m, int n, int k) { return gemm_mfma_workspace_need(m, n, k); }

const char* chimera_op_gemm_group_last_kernel(void) { return gemm_mfma_last_group_kernel(); }

int chimera_op_gemm_tuning(int tile_m, int tile_n, int splits, int async_mode) {
    return gemm_mfma_set_tuning(tile_m, tile_n, splits, async_mode);
}

int chimera_op_gemm_group_accumulate(int count, const int* h_m, const int* h_n, int k, const void* const* h_a,
                                     const int* h_lda, const void* const* h_b, const int* h_ldb, float* const* h_c,
                                     float* const* h_bsum, int overwrite, void* hip_stream) {
    if (count < 1 || count > 4) return fail(CHIMERA_EINVAL, "group of %d products (1..4)", count);
    if (!h_m || !h_n || !h_a || !h_lda || !h_b || !h_ldb || !h_c) return fail(CHIMERA_EINVAL, "NULL argument array");
    GemmArgs g[4] = {};
    for (int i = 0; i < count; ++i) {
        if (!h_a[i] || !h_b[i] || !h_c[i]) return fail(CHIMERA_EINVAL, "NULL operand in product %d", i);
        if (h_m[i] < 8 || h_n[i] < 8 || k < 1) return fail(CHIMERA_EINVAL, "product %d: sizes too small", i);
        if (h_lda[i] < h_m[i] || h_ldb[i] < h_n[i]) return fail(CHIMERA_EINVAL, "product %d: leading dimension too small", i);
        g[i].m = h_m[i]; g[i].n = h_n[i]; g[i].k = k;
        g[i].a = h_a[i]; g[i].lda = h_lda[i]; g[i].a_kc = 0;
        g[i].b = h_b[i]; g[i].ldb = h_ldb[i]; g[i].b_kc = 0;
        g[i].c = h_c[i]; g[i].epilogue = EPI_ACCUM_F32;
    }
    return gemm_mfma_bf16_group(count, g, h_bsum, overwrite, hip_stream);
}

int chimera_op_layernorm_fwd(int dtype, int rows, int cols, const void* d_x, const void* d_gamma, const void* d_beta,
                             void* d_y, float* d_mean, float* d_rstd, void* hip_stream) {
    if (!d_x || !d_gamma || !d_beta || !d_y || !d_mean || !d_rstd) return fail(CHIMERA_EINVAL, "NULL operand");
    return layernorm_fwd(dtype, rows, cols, d_x, 0, d_gamma, d_beta, d_y, d_mean, d_rstd, hip_stream);
}

size_t chimera_op_layernorm_bwd_scratch_floats(int rows, int cols) { return layernorm_bwd_scratch_floats(rows, cols); }

int chimera_op_layernorm_bwd(int dtype, int rows, int cols, const void* d_dy, const void* d_x, const float* d_mean,
                             const float* d_rstd, const void* d_gamma, const void* d_res, void* d_dx, float* d_dgamma,
                             float* d_dbeta, float* d_scratch, void* hip_stream) {
    if (!d_dy || !d_x || !d_mean || !d_rstd || !d_gamma || !d_res || !d_dx || !d_dgamma || !d_dbeta || !d_scratch)
        return fail(CHIMERA_EINVAL, "NULL operand");
    return layernorm_bwd(dtype, rows, cols, d_dy, d_x, 0, d_mean, d_rstd, d_gamma, d_res, 0, d_dx, nullptr, d_dgamma, d_dbeta, d_scratch,
                         0, hip_stream);
}

size_t chimera_op_layernorm_bwd_noalloc_max_scratch_floats(void) { return layernorm_bwd_static_scratch_floats(); }

int chimera_op_layernorm_bwd_noalloc(int dtype, int rows, int cols, const void* d_dy, const void* d_x, const float* d_mean,
                                     const float* d_rstd, const void* d_gamma, const void* d_res, void* d_dx,
                                     float* d_dgamma, float* d_dbeta, void* hip_stream) {
    if (!d_dy || !d_x || !d_mean || !d_rstd || !d_gamma || !d_res || !d_dx || !d_dgamma || !d_dbeta)
        return fail(CHIMERA_EINVAL, "NULL operand");
    return layernorm_bwd_noalloc(dtype, rows, cols, d_dy, d_x, d_mean, d_rstd, d_gamma, d_res, d_dx, d_dgamma, d_dbeta, hip_stream);
}

size_t chimera_op_colsum_scratch_floats(int rows, int cols) { return colsum_scratch_floats(rows, cols); }

int chimera_op_colsum(int dtype, int rows, int cols, const void* d_x, float* d_out, float* d_scratch, void* hip_stream) {
    if (!d_x || !d_out || !d_scratch) return fail(CHIMERA_EINVAL, "NULL operand");
    return colsum(dtype, rows, cols, d_x, d_out, d_scratch, hip_stream);
}

int chimera_op_attention_fwd(int dtype, int impl, int batch, int seq, int heads, int head_dim, int causal,
                             const void* d_qkv, void* d_ctx, float* d_lse, void* hip_stream) {
    if (!d_qkv || !d_ctx || !d_lse) return fail(CHIMERA_EINVAL, "NULL operand");
    AttnArgs a{};
    a.batch = batch; a.seq = seq; a.heads = heads; a.head_dim = head_dim; a.causal = causal ? 1 : 0;
    a.qkv = d_qkv; a.ctx = d_ctx; a.lse = d_lse;
    if (impl == 0 && dtype == CHIMERA_BF16 && attention_mfma_supports(a)) return attention_fwd_mfma(a, hip_stream);
    return attention_fwd_reference(dtype, a, hip_stream);
}

int chimera_op_attention_bwd(int dtype, int impl, int batch, int seq, int heads, int head_dim, int causal,
                             const void* d_qkv, const void* d_ctx, const float* d_lse, const void* d_dctx, void* d_dqkv,
                             float* d_delta, void* hip_stream) {
    if (!d_qkv || !d_ctx || !d_lse || !d_dctx || !d_dqkv || !d_delta) return fail(CHIMERA_EINVAL, "NULL operand");
    AttnArgs a{};
    a.batch = batch; a.seq = seq; a.heads = heads; a.head_dim = head_dim; a.causal = causal ? 1 : 0;
    a.qkv = d_qkv; a.ctx = (void*)d_ctx; a.lse = (float*)d_lse; a.dctx = d_dctx; a.dqkv = d_dqkv; a.delta = d_delta;
    if (impl == 0 && dtype == CHIMERA_BF16 && attention_mfma_supports(a)) return attention_bwd_mfma(a, hip_stream);
    return attention_bwd_reference(dtype, a, hip_stream);
}

}  // extern "C"
