// Declarations shared by the library's translation units (host side).
#pragma once

#include <cstdarg>
#include <cstddef>
#include <cstdint>
#include <vector>

#include "../../include/chimera.h"

namespace chimera {

using Op = chimera_op;

// Records the message for chimera_last_error() and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

struct ReplayStats {
    int64_t makespan = 0;
    std::vector<int64_t> bubbles;
    std::vector<int32_t> stash_peak;
    int32_t cf = 0, cb = 0;
};
template <typename T> struct ReplayStatsT {
    T makespan = 0;
    std::vector<T> bubbles;
    std::vector<int32_t> stash_peak_halves;      // most activations held, in half micro-batches
    int32_t cf = 0, cb = 0;
};
struct ModelResult { double T, compute, p2p, allreduce, unoverlapped; int c_f, c_b; };

int build_schedule(int algo, int D, int N, std::vector<std::vector<Op>>& lists);
int build_schedule(int algo, int D, int N, int f, std::vector<std::vector<Op>>& lists);
int model_iteration(int algo, int D, int N, int f, int W, double f_t, double b_t, double alpha, double beta,
                    double act_words, double grad_words, int eager, ModelResult* out);
int replay(const std::vector<std::vector<Op>>& lists, int D, int N, int64_t cost_f, int64_t cost_b,
           std::vector<std::vector<int64_t>>& start, ReplayStats* stats);
int annotate(std::vector<std::vector<Op>>& lists, int D, int N);

// ------------------------------------------------------------------ kernels
// Every launcher enqueues on `stream` (a hipStream_t as void*) and returns a
// CHIMERA_* code; shapes are validated here, on the host, before any launch.

enum Epilogue {
    EPI_NONE = 0,           // C = acc
    EPI_BIAS = 1,           // C = acc + bias[n]
    EPI_BIAS_GELU = 2,      // C = acc + bias[n], C2 = GeLU(C)
    EPI_BIAS_RESIDUAL = 3,  // C = acc + bias[n] + R[m,n]
    EPI_DGELU = 4,          // C = acc * GeLU'(R[m,n])
    EPI_ACCUM_F32 = 5       // C (float) += acc
};

struct GemmArgs {
    int m, n, k;
    const void* a; int lda; int a_kc;   // a_kc: A stored [m,k]; else [k,m]
    const void* b; int ldb; int b_kc;   // b_kc: B stored [n,k]; else [k,n]
    const void* bias;                   // [n], stage dtype
    const void* r;                      // [m,n], stage dtype (float if r_f32)
    int r_f32, c_f32;                   // EPI_BIAS_RESIDUAL on bf16 only: R is / C becomes float
    void* c;                            // [m,n]
    void* c2;                           // [m,n]
    int epilogue;
    int gelu_erf;
    void* ws;                           // optional split-K workspace (bf16 matrix-core path), may be null
    size_t ws_bytes;
};

int gemm_reference(int dtype, const GemmArgs& g, void* stream);
int gemm_mfma_bf16(const GemmArgs& g, void* stream);
bool gemm_mfma_supports(const GemmArgs& g);
// `count` float-accumulating products (index-contiguous operands, one contraction length) in one launch;
// bsum (may be null, entries may be null): bsum[p][j] += sum_k B_p(k, j), the bias gradient of a linear layer;
// overwrite != 0: C_p and bsum_p receive the results instead of accumulating them
bool gemm_mfma_group_supports(int count, const GemmArgs* g);
int gemm_mfma_bf16_group(int count, const GemmArgs* g, float* const* bsum, int overwrite, void* stream);
// The same in steps, for callers that time the kernels one by one: the plan says which tile the
// group takes and whether the last row bands of one product (`tail`, product `tail_of`) leave as a
// second launch of 128x128 tiles; `head` holds the products of the first launch.
struct GemmGroupPlan { GemmArgs head[4]; GemmArgs tail; int count, tile, has_tail, tail_of; };
int gemm_mfma_group_plan(int count, const GemmArgs* g, GemmGroupPlan* plan);
int gemm_mfma_group_launch_head(const GemmGroupPlan& plan, float* const* bsum, int overwrite, void* stream);
int gemm_mfma_group_launch_tail(const GemmGroupPlan& plan, int overwrite, void* stream);
int gemm_mfma_set_tuning(int bm, int bn, int splits, int async_mode);
const char* gemm_mfma_last_group_kernel();   // instantiation(s) of the last grouped launch on this thread
size_t gemm_mfma_workspace_bytes(int m, int n, int splits);
size_t gemm_mfma_workspace_need(int m, int n, int k);   // bytes the tile heuristic wants for this shape (0 = none)

// x_f32 / res_f32: that operand is float although the stage dtype is bf16 (the
// residual stream inside a bf16 stage is kept in float).  dx_lo (stage dtype) and
// dx_hi (float) may each be null, not both.
int layernorm_fwd(int dtype, int rows, int cols, const void* x, int x_f32, const void* gamma, const void* beta,
                  void* y, float* mean, float* rstd, void* stream);
size_t layernorm_bwd_scratch_floats(int rows, int cols);
int layernorm_bwd(int dtype, int rows, int cols, const void* dy, const void* x, int x_f32, const float* mean,
                  const float* rstd, const void* gamma, const void* res, int res_f32, void* dx_lo, float* dx_hi,
                  float* dgamma, float* dbeta, float* scratch, int overwrite, void* stream);
// The same with the partial sums in the library's static device array (no workspace argument, no allocation);
// ENOMEM when layernorm_bwd_scratch_floats(rows, cols) exceeds layernorm_bwd_static_scratch_floats().
size_t layernorm_bwd_static_scratch_floats();
int layernorm_bwd_noalloc(int dtype, int rows, int cols, const void* dy, const void* x, const float* mean, const float* rstd,
                          const void* gamma, const void* res, void* dx, float* dgamma, float* dbeta, void* stream);
// dgamma == nullptr: the per-block partial sums stay in `scratch` ([blocks][dgamma | dbeta], the
// size layernorm_bwd_scratch_floats gives) and layernorm_bwd_reduce finishes `count` such passes
// of equal shape and element type `dtype` in one launch: pass y, at partial + y * part_stride, belongs to LayerNorm y & 1
// of layer y >> 1, whose gradients lie at grads + layer * layer_stride + off.gamma / off.beta.
struct LnGradOffsets { size_t gamma[2], beta[2]; };
int layernorm_bwd_reduce(int dtype, int rows, int cols, int count, const float* partial, size_t part_stride, float* grads,
                         size_t layer_stride, const LnGradOffsets& off, int overwrite, void* stream);
size_t colsum_scratch_floats(int rows, int cols);
int colsum(int dtype, int rows, int cols, const void* x, float* out, float* scratch, void* stream);
int fill_zero_f32(float* p, size_t n, void* stream);

struct AttnArgs {
    int batch, seq, heads, head_dim, causal;
    const void* qkv;      // [M, 3H]
    void* ctx;            // fwd out / bwd in [M, H]
    float* lse;           // [batch, heads, seq]
    const void* dctx;     // bwd [M, H]
    void* dqkv;           // bwd [M, 3H]
    float* delta;         // bwd scratch [batch, heads, seq]
};
int attention_fwd_reference(int dtype, const AttnArgs& a, void* stream);
int attention_bwd_reference(int dtype, const AttnArgs& a, void* stream);
bool attention_mfma_supports(const AttnArgs& a);
int attention_fwd_mfma(const AttnArgs& a, void* stream);
int attention_bwd_mfma(const AttnArgs& a, void* stream);

}  // namespace chimera
