// The two ends of the pipeline (section 4.1 of the paper notes that the first stage of a
// language model carries an extra embedding layer; the last stage turns hidden states into a
// loss).  GPT-2 reading:
//   embedding  x[t] = wte[token[t]] + wpe[t mod S]
//   head       h = LayerNorm(y),  z = h W (W stored [H, V]),
//              loss = scale * sum_t (logsumexp(z[t]) - z[t, target[t]])
// with the matching backward.  The matrix products and the LayerNorm are the stage's own
// kernels; this file adds the gather / scatter of the embedding and the fused
// softmax-cross-entropy over a vocabulary row.  No atomics: every sum has a fixed order.
#include "device.h"

#include <algorithm>

namespace chimera {
namespace {

constexpr int EDGE_THREADS = 256;

// ---- embedding forward: one wavefront per token
template <typename T>
__global__ __launch_bounds__(EDGE_THREADS) void embed_fwd_kernel(const int* __restrict__ tokens, const T* __restrict__ wte,
                                                                 const T* __restrict__ wpe, T* __restrict__ x, int M, int S,
                                                                 int H, int vocab) {
    constexpr int V = Elem<T>::VEC;
    const int t = blockIdx.x * (EDGE_THREADS / WAVE) + threadIdx.x / WAVE, lane = threadIdx.x % WAVE;
    if (t >= M) return;
    const int tok = min(max(tokens[t], 0), vocab - 1);         // ids outside the table are clamped, never followed
    const T* a = wte + (size_t)tok * H;
    const T* p = wpe + (size_t)(t % S) * H;
    for (int c = lane; c < H / V; c += WAVE) {
        float u[V], w[V];
        load_vec<T>(a + c * V, u);
        load_vec<T>(p + c * V, w);
#pragma unroll
        for (int e = 0; e < V; ++e) u[e] += w[e];
        store_vec<T>(x + (size_t)t * H + c * V, u);
    }
}

// ---- embedding backward, position table: dwpe[p] += sum over the sequences of dx[b*S + p], b ascending
template <typename T>
__global__ __launch_bounds__(EDGE_THREADS) void embed_bwd_wpe_kernel(const T* __restrict__ dx, float* __restrict__ dwpe, int B,
                                                                     int S, int H) {
    constexpr int V = Elem<T>::VEC;
    const int p = blockIdx.x;
    for (int c = threadIdx.x; c < H / V; c += EDGE_THREADS) {
        float acc[V];
#pragma unroll
        for (int e = 0; e < V; ++e) acc[e] = 0.f;
        for (int b = 0; b < B; ++b) {
            float v[V];
            load_vec<T>(dx + ((size_t)b * S + p) * H + c * V, v);
#pragma unroll
            for (int e = 0; e < V; ++e) acc[e] += v[e];
        }
        float* out = dwpe + (size_t)p * H + c * V;
#pragma unroll
        for (int e = 0; e < V; ++e) out[e] += acc[e];
    }
}

// ---- embedding backward, token table.  One workgroup per position t.  It works only if t is the
// first position that carries its token; it then adds up, in ascending position order, the rows of
// every position with that token and adds the sum to the token's row.  One owner per table row
// and a fixed order of additions: reproducible without atomics or a sort.
template <typename T>
__global__ __launch_bounds__(EDGE_THREADS) void embed_bwd_wte_kernel(const int* __restrict__ tokens, const T* __restrict__ dx,
                                                                     float* __restrict__ dwte, int M, int H, int vocab) {
    constexpr int V = Elem<T>::VEC;
    __shared__ int hit[EDGE_THREADS];
    __shared__ int earlier;
    const int t = blockIdx.x, tid = threadIdx.x;
    const int tok = min(max(tokens[t], 0), vocab - 1);
    if (tid == 0) earlier = 0;
    __syncthreads();
    int seen = 0;
    for (int u = tid; u < t; u += EDGE_THREADS) seen |= min(max(tokens[u], 0), vocab - 1) == tok;
    if (seen) earlier = 1;                                      // benign race: every writer stores 1
    __syncthreads();
    if (earlier) return;                                        // uniform: read after the barrier
    constexpr int MAXC = 2;                                     // chunks of V columns per thread: H <= 2 * 256 * V
    float acc[MAXC][V];
#pragma unroll
    for (int i = 0; i < MAXC; ++i)
#pragma unroll
        for (int e = 0; e < V; ++e) acc[i][e] = 0.f;
    for (int u0 = t - t % EDGE_THREADS; u0 < M; u0 += EDGE_THREADS) {
        const int u = u0 + tid;
        hit[tid] = u >= t && u < M && min(max(tokens[u], 0), vocab - 1) == tok;
        __syncthreads();
        for (int j = 0; j < EDGE_THREADS; ++j) {
            if (!hit[j]) continue;                              // uniform
#pragma unroll
            for (int i = 0; i < MAXC; ++i) {
                const int c = tid + i * EDGE_THREADS;
                if (c < H / V) {
                    float v[V];
                    load_vec<T>(dx + (size_t)(u0 + j) * H + c * V, v);
#pragma unroll
                    for (int e = 0; e < V; ++e) acc[i][e] += v[e];
                }
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        const int c = tid + i * EDGE_THREADS;
        if (c < H / V) {
            float* out = dwte + (size_t)tok * H + c * V;
#pragma unroll
            for (int e = 0; e < V; ++e) out[e] += acc[i][e];
        }
    }
}

// ---- softmax cross-entropy over one vocabulary row per workgroup, in place:
// z[t, :] <- scale * (softmax(z[t, :]) - onehot(target[t])),  loss_rows[t] = scale * (lse - z[t, target]).
// One online pass for the running maximum and sum, one pass to write.
template <typename T>
__global__ __launch_bounds__(EDGE_THREADS) void xent_kernel(T* __restrict__ z, const int* __restrict__ targets,
                                                            float* __restrict__ loss_rows, int vocab, float scale) {
    constexpr int V = Elem<T>::VEC;
    constexpr int NW = EDGE_THREADS / WAVE;
    __shared__ float red_m[NW], red_s[NW];
    const int t = blockIdx.x, tid = threadIdx.x, lane = tid % WAVE, wave = tid / WAVE;
    T* row = z + (size_t)t * vocab;
    const int tgt = min(max(targets[t], 0), vocab - 1);
    float m = -3.0e38f, s = 0.f;
    for (int c = tid; c < vocab / V; c += EDGE_THREADS) {
        float v[V];
        load_vec<T>(row + c * V, v);
        float cm = v[0];
#pragma unroll
        for (int e = 1; e < V; ++e) cm = fmaxf(cm, v[e]);
        const float nm = fmaxf(m, cm);
        float add = 0.f;
#pragma unroll
        for (int e = 0; e < V; ++e) add += expf(v[e] - nm);
        s = s * expf(m - nm) + add;
        m = nm;
    }
    // combine (max, sum) pairs: across the lanes, then across the wavefronts in fixed order
    const float wm = wave_max(m);
    const float ws = wave_sum(s * expf(m - wm));
    if (lane == 0) { red_m[wave] = wm; red_s[wave] = ws; }
    __syncthreads();
    float gm = red_m[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) gm = fmaxf(gm, red_m[w]);
    float gs = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) gs += red_s[w] * expf(red_m[w] - gm);
    const float lse = gm + logf(gs);
    const float inv = 1.0f / gs;
    if (tid == 0) loss_rows[t] = scale * (lse - Elem<T>::to_f(row[tgt]));
    __syncthreads();                                  // the target logit is read before anyone overwrites it
    for (int c = tid; c < vocab / V; c += EDGE_THREADS) {
        float v[V];
        load_vec<T>(row + c * V, v);
#pragma unroll
        for (int e = 0; e < V; ++e) {
            const float p = expf(v[e] - gm) * inv;
            v[e] = scale * (p - ((c * V + e) == tgt ? 1.0f : 0.0f));
        }
        store_vec<T>(row + c * V, v);
    }
}

// loss[0] += sum of loss_rows in a fixed order (one workgroup)
__global__ __launch_bounds__(EDGE_THREADS) void loss_sum_kernel(const float* __restrict__ loss_rows, int n, float* __restrict__ loss) {
    __shared__ float red[EDGE_THREADS];
    float s = 0.f;
    for (int i = threadIdx.x; i < n; i += EDGE_THREADS) s += loss_rows[i];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = EDGE_THREADS / 2; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) loss[0] += red[0];
}

int check_edge(int dtype, int tokens, int seq, int hidden, int vocab, bool vocab_rows_only) {
    if (dtype != CHIMERA_F32 && dtype != CHIMERA_BF16) return fail(CHIMERA_EINVAL, "unknown dtype %d", dtype);
    if (tokens < 1 || seq < 1 || hidden < 1 || vocab < 1) return fail(CHIMERA_EINVAL, "sizes must be positive");
    if (tokens % seq) return fail(CHIMERA_EINVAL, "tokens=%d is not a multiple of seq=%d", tokens, seq);
    // the vocabulary only indexes table rows in the embedding; in the head it is a matrix dimension
    if (hidden % 8 || (!vocab_rows_only && vocab % 8))
        return fail(CHIMERA_EINVAL, "hidden=%d%s must be a multiple of 8", hidden, vocab_rows_only ? "" : " and the vocabulary");
    return CHIMERA_OK;
}

size_t aligned(size_t b) { return (b + 255) / 256 * 256; }

struct HeadLayout { size_t h, mean, rstd, logits, loss_rows, dh, scratch, total; };
HeadLayout head_layout(int dtype, int M, int H, int V) {
    const size_t e = dtype == CHIMERA_F32 ? 4 : 2;
    HeadLayout l{};
    size_t b = 0;
    auto take = [&](size_t bytes) { size_t r = b; b += aligned(bytes); return r; };
    l.h = take((size_t)M * H * e);
    l.mean = take((size_t)M * 4);
    l.rstd = take((size_t)M * 4);
    l.logits = take((size_t)M * V * e);
    l.loss_rows = take((size_t)M * 4);
    l.dh = take((size_t)M * H * e);
    l.scratch = take(layernorm_bwd_scratch_floats(M, H) * 4);
    l.total = b;
    return l;
}

}  // namespace
}  // namespace chimera

using namespace chimera;

#define EDGE_TRY(expr) do { int rc__ = (expr); if (rc__) return rc__; } while (0)

extern "C" {

int chimera_op_embedding_fwd(int dtype, int tokens, int seq, int hidden, int vocab, const int32_t* d_tokens,
                             const void* d_wte, const void* d_wpe, void* d_x, void* hip_stream) {
    EDGE_TRY(check_edge(dtype, tokens, seq, hidden, vocab, true));
    if (!d_tokens || !d_wte || !d_wpe || !d_x) return fail(CHIMERA_EINVAL, "NULL operand");
    if (((uintptr_t)d_wte | (uintptr_t)d_wpe | (uintptr_t)d_x) & 15) return fail(CHIMERA_EINVAL, "buffers must be 16-byte aligned");
    const dim3 grid((tokens + EDGE_THREADS / WAVE - 1) / (EDGE_THREADS / WAVE)), block(EDGE_THREADS);
    hipStream_t s = (hipStream_t)hip_stream;
    if (dtype == CHIMERA_F32)
        hipLaunchKernelGGL(embed_fwd_kernel<float>, grid, block, 0, s, d_tokens, (const float*)d_wte, (const float*)d_wpe,
                           (float*)d_x, tokens, seq, hidden, vocab);
    else
        hipLaunchKernelGGL(embed_fwd_kernel<bf16_t>, grid, block, 0, s, d_tokens, (const bf16_t*)d_wte, (const bf16_t*)d_wpe,
                           (bf16_t*)d_x, tokens, seq, hidden, vocab);
    CHIMERA_LAUNCH_CHECK("embedding forward");
    return CHIMERA_OK;
}

int chimera_op_embedding_bwd(int dtype, int tokens, int seq, int hidden, int vocab, const int32_t* d_tokens, const void* d_dx,
                             float* d_dwte, float* d_dwpe, void* hip_stream) {
    EDGE_TRY(check_edge(dtype, tokens, seq, hidden, vocab, true));
    if (!d_tokens || !d_dx || !d_dwte || !d_dwpe) return fail(CHIMERA_EINVAL, "NULL operand");
    if ((uintptr_t)d_dx & 15) return fail(CHIMERA_EINVAL, "dx must be 16-byte aligned");
    const int vec = dtype == CHIMERA_F32 ? 4 : 8;
    if (hidden / vec > 2 * EDGE_THREADS) return fail(CHIMERA_EINVAL, "hidden=%d too wide for the embedding backward (max %d)", hidden, 2 * EDGE_THREADS * vec);
    hipStream_t s = (hipStream_t)hip_stream;
    if (dtype == CHIMERA_F32) {
        hipLaunchKernelGGL(embed_bwd_wte_kernel<float>, dim3(tokens), dim3(EDGE_THREADS), 0, s, d_tokens, (const float*)d_dx, d_dwte, tokens, hidden, vocab);
        hipLaunchKernelGGL(embed_bwd_wpe_kernel<float>, dim3(seq), dim3(EDGE_THREADS), 0, s, (const float*)d_dx, d_dwpe, tokens / seq, seq, hidden);
    } else {
        hipLaunchKernelGGL(embed_bwd_wte_kernel<bf16_t>, dim3(tokens), dim3(EDGE_THREADS), 0, s, d_tokens, (const bf16_t*)d_dx, d_dwte, tokens, hidden, vocab);
        hipLaunchKernelGGL(embed_bwd_wpe_kernel<bf16_t>, dim3(seq), dim3(EDGE_THREADS), 0, s, (const bf16_t*)d_dx, d_dwpe, tokens / seq, seq, hidden);
    }
    CHIMERA_LAUNCH_CHECK("embedding backward");
    return CHIMERA_OK;
}

int chimera_op_softmax_xent(int dtype, int rows, int vocab, void* d_logits, const int32_t* d_targets, float scale,
                            float* d_loss_rows, float* d_loss, void* hip_stream) {
    if (dtype != CHIMERA_F32 && dtype != CHIMERA_BF16) return fail(CHIMERA_EINVAL, "unknown dtype %d", dtype);
    if (rows < 1 || vocab < 1 || vocab % 8) return fail(CHIMERA_EINVAL, "rows=%d must be positive, vocab=%d a positive multiple of 8", rows, vocab);
    if (!d_logits || !d_targets || !d_loss_rows || !d_loss) return fail(CHIMERA_EINVAL, "NULL operand");
    if ((uintptr_t)d_logits & 15) return fail(CHIMERA_EINVAL, "logits must be 16-byte aligned");
    hipStream_t s = (hipStream_t)hip_stream;
    if (dtype == CHIMERA_F32)
        hipLaunchKernelGGL(xent_kernel<float>, dim3(rows), dim3(EDGE_THREADS), 0, s, (float*)d_logits, d_targets, d_loss_rows, vocab, scale);
    else
        hipLaunchKernelGGL(xent_kernel<bf16_t>, dim3(rows), dim3(EDGE_THREADS), 0, s, (bf16_t*)d_logits, d_targets, d_loss_rows, vocab, scale);
    CHIMERA_LAUNCH_CHECK("softmax cross-entropy");
    hipLaunchKernelGGL(loss_sum_kernel, dim3(1), dim3(EDGE_THREADS), 0, s, d_loss_rows, rows, d_loss);
    CHIMERA_LAUNCH_CHECK("loss sum");
    return CHIMERA_OK;
}

size_t chimera_head_workspace_bytes(int dtype, int tokens, int hidden, int vocab) {
    if (tokens < 1 || hidden < 1 || vocab < 1) return 0;
    return head_layout(dtype, tokens, hidden, vocab).total;
}

int chimera_head_loss(int dtype, int tokens, int hidden, int vocab, const void* d_y, const int32_t* d_targets,
                      const void* d_lnf_g, const void* d_lnf_b, const void* d_w_head, float scale, void* d_dy,
                      float* d_dlnf_g, float* d_dlnf_b, float* d_dw_head, float* d_loss, void* d_workspace,
                      size_t workspace_bytes, void* hip_stream) {
    EDGE_TRY(check_edge(dtype, tokens, 1, hidden, vocab, false));
    if (!d_y || !d_targets || !d_lnf_g || !d_lnf_b || !d_w_head || !d_dy || !d_dlnf_g || !d_dlnf_b || !d_dw_head || !d_loss || !d_workspace)
        return fail(CHIMERA_EINVAL, "NULL operand");
    const HeadLayout l = head_layout(dtype, tokens, hidden, vocab);
    if (workspace_bytes < l.total) return fail(CHIMERA_ENOMEM, "workspace holds %zu bytes, need %zu", workspace_bytes, l.total);
    if (((uintptr_t)d_workspace & 255) || (((uintptr_t)d_y | (uintptr_t)d_dy | (uintptr_t)d_w_head | (uintptr_t)d_dw_head) & 15))
        return fail(CHIMERA_EINVAL, "workspace must be 256-byte aligned, tensors 16-byte aligned");
    const int M = tokens, H = hidden, V = vocab;
    char* ws = (char*)d_workspace;
    void* h = ws + l.h;
    float* mean = (float*)(ws + l.mean);
    float* rstd = (float*)(ws + l.rstd);
    void* logits = ws + l.logits;
    float* loss_rows = (float*)(ws + l.loss_rows);
    void* dh = ws + l.dh;
    float* scratch = (float*)(ws + l.scratch);
    auto gemm = [&](const GemmArgs& g) {
        if (dtype == CHIMERA_BF16 && gemm_mfma_supports(g)) return gemm_mfma_bf16(g, hip_stream);
        return gemm_reference(dtype, g, hip_stream);
    };
    // h = LayerNorm(y)
    EDGE_TRY(layernorm_fwd(dtype, M, H, d_y, 0, d_lnf_g, d_lnf_b, h, mean, rstd, hip_stream));
    // z = h W
    GemmArgs f{};
    f.m = M; f.n = V; f.k = H; f.a = h; f.lda = H; f.a_kc = 1; f.b = d_w_head; f.ldb = V; f.b_kc = 0; f.c = logits; f.epilogue = EPI_NONE;
    EDGE_TRY(gemm(f));
    // loss and dz (in place of z)
    EDGE_TRY(chimera_op_softmax_xent(dtype, M, V, logits, d_targets, scale, loss_rows, d_loss, hip_stream));
    // dh = dz W^T
    GemmArgs d{};
    d.m = M; d.n = H; d.k = V; d.a = logits; d.lda = V; d.a_kc = 1; d.b = d_w_head; d.ldb = V; d.b_kc = 1; d.c = dh; d.epilogue = EPI_NONE;
    EDGE_TRY(gemm(d));
    // dW += h^T dz
    GemmArgs w{};
    w.m = H; w.n = V; w.k = M; w.a = h; w.lda = H; w.a_kc = 0; w.b = logits; w.ldb = V; w.b_kc = 0; w.c = d_dw_head; w.epilogue = EPI_ACCUM_F32;
    EDGE_TRY(gemm(w));
    // dy, dg, db: LayerNorm backward without a residual path
    return layernorm_bwd(dtype, M, H, dh, d_y, 0, mean, rstd, d_lnf_g, nullptr, 0, d_dy, nullptr, d_dlnf_g, d_dlnf_b, scratch, 0, hip_stream);
}

}  // extern "C"
