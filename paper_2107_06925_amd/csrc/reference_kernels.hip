// Plain kernels for GEMM and attention: any shape, float or bf16 storage,
// float arithmetic on the vector ALUs.  They carry the fp32 workload and every
// shape the matrix-core kernels do not take, and they are what the matrix-core
// kernels can be switched out for (CHIMERA_OPT_KERNELS = 1).
#include "device.h"

namespace chimera {

namespace {

// ---------------------------------------------------------------------- GEMM
// 64x64 output tile per 256-thread block, 4x4 outputs per thread, k step 16.
constexpr int RT = 64, RK = 16;

template <typename T>
__device__ __forceinline__ void epilogue_scalar(const GemmArgs& g, int row, int col, float acc) {
    const size_t idx = (size_t)row * g.n + col;
    switch (g.epilogue) {
        case EPI_NONE: ((T*)g.c)[idx] = Elem<T>::from_f(acc); break;
        case EPI_BIAS: ((T*)g.c)[idx] = Elem<T>::from_f(acc + Elem<T>::to_f(((const T*)g.bias)[col])); break;
        case EPI_BIAS_GELU: {
            const float u = acc + Elem<T>::to_f(((const T*)g.bias)[col]);
            ((T*)g.c)[idx] = Elem<T>::from_f(u);
            ((T*)g.c2)[idx] = Elem<T>::from_f(gelu_f(u, g.gelu_erf));
            break;
        }
        case EPI_BIAS_RESIDUAL: {
            const float rv = g.r_f32 ? ((const float*)g.r)[idx] : Elem<T>::to_f(((const T*)g.r)[idx]);
            const float v = acc + Elem<T>::to_f(((const T*)g.bias)[col]) + rv;
            if (g.c_f32) ((float*)g.c)[idx] = v; else ((T*)g.c)[idx] = Elem<T>::from_f(v);
            break;
        }
        case EPI_DGELU:
            ((T*)g.c)[idx] = Elem<T>::from_f(acc * gelu_grad_f(Elem<T>::to_f(((const T*)g.r)[idx]), g.gelu_erf));
            break;
        case EPI_ACCUM_F32: ((float*)g.c)[idx] += acc; break;
    }
}

template <typename T>
__global__ __launch_bounds__(256) void gemm_ref_kernel(GemmArgs g) {
    __shared__ float As[RK][RT + 1], Bs[RK][RT + 1];
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    const int i0 = blockIdx.y * RT, j0 = blockIdx.x * RT;
    const T* A = (const T*)g.a;
    const T* B = (const T*)g.b;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < g.k; k0 += RK) {
        for (int e = threadIdx.x; e < RT * RK; e += 256) {
            int i, kk;
            if (g.a_kc) { kk = e % RK; i = e / RK; } else { i = e % RT; kk = e / RT; }
            float v = 0.f;
            if (i0 + i < g.m && k0 + kk < g.k)
                v = Elem<T>::to_f(g.a_kc ? A[(size_t)(i0 + i) * g.lda + k0 + kk] : A[(size_t)(k0 + kk) * g.lda + i0 + i]);
            As[kk][i] = v;
            int j;
            if (g.b_kc) { kk = e % RK; j = e / RK; } else { j = e % RT; kk = e / RT; }
            v = 0.f;
            if (j0 + j < g.n && k0 + kk < g.k)
                v = Elem<T>::to_f(g.b_kc ? B[(size_t)(j0 + j) * g.ldb + k0 + kk] : B[(size_t)(k0 + kk) * g.ldb + j0 + j]);
            Bs[kk][j] = v;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < RK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) { a[r] = As[kk][ty * 4 + r]; b[r] = Bs[kk][tx * 4 + r]; }
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[r][c] += a[r] * b[c];
        }
        __syncthreads();
    }
    for (int r = 0; r < 4; ++r)
        for (int c = 0; c < 4; ++c) {
            const int row = i0 + ty * 4 + r, col = j0 + tx * 4 + c;
            if (row < g.m && col < g.n) epilogue_scalar<T>(g, row, col, acc[r][c]);
        }
}

// ----------------------------------------------------------------- attention
// One wavefront per (query | key) row.  Scores of the row are staged in LDS.
// Token t = b*seq + s; q, k, v of head h start at columns h*d, H + h*d, 2H + h*d.
template <typename T>
__global__ __launch_bounds__(WAVE) void attn_fwd_ref_kernel(AttnArgs a) {
    extern __shared__ float sm[];
    const int S = a.seq, d = a.head_dim, H = a.heads * d;
    float* ps = sm;          // [S]
    float* qs = sm + S;      // [d]
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const T* base = (const T*)a.qkv + (size_t)b * S * 3 * H + h * d;
    const float scale = 1.0f / sqrtf((float)d);
    for (int t = lane; t < d; t += WAVE) qs[t] = Elem<T>::to_f(base[(size_t)i * 3 * H + t]);
    __syncthreads();
    const int n = a.causal ? i + 1 : S;
    float mx = -INFINITY;
    for (int j = lane; j < n; j += WAVE) {
        const T* kr = base + (size_t)j * 3 * H + H;
        float s = 0.f;
        for (int t = 0; t < d; ++t) s += qs[t] * Elem<T>::to_f(kr[t]);
        s *= scale;
        ps[j] = s;
        mx = fmaxf(mx, s);
    }
    mx = wave_max(mx);
    float sum = 0.f;
    for (int j = lane; j < n; j += WAVE) {
        const float e = expf(ps[j] - mx);
        ps[j] = e;
        sum += e;
    }
    sum = wave_sum(sum);
    __syncthreads();
    T* out = (T*)a.ctx + ((size_t)b * S + i) * H + h * d;
    for (int t = lane; t < d; t += WAVE) {
        float o = 0.f;
        for (int j = 0; j < n; ++j) o += ps[j] * Elem<T>::to_f(base[(size_t)j * 3 * H + 2 * H + t]);
        out[t] = Elem<T>::from_f(o / sum);
    }
    if (lane == 0) a.lse[((size_t)b * a.heads + h) * S + i] = mx + logf(sum);
}

// dq of one query row; also delta = sum_t dctx * ctx of that row.
template <typename T>
__global__ __launch_bounds__(WAVE) void attn_bwd_dq_ref_kernel(AttnArgs a) {
    extern __shared__ float sm[];
    const int S = a.seq, d = a.head_dim, H = a.heads * d;
    float* ds = sm;             // [S]
    float* qs = sm + S;         // [d]
    float* dos = sm + S + d;    // [d]
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const T* base = (const T*)a.qkv + (size_t)b * S * 3 * H + h * d;
    const T* dor = (const T*)a.dctx + ((size_t)b * S + i) * H + h * d;
    const T* orow = (const T*)a.ctx + ((size_t)b * S + i) * H + h * d;
    const float scale = 1.0f / sqrtf((float)d);
    float dl = 0.f;
    for (int t = lane; t < d; t += WAVE) {
        qs[t] = Elem<T>::to_f(base[(size_t)i * 3 * H + t]);
        dos[t] = Elem<T>::to_f(dor[t]);
        dl += dos[t] * Elem<T>::to_f(orow[t]);
    }
    dl = wave_sum(dl);
    const size_t li = ((size_t)b * a.heads + h) * S + i;
    if (lane == 0) a.delta[li] = dl;
    const float lse = a.lse[li];
    __syncthreads();
    const int n = a.causal ? i + 1 : S;
    for (int j = lane; j < n; j += WAVE) {
        const T* kr = base + (size_t)j * 3 * H + H;
        const T* vr = base + (size_t)j * 3 * H + 2 * H;
        float s = 0.f, dp = 0.f;
        for (int t = 0; t < d; ++t) { s += qs[t] * Elem<T>::to_f(kr[t]); dp += dos[t] * Elem<T>::to_f(vr[t]); }
        ds[j] = expf(s * scale - lse) * (dp - dl);
    }
    __syncthreads();
    T* out = (T*)a.dqkv + ((size_t)b * S + i) * 3 * H + h * d;
    for (int t = lane; t < d; t += WAVE) {
        float o = 0.f;
        for (int j = 0; j < n; ++j) o += ds[j] * Elem<T>::to_f(base[(size_t)j * 3 * H + H + t]);
        out[t] = Elem<T>::from_f(o * scale);
    }
}

// dk, dv of one key row (needs delta from the dq kernel).
template <typename T>
__global__ __launch_bounds__(WAVE) void attn_bwd_dkv_ref_kernel(AttnArgs a) {
    extern __shared__ float sm[];
    const int S = a.seq, d = a.head_dim, H = a.heads * d;
    float* ps = sm;                 // [S]
    float* dss = sm + S;            // [S]
    float* ks = sm + 2 * S;         // [d]
    float* vs = sm + 2 * S + d;     // [d]
    const int j = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const T* base = (const T*)a.qkv + (size_t)b * S * 3 * H + h * d;
    const T* dob = (const T*)a.dctx + (size_t)b * S * H + h * d;
    const float scale = 1.0f / sqrtf((float)d);
    for (int t = lane; t < d; t += WAVE) {
        ks[t] = Elem<T>::to_f(base[(size_t)j * 3 * H + H + t]);
        vs[t] = Elem<T>::to_f(base[(size_t)j * 3 * H + 2 * H + t]);
    }
    __syncthreads();
    const int first = a.causal ? j : 0;
    const size_t l0 = ((size_t)b * a.heads + h) * S;
    for (int i = first + lane; i < S; i += WAVE) {
        const T* qr = base + (size_t)i * 3 * H;
        const T* dor = dob + (size_t)i * H;
        float s = 0.f, dp = 0.f;
        for (int t = 0; t < d; ++t) { s += Elem<T>::to_f(qr[t]) * ks[t]; dp += Elem<T>::to_f(dor[t]) * vs[t]; }
        const float p = expf(s * scale - a.lse[l0 + i]);
        ps[i] = p;
        dss[i] = p * (dp - a.delta[l0 + i]);
    }
    __syncthreads();
    T* out = (T*)a.dqkv + ((size_t)b * S + j) * 3 * H + h * d;
    for (int t = lane; t < d; t += WAVE) {
        float dk = 0.f, dv = 0.f;
        for (int i = first; i < S; ++i) {
            dk += dss[i] * Elem<T>::to_f(base[(size_t)i * 3 * H + t]);
            dv += ps[i] * Elem<T>::to_f(dob[(size_t)i * H + t]);
        }
        out[H + t] = Elem<T>::from_f(dk * scale);
        out[2 * H + t] = Elem<T>::from_f(dv);
    }
}

int check_attn(int dtype, const AttnArgs& a) {
    if (dtype != CHIMERA_F32 && dtype != CHIMERA_BF16) return fail(CHIMERA_EINVAL, "unknown dtype %d", dtype);
    if (a.batch < 1 || a.seq < 1 || a.heads < 1 || a.head_dim < 1)
        return fail(CHIMERA_EINVAL, "attention sizes must be positive");
    if (a.batch > 65535 || a.heads > 65535) return fail(CHIMERA_EINVAL, "batch and heads must be below 65536");
    if ((size_t)(2 * a.seq + 2 * a.head_dim) * sizeof(float) > 64 * 1024)
        return fail(CHIMERA_EINVAL, "reference attention: seq=%d too long", a.seq);
    return CHIMERA_OK;
}

}  // namespace

int gemm_reference(int dtype, const GemmArgs& g, void* stream) {
    if (dtype != CHIMERA_F32 && dtype != CHIMERA_BF16) return fail(CHIMERA_EINVAL, "unknown dtype %d", dtype);
    if (g.m < 1 || g.n < 1 || g.k < 1) return fail(CHIMERA_EINVAL, "gemm sizes must be positive");
    if (g.epilogue < EPI_NONE || g.epilogue > EPI_ACCUM_F32) return fail(CHIMERA_EINVAL, "unknown epilogue %d", g.epilogue);
    const dim3 grid((g.n + RT - 1) / RT, (g.m + RT - 1) / RT);
    if (grid.y > 65535) return fail(CHIMERA_EINVAL, "gemm m=%d too large for the reference kernel", g.m);
    if (dtype == CHIMERA_F32) hipLaunchKernelGGL(gemm_ref_kernel<float>, grid, dim3(256), 0, (hipStream_t)stream, g);
    else hipLaunchKernelGGL(gemm_ref_kernel<bf16_t>, grid, dim3(256), 0, (hipStream_t)stream, g);
    CHIMERA_LAUNCH_CHECK("reference gemm");
    return CHIMERA_OK;
}

int attention_fwd_reference(int dtype, const AttnArgs& a, void* stream) {
    if (int rc = check_attn(dtype, a)) return rc;
    const dim3 grid(a.seq, a.heads, a.batch);
    const size_t lds = (size_t)(a.seq + a.head_dim) * sizeof(float);
    if (dtype == CHIMERA_F32) hipLaunchKernelGGL(attn_fwd_ref_kernel<float>, grid, dim3(WAVE), lds, (hipStream_t)stream, a);
    else hipLaunchKernelGGL(attn_fwd_ref_kernel<bf16_t>, grid, dim3(WAVE), lds, (hipStream_t)stream, a);
    CHIMERA_LAUNCH_CHECK("reference attention forward");
    return CHIMERA_OK;
}

int attention_bwd_reference(int dtype, const AttnArgs& a, void* stream) {
    if (int rc = check_attn(dtype, a)) return rc;
    const dim3 grid(a.seq, a.heads, a.batch);
    const size_t lds1 = (size_t)(a.seq + 2 * a.head_dim) * sizeof(float);
    const size_t lds2 = (size_t)(2 * a.seq + 2 * a.head_dim) * sizeof(float);
    hipStream_t s = (hipStream_t)stream;
    if (dtype == CHIMERA_F32) {
        hipLaunchKernelGGL(attn_bwd_dq_ref_kernel<float>, grid, dim3(WAVE), lds1, s, a);
        hipLaunchKernelGGL(attn_bwd_dkv_ref_kernel<float>, grid, dim3(WAVE), lds2, s, a);
    } else {
        hipLaunchKernelGGL(attn_bwd_dq_ref_kernel<bf16_t>, grid, dim3(WAVE), lds1, s, a);
        hipLaunchKernelGGL(attn_bwd_dkv_ref_kernel<bf16_t>, grid, dim3(WAVE), lds2, s, a);
    }
    CHIMERA_LAUNCH_CHECK("reference attention backward");
    return CHIMERA_OK;
}

}  // namespace chimera
