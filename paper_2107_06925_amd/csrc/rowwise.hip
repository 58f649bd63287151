// HBM-bound kernels of a Transformer block: LayerNorm forward and backward,
// column sums (bias gradients), partial-sum reduction and fill.  One 64-lane
// wavefront owns a row; every access is a 16-byte vector, lanes side by side,
// so a wavefront reads 1 KiB contiguous per step.  Column reductions are
// two-phase (per-block partials, then a fixed-order sum) so that results do
// not depend on scheduling.
#include "device.h"

#include <mutex>

// Scratch of chimera_op_layernorm_bwd_noalloc: the per-block partial sums of dgamma and
// dbeta, held by every GPU the library runs on until the process ends.  Host code never
// uses this name as an address; it asks the runtime for the array's device address once
// per device (static_scratch below).
constexpr size_t LN_STATIC_SCRATCH_FLOATS = (size_t)4 << 20;        // 16 MiB
static __device__ __align__(256) float scratch[LN_STATIC_SCRATCH_FLOATS];

namespace chimera {

namespace {

constexpr int LN_WAVES = 4;        // wavefronts (rows in flight) per block
constexpr int LNB_ROWS = 8;        // rows per block in the LayerNorm backward
constexpr int CS_ROWS = 64;        // rows per block in the column sum

// ------------------------------------------------------------- LayerNorm fwd
// y = (x - mean) * rstd * gamma + beta, biased variance, eps 1e-5.
// T chunks per lane are kept in registers between the passes.
template <typename TX, typename T, int MAXT>
__global__ __launch_bounds__(LN_WAVES* WAVE) void ln_fwd_kernel(const TX* __restrict__ x, const T* __restrict__ gamma,
                                                                const T* __restrict__ beta, T* __restrict__ y,
                                                                float* __restrict__ mean, float* __restrict__ rstd,
                                                                int rows, int cols) {
    constexpr int V = Elem<T>::VEC;
    const int lane = threadIdx.x % WAVE;
    const int row = blockIdx.x * LN_WAVES + threadIdx.x / WAVE;
    if (row >= rows) return;
    const int nchunk = cols / V;
    const TX* xr = x + (size_t)row * cols;
    float v[MAXT][V];
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < MAXT; ++t) {
        const int c = lane + t * WAVE;
        if (c < nchunk) {
            load_elems<TX, V>(xr + c * V, v[t]);
#pragma unroll
            for (int e = 0; e < V; ++e) s += v[t][e];
        }
    }
    const float mu = wave_sum(s) / (float)cols;
    float q = 0.f;
#pragma unroll
    for (int t = 0; t < MAXT; ++t) {
        const int c = lane + t * WAVE;
        if (c < nchunk) {
#pragma unroll
            for (int e = 0; e < V; ++e) { const float d = v[t][e] - mu; q += d * d; }
        }
    }
    const float rs = 1.0f / sqrtf(wave_sum(q) / (float)cols + LN_EPS);
    if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
    T* yr = y + (size_t)row * cols;
#pragma unroll
    for (int t = 0; t < MAXT; ++t) {
        const int c = lane + t * WAVE;
        if (c < nchunk) {
            float g[V], b[V], o[V];
            load_vec<T>(gamma + c * V, g);
            load_vec<T>(beta + c * V, b);
#pragma unroll
            for (int e = 0; e < V; ++e) o[e] = (v[t][e] - mu) * rs * g[e] + b[e];
            store_vec<T>(yr + c * V, o);
        }
    }
}

// ------------------------------------------------------------- LayerNorm bwd
// With xhat = (x - mean) rstd and dxhat = dy * gamma:
//   dx = res + rstd * (dxhat - mean_c(dxhat) - xhat * mean_c(dxhat * xhat))
//   dgamma += sum_rows dy * xhat,  dbeta += sum_rows dy.
// A block takes LNB_ROWS rows; every lane owns fixed columns, so the column
// sums accumulate in registers, are combined over the block's wavefronts in
// LDS in a fixed order and leave as one partial row per block:
// partial[block][0][cols] = dgamma part, partial[block][1][cols] = dbeta part.
// x may be float while dy is bf16 (TX), the residual gradient likewise (TR); dx is
// written as T (dx_lo, may be null) and/or as float (dx_hi, may be null).
template <typename TX, typename TR, typename T, int MAXT>
__global__ __launch_bounds__(LN_WAVES* WAVE) void ln_bwd_kernel(const T* __restrict__ dy, const TX* __restrict__ x,
                                                                const float* __restrict__ mean,
                                                                const float* __restrict__ rstd,
                                                                const T* __restrict__ gamma, const TR* __restrict__ res,
                                                                T* __restrict__ dx_lo, float* __restrict__ dx_hi,
                                                                float* __restrict__ partial, int rows, int cols) {
    constexpr int V = Elem<T>::VEC;
    extern __shared__ float red[];   // [LN_WAVES][2][cols]
    const int lane = threadIdx.x % WAVE, wave = threadIdx.x / WAVE;
    const int nchunk = cols / V;
    float ag[MAXT][V], ab[MAXT][V], g[MAXT][V];
#pragma unroll
    for (int t = 0; t < MAXT; ++t) {
        const int c = lane + t * WAVE;
#pragma unroll
        for (int e = 0; e < V; ++e) { ag[t][e] = 0.f; ab[t][e] = 0.f; g[t][e] = 0.f; }
        if (c < nchunk) load_vec<T>(gamma + c * V, g[t]);
    }
    const int row0 = blockIdx.x * LNB_ROWS;
#pragma unroll
    for (int rr = 0; rr < LNB_ROWS / LN_WAVES; ++rr) {   // unrolled: the rows of a wavefront are independent
        const int row = row0 + wave + rr * LN_WAVES;
        if (row >= rows) continue;
        const float mu = mean[row], rs = rstd[row];
        float dxh[MAXT][V], xh[MAXT][V];
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int t = 0; t < MAXT; ++t) {
            const int c = lane + t * WAVE;
            if (c < nchunk) {
                float d[V], xv[V];
                load_vec<T>(dy + (size_t)row * cols + c * V, d);
                load_elems<TX, V>(x + (size_t)row * cols + c * V, xv);
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    xh[t][e] = (xv[e] - mu) * rs;
                    dxh[t][e] = d[e] * g[t][e];
                    s1 += dxh[t][e];
                    s2 += dxh[t][e] * xh[t][e];
                    ag[t][e] += d[e] * xh[t][e];
                    ab[t][e] += d[e];
                }
            }
        }
        const float m1 = wave_sum(s1) / (float)cols;
        const float m2 = wave_sum(s2) / (float)cols;
#pragma unroll
        for (int t = 0; t < MAXT; ++t) {
            const int c = lane + t * WAVE;
            if (c < nchunk) {
                float rv[V], o[V];
                if (res) load_elems<TR, V>(res + (size_t)row * cols + c * V, rv);       // no residual path: dx = LN'(dy)
                else
#pragma unroll
                    for (int e = 0; e < V; ++e) rv[e] = 0.f;
#pragma unroll
                for (int e = 0; e < V; ++e) o[e] = rv[e] + rs * (dxh[t][e] - m1 - xh[t][e] * m2);
                if (dx_lo) store_vec<T>(dx_lo + (size_t)row * cols + c * V, o);
                if (dx_hi) store_elems<float, V>(dx_hi + (size_t)row * cols + c * V, o);
            }
        }
    }
    // Fixed-order combination over the wavefronts of the block: every wavefront parks its sums
    // in its own LDS rows (16-byte stores), one barrier, then each thread adds the LN_WAVES
    // values of its columns in wavefront order and writes the block's partial row.
    float* mine = red + (size_t)wave * 2 * cols;
#pragma unroll
    for (int t = 0; t < MAXT; ++t) {
        const int c = lane + t * WAVE;
        if (c < nchunk) {
            store_elems<float, V>(mine + c * V, ag[t]);
            store_elems<float, V>(mine + cols + c * V, ab[t]);
        }
    }
    __syncthreads();
    float* out = partial + (size_t)blockIdx.x * 2 * cols;
    for (int i = threadIdx.x * 4; i < 2 * cols; i += LN_WAVES * WAVE * 4) {
        float4 acc = *reinterpret_cast<const float4*>(red + i);
#pragma unroll
        for (int w = 1; w < LN_WAVES; ++w) {
            const float4 v = *reinterpret_cast<const float4*>(red + (size_t)w * 2 * cols + i);
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
        *reinterpret_cast<float4*>(out + i) = acc;
    }
}

// V consecutive elements of type T as they come from memory (16-byte pieces), widened later.
template <typename T, int V> struct RawElems {
    static constexpr int PER = Elem<T>::VEC, N = V / PER;
    uint4 q[N];
    __device__ __forceinline__ void load(const T* p) {
#pragma unroll
        for (int i = 0; i < N; ++i) q[i] = *reinterpret_cast<const uint4*>(p + i * PER);
    }
    __device__ __forceinline__ void unpack(float* out) const {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const unsigned w[4] = {q[i].x, q[i].y, q[i].z, q[i].w};
            if constexpr (PER == 4) {
#pragma unroll
                for (int j = 0; j < 4; ++j) out[i * 4 + j] = __uint_as_float(w[j]);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    out[i * 8 + 2 * j] = __uint_as_float(w[j] << 16);
                    out[i * 8 + 2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
                }
            }
        }
    }
};

// Wide rows (more than two 16-byte chunks per lane of one wavefront): the whole workgroup
// shares a row, so a thread keeps one chunk (MAXT of them beyond 256 chunks) instead of
// four or eight, and the column sums of its chunks never leave its registers.  A workgroup
// takes LNW_ROWS rows and requests the operands of ALL of them before it touches any: the
// kernel moves 16 bytes per element and does little arithmetic, so what it needs is bytes in
// flight (about 40 KB per row here), not occupancy.  The rows' sums meet in LDS behind one
// barrier for the whole workgroup.
constexpr int LNW_THREADS = 256;
constexpr int LNW_ROWS = 4;
template <typename TX, typename TR, typename T, int MAXT>
__global__ __launch_bounds__(LNW_THREADS) void ln_bwd_wide_kernel(const T* __restrict__ dy, const TX* __restrict__ x,
                                                                  const float* __restrict__ mean,
                                                                  const float* __restrict__ rstd,
                                                                  const T* __restrict__ gamma, const TR* __restrict__ res,
                                                                  T* __restrict__ dx_lo, float* __restrict__ dx_hi,
                                                                  float* __restrict__ partial, int rows, int cols) {
    constexpr int V = Elem<T>::VEC;
    constexpr int NW = LNW_THREADS / WAVE, R = LNW_ROWS;
    __shared__ float sums[NW][R][2];
    const int tid = threadIdx.x, lane = tid % WAVE, wave = tid / WAVE;
    const int nchunk = cols / V;
    const int row0 = blockIdx.x * R;
    const int nrow = min(R, rows - row0);                     // the same for every thread of the block
    RawElems<T, V> r_dy[R][MAXT];
    RawElems<TX, V> r_x[R][MAXT];
    RawElems<TR, V> r_res[R][MAXT];
    float mu[R], rs[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        mu[r] = 0.f; rs[r] = 0.f;
        if (r < nrow) {
            const size_t ro = (size_t)(row0 + r) * cols;
            mu[r] = mean[row0 + r]; rs[r] = rstd[row0 + r];
#pragma unroll
            for (int t = 0; t < MAXT; ++t) {
                const int c = tid + t * LNW_THREADS;
                if (c < nchunk) {
                    r_dy[r][t].load(dy + ro + c * V);
                    r_x[r][t].load(x + ro + c * V);
                    if (res) r_res[r][t].load(res + ro + c * V);
                }
            }
        }
    }
    float ag[MAXT][V], ab[MAXT][V], g[MAXT][V];
#pragma unroll
    for (int t = 0; t < MAXT; ++t) {
        const int c = tid + t * LNW_THREADS;
#pragma unroll
        for (int e = 0; e < V; ++e) { ag[t][e] = 0.f; ab[t][e] = 0.f; g[t][e] = 0.f; }
        if (c < nchunk) load_vec<T>(gamma + c * V, g[t]);
    }
    float s1[R], s2[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        s1[r] = 0.f; s2[r] = 0.f;
        if (r < nrow) {
#pragma unroll
            for (int t = 0; t < MAXT; ++t) {
                const int c = tid + t * LNW_THREADS;
                if (c < nchunk) {
                    float d[V], xv[V];
                    r_dy[r][t].unpack(d);
                    r_x[r][t].unpack(xv);
#pragma unroll
                    for (int e = 0; e < V; ++e) {
                        const float xh = (xv[e] - mu[r]) * rs[r];
                        const float dxh = d[e] * g[t][e];
                        s1[r] += dxh;
                        s2[r] += dxh * xh;
                        ag[t][e] += d[e] * xh;
                        ab[t][e] += d[e];
                    }
                }
            }
        }
        s1[r] = wave_sum(s1[r]);
        s2[r] = wave_sum(s2[r]);
    }
    if (lane == 0)
#pragma unroll
        for (int r = 0; r < R; ++r) { sums[wave][r][0] = s1[r]; sums[wave][r][1] = s2[r]; }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (r >= nrow) continue;
        float m1 = 0.f, m2 = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) { m1 += sums[w][r][0]; m2 += sums[w][r][1]; }
        m1 /= (float)cols;
        m2 /= (float)cols;
        const size_t ro = (size_t)(row0 + r) * cols;
#pragma unroll
        for (int t = 0; t < MAXT; ++t) {
            const int c = tid + t * LNW_THREADS;
            if (c < nchunk) {
                float d[V], xv[V], rv[V], o[V];
                r_dy[r][t].unpack(d);
                r_x[r][t].unpack(xv);
                if (res) r_res[r][t].unpack(rv);                                          // no residual path: dx = LN'(dy)
                else
#pragma unroll
                    for (int e = 0; e < V; ++e) rv[e] = 0.f;
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    const float xh = (xv[e] - mu[r]) * rs[r];
                    o[e] = rv[e] + rs[r] * (d[e] * g[t][e] - m1 - xh * m2);
                }
                if (dx_lo) store_vec<T>(dx_lo + ro + c * V, o);
                if (dx_hi) store_elems<float, V>(dx_hi + ro + c * V, o);
            }
        }
    }
    float* out = partial + (size_t)blockIdx.x * 2 * cols;
#pragma unroll
    for (int t = 0; t < MAXT; ++t) {
        const int c = tid + t * LNW_THREADS;
        if (c < nchunk) {
            store_elems<float, V>(out + c * V, ag[t]);
            store_elems<float, V>(out + cols + c * V, ab[t]);
        }
    }
}

// ---------------------------------------------------------------- column sum
// partial[blockIdx.y][cols] = sum of CS_ROWS rows of x; lanes own columns.
template <typename T>
__global__ __launch_bounds__(LN_WAVES* WAVE) void colsum_kernel(const T* __restrict__ x, float* __restrict__ partial,
                                                                int rows, int cols) {
    constexpr int V = Elem<T>::VEC;
    __shared__ float red[WAVE * V];
    const int lane = threadIdx.x % WAVE, wave = threadIdx.x / WAVE;
    const int c = blockIdx.x * WAVE + lane;     // chunk of V columns
    const bool live = c < cols / V;
    float acc[V];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] = 0.f;
    const int row0 = blockIdx.y * CS_ROWS;
    const int row1 = min(rows, row0 + CS_ROWS);
    if (live)
        for (int row = row0 + wave; row < row1; row += LN_WAVES) {
            float v[V];
            load_vec<T>(x + (size_t)row * cols + c * V, v);
#pragma unroll
            for (int e = 0; e < V; ++e) acc[e] += v[e];
        }
    for (int w = 0; w < LN_WAVES; ++w) {
        if (wave == w) {
#pragma unroll
            for (int e = 0; e < V; ++e) {
                if (w == 0) red[lane * V + e] = acc[e];
                else red[lane * V + e] += acc[e];
            }
        }
        __syncthreads();
    }
    if (wave == 0 && live) {
        float* out = partial + (size_t)blockIdx.y * cols + c * V;
#pragma unroll
        for (int e = 0; e < V; ++e) out[e] = red[lane * V + e];
    }
}

// out[i] += sum_p partial[p][i].  A block of 256 threads owns 32 columns: thread
// (q, c) sums parts q, q+8, q+16, ... of column c with independent loads in
// flight, then the 8 sub-sums are added in fixed order through LDS.
// `split` > 0: columns [0, split) go to out, columns [split, n) to out2 (LayerNorm
// backward keeps dgamma and dbeta partials side by side).  overwrite != 0: the sums
// replace what out / out2 held instead of being added to it.
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ partial, int nparts, int n,
                                                              float* __restrict__ out, float* __restrict__ out2, int split,
                                                              int overwrite) {
    __shared__ float red[8][32];
    const int c = threadIdx.x & 31, q = threadIdx.x >> 5;
    const int i = blockIdx.x * 32 + c;
    float s = 0.f;
    if (i < n) {
        int p = q;
        for (; p + 24 < nparts; p += 32) {
            const float a0 = partial[(size_t)p * n + i], a1 = partial[(size_t)(p + 8) * n + i];
            const float a2 = partial[(size_t)(p + 16) * n + i], a3 = partial[(size_t)(p + 24) * n + i];
            s += (a0 + a1) + (a2 + a3);
        }
        for (; p < nparts; p += 8) s += partial[(size_t)p * n + i];
    }
    red[q][c] = s;
    __syncthreads();
    if (q == 0 && i < n) {
        float t = red[0][c];
#pragma unroll
        for (int k = 1; k < 8; ++k) t += red[k][c];
        float* dst = (split > 0 && i >= split) ? out2 + (i - split) : out + i;
        *dst = overwrite ? t : *dst + t;
    }
}

// The same for `gridDim.y` partial blocks at once (the LayerNorm backward passes of a whole
// stage): block row y reduces partial + y * part_stride, laid out [nparts][dgamma | dbeta], into
// the gradients of LayerNorm y = 2 * layer + (0: first, 1: second LayerNorm of the block).
// A block of 256 threads owns 64 columns: thread (q, c) sums parts q, q+16, q+32, ... of the four
// columns 4c..4c+3 (16-byte loads, four in flight), then the 16 sub-sums meet in LDS in fixed order.
__global__ __launch_bounds__(256) void reduce_partials_batched_kernel(const float* __restrict__ partial, size_t part_stride,
                                                                      int nparts, int cols, float* __restrict__ grads,
                                                                      size_t layer_stride, LnGradOffsets off, int overwrite) {
    __shared__ float4 red[16][16];
    const int c = threadIdx.x & 15, q = threadIdx.x >> 4, n = 2 * cols;
    const int i = blockIdx.x * 64 + c * 4, y = blockIdx.y;
    const float* part = partial + (size_t)y * part_stride;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    auto add = [&](const float4& v) { s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w; };
    if (i < n) {
        int p = q;
        for (; p + 48 < nparts; p += 64) {
            const float4 a0 = *reinterpret_cast<const float4*>(part + (size_t)p * n + i);
            const float4 a1 = *reinterpret_cast<const float4*>(part + (size_t)(p + 16) * n + i);
            const float4 a2 = *reinterpret_cast<const float4*>(part + (size_t)(p + 32) * n + i);
            const float4 a3 = *reinterpret_cast<const float4*>(part + (size_t)(p + 48) * n + i);
            add(make_float4((a0.x + a1.x) + (a2.x + a3.x), (a0.y + a1.y) + (a2.y + a3.y), (a0.z + a1.z) + (a2.z + a3.z),
                            (a0.w + a1.w) + (a2.w + a3.w)));
        }
        for (; p < nparts; p += 16) add(*reinterpret_cast<const float4*>(part + (size_t)p * n + i));
    }
    red[q][c] = s;
    __syncthreads();
    if (q == 0 && i < n) {
        float4 t = red[0][c];
#pragma unroll
        for (int k = 1; k < 16; ++k) { const float4 v = red[k][c]; t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w; }
        float* g = grads + (size_t)(y >> 1) * layer_stride;
        // cols is a multiple of 8, so the four columns lie on one side of the dgamma | dbeta seam
        float* dst = i < cols ? g + off.gamma[y & 1] + i : g + off.beta[y & 1] + (i - cols);
        const float tv[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) dst[e] = overwrite ? tv[e] : dst[e] + tv[e];
    }
}

__global__ void fill_zero_kernel(float4* __restrict__ p, size_t n4, float* __restrict__ tail, int ntail) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (blockIdx.x == 0 && (int)threadIdx.x < ntail) tail[threadIdx.x] = 0.f;
}

template <typename TX, typename T>
int ln_fwd_launch(int rows, int cols, const void* x, const void* gamma, const void* beta, void* y, float* mean,
                  float* rstd, hipStream_t s) {
    constexpr int V = Elem<T>::VEC;
    const int per_lane = (cols / V + WAVE - 1) / WAVE;
    const dim3 grid((rows + LN_WAVES - 1) / LN_WAVES), block(LN_WAVES * WAVE);
#define LN_FWD_CASE(N)                                                                                             \
    hipLaunchKernelGGL((ln_fwd_kernel<TX, T, N>), grid, block, 0, s, (const TX*)x, (const T*)gamma, (const T*)beta, \
                       (T*)y, mean, rstd, rows, cols)
    if (per_lane <= 1) LN_FWD_CASE(1);
    else if (per_lane <= 2) LN_FWD_CASE(2);
    else if (per_lane <= 4) LN_FWD_CASE(4);
    else if (per_lane <= 8) LN_FWD_CASE(8);
    else return fail(CHIMERA_EINVAL, "LayerNorm width %d too large (max %d)", cols, 8 * WAVE * V);
#undef LN_FWD_CASE
    CHIMERA_LAUNCH_CHECK("layernorm forward");
    return CHIMERA_OK;
}

// Workgroups (= partial-sum rows) of a LayerNorm backward over rows x cols elements of type T:
// the wavefront-per-row kernel takes LNB_ROWS rows per workgroup, the wide-row kernel LNW_ROWS.
template <typename T> int ln_bwd_blocks(int rows, int cols) {
    const bool wide = (cols / Elem<T>::VEC + WAVE - 1) / WAVE > 2;
    const int per = wide ? LNW_ROWS : LNB_ROWS;
    return (rows + per - 1) / per;
}

template <typename TX, typename TR, typename T>
int ln_bwd_launch(int rows, int cols, const void* dy, const void* x, const float* mean, const float* rstd,
                  const void* gamma, const void* res, void* dx_lo, float* dx_hi, float* dgamma, float* dbeta,
                  float* scratch, int overwrite, hipStream_t s) {
    constexpr int V = Elem<T>::VEC;
    const int per_lane = (cols / V + WAVE - 1) / WAVE;
    const int nblk = ln_bwd_blocks<T>(rows, cols);
    const dim3 grid(nblk), block(LN_WAVES * WAVE);
    const size_t lds = (size_t)LN_WAVES * 2 * cols * sizeof(float);
#define LN_BWD_CASE(N)                                                                                              \
    hipLaunchKernelGGL((ln_bwd_kernel<TX, TR, T, N>), grid, block, lds, s, (const T*)dy, (const TX*)x, mean, rstd,   \
                       (const T*)gamma, (const TR*)res, (T*)dx_lo, dx_hi, scratch, rows, cols)
#define LN_BWD_WIDE(N)                                                                                              \
    hipLaunchKernelGGL((ln_bwd_wide_kernel<TX, TR, T, N>), grid, dim3(LNW_THREADS), 0, s, (const T*)dy, (const TX*)x,   \
                       mean, rstd, (const T*)gamma, (const TR*)res, (T*)dx_lo, dx_hi, scratch, rows, cols)
    const int per_thread = (cols / V + LNW_THREADS - 1) / LNW_THREADS;
    if (per_lane <= 1) LN_BWD_CASE(1);
    else if (per_lane <= 2) LN_BWD_CASE(2);
    else if (per_thread <= 1) LN_BWD_WIDE(1);
    else if (per_thread <= 2) LN_BWD_WIDE(2);
    else return fail(CHIMERA_EINVAL, "LayerNorm width %d too large for the backward (max %d)", cols, 2 * LNW_THREADS * V);
#undef LN_BWD_CASE
#undef LN_BWD_WIDE
    CHIMERA_LAUNCH_CHECK("layernorm backward");
    if (!dgamma) return CHIMERA_OK;            // the caller reduces the partial sums later (layernorm_bwd_reduce)
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((2 * cols + 31) / 32), dim3(256), 0, s, scratch, nblk, 2 * cols,
                       dgamma, dbeta, cols, overwrite);
    CHIMERA_LAUNCH_CHECK("layernorm backward reduce");
    return CHIMERA_OK;
}

template <typename T>
int colsum_launch(int rows, int cols, const void* x, float* out, float* scratch, hipStream_t s) {
    constexpr int V = Elem<T>::VEC;
    const int nparts = (rows + CS_ROWS - 1) / CS_ROWS;
    const dim3 grid((cols / V + WAVE - 1) / WAVE, nparts), block(LN_WAVES * WAVE);
    hipLaunchKernelGGL((colsum_kernel<T>), grid, block, 0, s, (const T*)x, scratch, rows, cols);
    CHIMERA_LAUNCH_CHECK("column sum");
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((cols + 31) / 32), dim3(256), 0, s, scratch, nparts, cols, out,
                       (float*)nullptr, 0, 0);
    CHIMERA_LAUNCH_CHECK("column sum reduce");
    return CHIMERA_OK;
}

int check_rowwise(int dtype, int rows, int cols) {
    if (dtype != CHIMERA_F32 && dtype != CHIMERA_BF16) return fail(CHIMERA_EINVAL, "unknown dtype %d", dtype);
    if (rows < 1 || cols < 1) return fail(CHIMERA_EINVAL, "rows=%d cols=%d must be positive", rows, cols);
    if (cols % 8) return fail(CHIMERA_EINVAL, "cols=%d must be a multiple of 8", cols);
    return CHIMERA_OK;
}

}  // namespace

int layernorm_fwd(int dtype, int rows, int cols, const void* x, int x_f32, const void* gamma, const void* beta, void* y,
                  float* mean, float* rstd, void* stream) {
    if (int rc = check_rowwise(dtype, rows, cols)) return rc;
    hipStream_t s = (hipStream_t)stream;
    if (dtype == CHIMERA_F32) return ln_fwd_launch<float, float>(rows, cols, x, gamma, beta, y, mean, rstd, s);
    return x_f32 ? ln_fwd_launch<float, bf16_t>(rows, cols, x, gamma, beta, y, mean, rstd, s)
                 : ln_fwd_launch<bf16_t, bf16_t>(rows, cols, x, gamma, beta, y, mean, rstd, s);
}

// enough for either element type (a float row of `cols` has twice the chunks of a bf16 row, so
// it may take the wide-row kernel, with fewer rows per workgroup, where the bf16 row does not)
size_t layernorm_bwd_scratch_floats(int rows, int cols) {
    return (size_t)std::max(ln_bwd_blocks<float>(rows, cols), ln_bwd_blocks<bf16_t>(rows, cols)) * 2 * cols;
}

int layernorm_bwd(int dtype, int rows, int cols, const void* dy, const void* x, int x_f32, const float* mean,
                  const float* rstd, const void* gamma, const void* res, int res_f32, void* dx_lo, float* dx_hi,
                  float* dgamma, float* dbeta, float* scratch, int overwrite, void* stream) {
    if (int rc = check_rowwise(dtype, rows, cols)) return rc;
    if (!dx_lo && !dx_hi) return fail(CHIMERA_EINVAL, "layernorm backward needs an output");
    hipStream_t s = (hipStream_t)stream;
#define LN_BWD_ARGS rows, cols, dy, x, mean, rstd, gamma, res, dx_lo, dx_hi, dgamma, dbeta, scratch, overwrite, s
    if (dtype == CHIMERA_F32) return ln_bwd_launch<float, float, float>(LN_BWD_ARGS);
    if (x_f32) return res_f32 ? ln_bwd_launch<float, float, bf16_t>(LN_BWD_ARGS) : ln_bwd_launch<float, bf16_t, bf16_t>(LN_BWD_ARGS);
    return res_f32 ? ln_bwd_launch<bf16_t, float, bf16_t>(LN_BWD_ARGS) : ln_bwd_launch<bf16_t, bf16_t, bf16_t>(LN_BWD_ARGS);
#undef LN_BWD_ARGS
}

// Device address of the static scratch array on the current device, looked up once per
// device (each GPU holds its own copy at its own address).
int static_scratch(float** out) {
    constexpr int MAX_DEVICES = 64;
    static std::mutex mu;
    static float* ptr[MAX_DEVICES] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(CHIMERA_EDEVICE, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(CHIMERA_EDEVICE, "device index %d outside [0,%d)", dev, MAX_DEVICES);
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        float* p = nullptr;
        e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail(CHIMERA_EDEVICE, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return CHIMERA_OK;
}

size_t layernorm_bwd_static_scratch_floats() { return LN_STATIC_SCRATCH_FLOATS; }

int layernorm_bwd_noalloc(int dtype, int rows, int cols, const void* dy, const void* x, const float* mean, const float* rstd,
                          const void* gamma, const void* res, void* dx, float* dgamma, float* dbeta, void* stream) {
    if (int rc = check_rowwise(dtype, rows, cols)) return rc;
    const size_t need = layernorm_bwd_scratch_floats(rows, cols);
    if (need > LN_STATIC_SCRATCH_FLOATS)
        return fail(CHIMERA_ENOMEM, "layernorm backward of %d x %d needs %zu scratch floats, the static scratch holds %zu",
                    rows, cols, need, (size_t)LN_STATIC_SCRATCH_FLOATS);
    float* sc = nullptr;
    if (int rc = static_scratch(&sc)) return rc;
    return layernorm_bwd(dtype, rows, cols, dy, x, 0, mean, rstd, gamma, res, 0, dx, nullptr, dgamma, dbeta, sc, 0, stream);
}

int layernorm_bwd_reduce(int dtype, int rows, int cols, int count, const float* partial, size_t part_stride, float* grads,
                         size_t layer_stride, const LnGradOffsets& off, int overwrite, void* stream) {
    if (count < 1) return CHIMERA_OK;
    if (rows < 1 || cols < 1 || !partial || !grads || count > 65535) return fail(CHIMERA_EINVAL, "layernorm backward reduce: bad arguments");
    const int nblk = dtype == CHIMERA_F32 ? ln_bwd_blocks<float>(rows, cols) : ln_bwd_blocks<bf16_t>(rows, cols);
    hipLaunchKernelGGL(reduce_partials_batched_kernel, dim3((2 * cols + 63) / 64, count), dim3(256), 0, (hipStream_t)stream,
                       partial, part_stride, nblk, cols, grads, layer_stride, off, overwrite);
    CHIMERA_LAUNCH_CHECK("layernorm backward reduce (batched)");
    return CHIMERA_OK;
}

size_t colsum_scratch_floats(int rows, int cols) { return (size_t)((rows + CS_ROWS - 1) / CS_ROWS) * cols; }

int colsum(int dtype, int rows, int cols, const void* x, float* out, float* scratch, void* stream) {
    if (int rc = check_rowwise(dtype, rows, cols)) return rc;
    hipStream_t s = (hipStream_t)stream;
    return dtype == CHIMERA_F32 ? colsum_launch<float>(rows, cols, x, out, scratch, s)
                                : colsum_launch<bf16_t>(rows, cols, x, out, scratch, s);
}

int fill_zero_f32(float* p, size_t n, void* stream) {
    if (!n) return CHIMERA_OK;
    const size_t n4 = n / 4;
    const int ntail = (int)(n - n4 * 4);
    const int blocks = (int)std::min<size_t>((n4 + 255) / 256 + 1, 4096);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (float4*)p, n4, p + n4 * 4, ntail);
    CHIMERA_LAUNCH_CHECK("fill");
    return CHIMERA_OK;
}

}  // namespace chimera
