// Fused attention on the CDNA4 matrix cores (bf16 in, float softmax and
// accumulation), forward and backward, for head_dim 64 and 128.
//
//   forward   per (sequence, head, 128 queries): loop over 64-key tiles with an
//             online softmax; writes ctx and the log-sum-exp of every row.
//   backward  delta = rowsum(dctx * ctx); then two kernels that both rebuild
//             P = exp(q k^T / sqrt(d) - lse) from the saved log-sum-exp:
//             dK/dV per (sequence, head, 128 keys) looping over 64-query tiles,
//             dQ    per (sequence, head, 128 queries) looping over 64-key tiles.
//             No atomics: every output element has one owner, so results are
//             reproducible bit for bit.
//
// Register/LDS choreography.  v_mfma_f32_32x32x16_bf16 takes, per lane l, 8
// contraction values of row (or column) l%32; which 8 contraction indices a
// lane group l/32 holds is free as long as both operands agree.  Its result
// gives lane l column l%32 and rows 8*(r/4) + 4*(l/32) + r%4 (r = register).
// So a score tile computed TRANSPOSED (keys x queries) leaves each lane with
// one query and 16 keys - exactly an operand of the next product (contraction
// over keys) with keys {4g..4g+3, 8+4g..8+4g+3} (g = l/32) per 16-key step.
// The other operand of that product (V^T, or Q^T, dO^T, K^T in the backward)
// is staged in LDS transposed, with the contraction index permuted inside
// every group of 16 so that those 8 values are one 16-byte read.  The
// transposition happens in registers between the coalesced global load and the
// LDS write; P never touches LDS, and no transposed tensor exists in HBM.
// The fixed operand of a wavefront (its 32 queries, or its 32 keys and values)
// is loaded straight from global memory into MFMA operand registers.
//
// LDS tiles are [rows][64] bf16 (128 bytes per row, 8 chunks of 16 bytes),
// chunk c of row r stored at c ^ (r & 7) ^ ((r >> 3) & 7).
#include "device.h"

namespace chimera {

namespace {

typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int NT = 256;
constexpr float NEG_BIG = -1.0e30f;
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ (row & 7) ^ ((row >> 3) & 7); }
__device__ __forceinline__ int tile_off(int row, int chunk) { return row * 64 + swz(row, chunk) * 8; }

__device__ __forceinline__ unsigned half_of(const uint4& q, int t) {
    const unsigned w = (t >> 1) == 0 ? q.x : (t >> 1) == 1 ? q.y : (t >> 1) == 2 ? q.z : q.w;
    return (t & 1) ? (w >> 16) : (w & 0xffffu);
}

__device__ __forceinline__ bf16x8 load_frag(const bf16_t* p, bool ok) {
    bf16x8 z;
#pragma unroll
    for (int i = 0; i < 8; ++i) z[i] = (bf16_t)0.f;
    return ok ? *reinterpret_cast<const bf16x8*>(p) : z;
}

// ---- cooperative tile movers (all NT threads call them) --------------------
// "Straight" tile: 64 rows x D columns of a row-major global matrix (row stride
// ld), kept as D/64 LDS tiles [64][64] (sub-tile s = columns 64s..64s+63).
template <int D> struct StraightRegs { uint4 v[64 * D / 8 / NT]; };

template <int D>
__device__ __forceinline__ void load_straight(StraightRegs<D>& r, const bf16_t* __restrict__ g, int ld, int row0,
                                              int row_end, int tid) {
    constexpr int CPR = D / 8;   // chunks per row
#pragma unroll
    for (int it = 0; it < 64 * CPR / NT; ++it) {
        const int c = tid + it * NT;
        const int row = c / CPR, ch = c % CPR;
        uint4 q = make_uint4(0u, 0u, 0u, 0u);
        if (row0 + row < row_end) q = *reinterpret_cast<const uint4*>(g + (size_t)(row0 + row) * ld + ch * 8);
        r.v[it] = q;
    }
}
template <int D>
__device__ __forceinline__ void store_straight(const StraightRegs<D>& r, bf16_t* lds, int tid) {
    constexpr int CPR = D / 8;
#pragma unroll
    for (int it = 0; it < 64 * CPR / NT; ++it) {
        const int c = tid + it * NT;
        const int row = c / CPR, ch = c % CPR;
        *reinterpret_cast<uint4*>(lds + (ch >> 3) * 4096 + tile_off(row, ch & 7)) = r.v[it];
    }
}

// "Transposed" tile: the same 64 x D global block, kept as D/64 LDS tiles
// [64 columns][64 rows]: LDS row = global column, contraction index = global
// row, permuted inside every 16: global row 16J + 8a + 4g + c sits at position
// 16J + 8g + 4a + c.  Unit of work: 8 columns x 4 rows (four 16-byte loads).
template <int D> struct TransRegs {
    static constexpr int UNITS = (D / 8) * 16;
    static constexpr int UPT = (UNITS + NT - 1) / NT;
    uint4 v[UPT * 4];
};
template <int D>
__device__ __forceinline__ void load_trans(TransRegs<D>& r, const bf16_t* __restrict__ g, int ld, int row0, int row_end,
                                           int tid) {
    constexpr int IG = D / 8;
#pragma unroll
    for (int it = 0; it < TransRegs<D>::UPT; ++it) {
        const int u = tid + it * NT;
        const int ig = u % IG, kg = u / IG;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const int row = row0 + kg * 4 + rr;
            uint4 q = make_uint4(0u, 0u, 0u, 0u);
            if (u < TransRegs<D>::UNITS && row < row_end) q = *reinterpret_cast<const uint4*>(g + (size_t)row * ld + ig * 8);
            r.v[it * 4 + rr] = q;
        }
    }
}
template <int D>
__device__ __forceinline__ void store_trans(const TransRegs<D>& r, bf16_t* lds, int tid) {
    constexpr int IG = D / 8;
#pragma unroll
    for (int it = 0; it < TransRegs<D>::UPT; ++it) {
        const int u = tid + it * NT;
        if (u >= TransRegs<D>::UNITS) continue;
        const int ig = u % IG, kg = u / IG;
        const int koff = kg * 4;
        const int J = koff >> 4, a = (koff >> 3) & 1, gg = (koff >> 2) & 1;
        const int chunk = 2 * J + gg, within = 4 * a;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int col = ig * 8 + t;             // global column = LDS row
            const unsigned w0 = half_of(r.v[it * 4 + 0], t) | (half_of(r.v[it * 4 + 1], t) << 16);
            const unsigned w1 = half_of(r.v[it * 4 + 2], t) | (half_of(r.v[it * 4 + 3], t) << 16);
            *reinterpret_cast<uint2*>(lds + (col >> 6) * 4096 + tile_off(col & 63, chunk) + within) = make_uint2(w0, w1);
        }
    }
}

// One 64 x D global block kept BOTH ways (straight in `lds_s`, transposed in `lds_t`) from a
// single set of loads: a thread's unit of 4 rows x 8 columns is four straight 16-byte
// chunks as loaded, and four 8-byte transposed pieces after the register shuffle.
template <int D>
__device__ __forceinline__ void store_both(const TransRegs<D>& r, bf16_t* lds_s, bf16_t* lds_t, int tid) {
    constexpr int IG = D / 8;
#pragma unroll
    for (int it = 0; it < TransRegs<D>::UPT; ++it) {
        const int u = tid + it * NT;
        if (u >= TransRegs<D>::UNITS) continue;
        const int ig = u % IG, kg = u / IG;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const int row = kg * 4 + rr;
            *reinterpret_cast<uint4*>(lds_s + (ig >> 3) * 4096 + tile_off(row, ig & 7)) = r.v[it * 4 + rr];
        }
    }
    store_trans<D>(r, lds_t, tid);
}

// Operand fragment of a straight tile: row `row` (0..63), contraction step kk (16 columns each).
template <int D>
__device__ __forceinline__ bf16x8 frag_straight(const bf16_t* lds, int row, int kk, int g) {
    return *reinterpret_cast<const bf16x8*>(lds + (kk >> 2) * 4096 + tile_off(row, (kk & 3) * 2 + g));
}
// Operand fragment of a transposed tile: LDS row `col` (0..D-1), 16-step J of the contraction index.
__device__ __forceinline__ bf16x8 frag_trans(const bf16_t* lds, int col, int J, int g) {
    return *reinterpret_cast<const bf16x8*>(lds + (col >> 6) * 4096 + tile_off(col & 63, 2 * J + g));
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int first) {
    bf16x8 o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (bf16_t)v[first + i];
    return o;
}

__device__ __forceinline__ float xor32(float v) { return __shfl_xor(v, 32, WAVE); }

// ------------------------------------------------------------------- forward
template <int D, bool CAUSAL>
__global__ __launch_bounds__(NT) void attn_fwd_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ ctx,
                                                      float* __restrict__ lse, int S, int heads, float scale_log2e) {
    constexpr int KS = D / 16, OT = D / 32;
    __shared__ __attribute__((aligned(16))) bf16_t Ks[2][64 * D];
    __shared__ __attribute__((aligned(16))) bf16_t Vt[2][64 * D];
    const int H = heads * D, ld = 3 * H;
    const int q0 = (gridDim.x - 1 - blockIdx.x) * 128;       // longest (causal) tiles first
    const int h = blockIdx.y, b = blockIdx.z;
    const bf16_t* base = qkv + (size_t)b * S * ld + h * D;
    const bf16_t* Kg = base + H;
    const bf16_t* Vg = base + 2 * H;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
    const int wq0 = q0 + wave * 32, qrow = wq0 + l32;

    bf16x8 qf[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) qf[kk] = load_frag(base + (size_t)qrow * ld + kk * 16 + g * 8, qrow < S);

    f32x16 o[OT];
#pragma unroll
    for (int t = 0; t < OT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[t][r] = 0.f;
    float m = NEG_BIG, lsum = 0.f;

    const int kv_end = CAUSAL ? min(S, q0 + 128) : S;
    const int ntiles = (kv_end + 63) / 64;
    StraightRegs<D> rk;
    TransRegs<D> rv;
    load_straight<D>(rk, Kg, ld, 0, S, tid);
    load_trans<D>(rv, Vg, ld, 0, S, tid);
    store_straight<D>(rk, Ks[0], tid);
    store_trans<D>(rv, Vt[0], tid);
    __syncthreads();

    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1, k0 = t * 64;
        if (t + 1 < ntiles) {
            load_straight<D>(rk, Kg, ld, k0 + 64, S, tid);
            load_trans<D>(rv, Vg, ld, k0 + 64, S, tid);
        }
        const bool live = !CAUSAL || k0 <= wq0 + 31;          // wavefront-uniform: some key is visible
        if (live) {
            f32x16 s[2];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kt][r] = 0.f;
#pragma unroll
                for (int kk = 0; kk < KS; ++kk)
                    s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_straight<D>(Ks[buf], kt * 32 + l32, kk, g), qf[kk],
                                                                    s[kt], 0, 0, 0);
            }
            const bool edge = (k0 + 63 >= S) || (CAUSAL && k0 + 63 > wq0);
            float mx = NEG_BIG;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float v = s[kt][r] * scale_log2e;
                    if (edge) {
                        const int key = k0 + kt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                        if (key >= S || (CAUSAL && key > qrow)) v = NEG_BIG;
                    }
                    s[kt][r] = v;
                    mx = fmaxf(mx, v);
                }
            mx = fmaxf(mx, xor32(mx));
            const float m_new = fmaxf(m, mx);
            const float alpha = exp2f(m - m_new);
            float rs = 0.f;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float p = exp2f(s[kt][r] - m_new);
                    s[kt][r] = p;
                    rs += p;
                }
            rs += xor32(rs);
            lsum = lsum * alpha + rs;
            m = m_new;
#pragma unroll
            for (int t2 = 0; t2 < OT; ++t2)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[t2][r] *= alpha;
#pragma unroll
            for (int J = 0; J < 4; ++J) {
                const bf16x8 pf = pack8(s[J >> 1], (J & 1) * 8);
#pragma unroll
                for (int t2 = 0; t2 < OT; ++t2)
                    o[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_trans(Vt[buf], t2 * 32 + l32, J, g), pf, o[t2], 0, 0, 0);
            }
        }
        if (t + 1 < ntiles) {
            store_straight<D>(rk, Ks[buf ^ 1], tid);
            store_trans<D>(rv, Vt[buf ^ 1], tid);
        }
        __syncthreads();
    }

    if (qrow < S) {
        const float inv = 1.0f / lsum;
        bf16_t* out = ctx + ((size_t)b * S + qrow) * H + h * D;
#pragma unroll
        for (int t2 = 0; t2 < OT; ++t2)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                bf16x4 v;
#pragma unroll
                for (int c = 0; c < 4; ++c) v[c] = (bf16_t)(o[t2][r4 * 4 + c] * inv);
                *reinterpret_cast<bf16x4*>(out + t2 * 32 + 8 * r4 + 4 * g) = v;
            }
        if (g == 0) lse[((size_t)b * heads + h) * S + qrow] = (m + log2f(lsum)) * LN2;
    }
}

// ------------------------------------------------------------------ backward
// delta[b, h, s] = sum over the head's d columns of dctx * ctx.  One wavefront per token.
template <int D>
__global__ __launch_bounds__(NT) void attn_delta_kernel(const bf16_t* __restrict__ dctx, const bf16_t* __restrict__ ctx,
                                                        float* __restrict__ delta, int batch, int S, int heads) {
    const int H = heads * D, lane = threadIdx.x & 63;
    const int token = blockIdx.x * (NT / WAVE) + (threadIdx.x >> 6);
    if (token >= batch * S) return;
    constexpr int LPH = D / 8;                   // lanes per head
    for (int c0 = 0; c0 < H / 8; c0 += WAVE) {
        const int c = c0 + lane;
        float s = 0.f;
        if (c < H / 8) {
            float a[8], bb[8];
            load_vec<bf16_t>(dctx + (size_t)token * H + c * 8, a);
            load_vec<bf16_t>(ctx + (size_t)token * H + c * 8, bb);
#pragma unroll
            for (int e = 0; e < 8; ++e) s += a[e] * bb[e];
        }
#pragma unroll
        for (int o = 1; o < LPH; o <<= 1) s += __shfl_xor(s, o, WAVE);
        if (c < H / 8 && (lane % LPH) == 0) {
            const int head = c / LPH;
            delta[((size_t)(token / S) * heads + head) * S + (token % S)] = s;
        }
    }
}

// dK, dV of 128 keys (32 per wavefront), looping over 64-query tiles.
//   S  = Q K^T (queries x keys)   P = exp2(S c - lse2)     dP = dO V^T
//   dS = P (dP - delta)           dV^T += dO^T P           dK^T += Q^T dS (then * 1/sqrt(d))
// The next tile's Q, dO, lse and delta are already on their way to registers while the
// matrix cores work on the current one; each 32-query half of a tile is finished (scores
// to dK/dV) before the next starts, which keeps the live score registers at 32.
template <int D, bool CAUSAL>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(D == 64 ? 2 : 1, 2)))
void attn_bwd_dkv_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dctx,
                         const float* __restrict__ lse, const float* __restrict__ delta,
                         bf16_t* __restrict__ dqkv, int S, int heads, float scale) {
    constexpr int KS = D / 16, OT = D / 32;
    __shared__ __attribute__((aligned(16))) bf16_t Qs[64 * D], Qt[64 * D], Os[64 * D], Ot[64 * D];
    __shared__ __attribute__((aligned(16))) float lse2[64], dl[64];
    const int H = heads * D, ld = 3 * H;
    const int j0 = blockIdx.x * 128, h = blockIdx.y, b = blockIdx.z;
    const bf16_t* base = qkv + (size_t)b * S * ld + h * D;
    const bf16_t* dOg = dctx + (size_t)b * S * H + h * D;
    const size_t stat0 = ((size_t)b * heads + h) * S;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
    const int wj0 = j0 + wave * 32, jrow = wj0 + l32;
    const float c2 = scale * LOG2E;

    bf16x8 kf[KS], vf[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
        kf[kk] = load_frag(base + H + (size_t)jrow * ld + kk * 16 + g * 8, jrow < S);
        vf[kk] = load_frag(base + 2 * H + (size_t)jrow * ld + kk * 16 + g * 8, jrow < S);
    }
    f32x16 dk[OT], dv[OT];
#pragma unroll
    for (int t = 0; t < OT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) { dk[t][r] = 0.f; dv[t][r] = 0.f; }

    const int qt0 = CAUSAL ? j0 / 64 : 0;
    const int ntiles = (S + 63) / 64;
    TransRegs<D> rq, ro;
    float stat = 0.f;                      // lse (threads 0..63) or delta (threads 64..127) of the next tile
    auto fetch = [&](int t) {
        const int i0 = t * 64;
        load_trans<D>(rq, base, ld, i0, S, tid);
        load_trans<D>(ro, dOg, H, i0, S, tid);
        if (tid < 128) {
            const int i = i0 + (tid & 63);
            stat = i < S ? (tid < 64 ? lse[stat0 + i] * LOG2E : delta[stat0 + i]) : 0.f;
        }
    };
    fetch(qt0);
    for (int t = qt0; t < ntiles; ++t) {
        const int i0 = t * 64;
        store_both<D>(rq, Qs, Qt, tid);
        store_both<D>(ro, Os, Ot, tid);
        if (tid < 64) lse2[tid] = stat;
        else if (tid < 128) dl[tid - 64] = stat;
        __syncthreads();
        if (t + 1 < ntiles) fetch(t + 1);
        const bool live = !CAUSAL || i0 + 63 >= wj0;           // some query of the tile sees some key of this wavefront
        if (live) {
            const bool edge = (i0 + 63 >= S) || (CAUSAL && i0 < wj0 + 31);
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                f32x16 p, dp;
#pragma unroll
                for (int r = 0; r < 16; ++r) { p[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
                for (int kk = 0; kk < KS; ++kk) {
                    p = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_straight<D>(Qs, it * 32 + l32, kk, g), kf[kk], p, 0, 0, 0);
                    dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_straight<D>(Os, it * 32 + l32, kk, g), vf[kk], dp, 0, 0, 0);
                }
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int il = it * 32 + 8 * r4 + 4 * g;       // 4 consecutive queries
                    const float4 l4 = *reinterpret_cast<const float4*>(&lse2[il]);
                    const float4 d4 = *reinterpret_cast<const float4*>(&dl[il]);
                    const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int r = r4 * 4 + c;
                        float pv = exp2f(p[r] * c2 - lv[c]);
                        if (edge) {
                            const int i = i0 + il + c;
                            if (i >= S || (CAUSAL && i < jrow)) pv = 0.f;
                        }
                        p[r] = pv;
                        dp[r] = pv * (dp[r] - dv4[c]);
                    }
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int J = it * 2 + j;
                    const bf16x8 pf = pack8(p, j * 8);
                    const bf16x8 dsf = pack8(dp, j * 8);
#pragma unroll
                    for (int t2 = 0; t2 < OT; ++t2) {
                        dv[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_trans(Ot, t2 * 32 + l32, J, g), pf, dv[t2], 0, 0, 0);
                        dk[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_trans(Qt, t2 * 32 + l32, J, g), dsf, dk[t2], 0, 0, 0);
                    }
                }
            }
        }
        __syncthreads();
    }
    if (jrow < S) {
        bf16_t* out = dqkv + ((size_t)b * S + jrow) * ld + h * D;
#pragma unroll
        for (int t2 = 0; t2 < OT; ++t2)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                bf16x4 a, c;
#pragma unroll
                for (int e = 0; e < 4; ++e) { a[e] = (bf16_t)(dk[t2][r4 * 4 + e] * scale); c[e] = (bf16_t)dv[t2][r4 * 4 + e]; }
                *reinterpret_cast<bf16x4*>(out + H + t2 * 32 + 8 * r4 + 4 * g) = a;
                *reinterpret_cast<bf16x4*>(out + 2 * H + t2 * 32 + 8 * r4 + 4 * g) = c;
            }
    }
}

// dQ of 128 queries (32 per wavefront), looping over 64-key tiles.
//   S^T = K Q^T (keys x queries)   P = exp2(S^T c - lse2)   dP^T = V dO^T
//   dS^T = P (dP^T - delta)        dQ^T += K^T dS^T (then * 1/sqrt(d))
template <int D, bool CAUSAL>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(D == 64 ? 2 : 1, 2)))
void attn_bwd_dq_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dctx,
                        const float* __restrict__ lse, const float* __restrict__ delta,
                        bf16_t* __restrict__ dqkv, int S, int heads, float scale) {
    constexpr int KS = D / 16, OT = D / 32;
    __shared__ __attribute__((aligned(16))) bf16_t Ks[64 * D], Kt[64 * D], Vs[64 * D];
    const int H = heads * D, ld = 3 * H;
    const int q0 = (gridDim.x - 1 - blockIdx.x) * 128, h = blockIdx.y, b = blockIdx.z;
    const bf16_t* base = qkv + (size_t)b * S * ld + h * D;
    const bf16_t* dOg = dctx + (size_t)b * S * H + h * D;
    const size_t stat0 = ((size_t)b * heads + h) * S;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
    const int wq0 = q0 + wave * 32, qrow = wq0 + l32;
    const float c2 = scale * LOG2E;

    bf16x8 qf[KS], of[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
        qf[kk] = load_frag(base + (size_t)qrow * ld + kk * 16 + g * 8, qrow < S);
        of[kk] = load_frag(dOg + (size_t)qrow * H + kk * 16 + g * 8, qrow < S);
    }
    const float my_lse2 = qrow < S ? lse[stat0 + qrow] * LOG2E : 0.f;
    const float my_dl = qrow < S ? delta[stat0 + qrow] : 0.f;
    f32x16 dq[OT];
#pragma unroll
    for (int t = 0; t < OT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) dq[t][r] = 0.f;

    const int kv_end = CAUSAL ? min(S, q0 + 128) : S;
    const int ntiles = (kv_end + 63) / 64;
    TransRegs<D> rk;
    StraightRegs<D> rv;
    auto fetch = [&](int t) {
        load_trans<D>(rk, base + H, ld, t * 64, S, tid);
        load_straight<D>(rv, base + 2 * H, ld, t * 64, S, tid);
    };
    fetch(0);
    for (int t = 0; t < ntiles; ++t) {
        const int k0 = t * 64;
        store_both<D>(rk, Ks, Kt, tid);
        store_straight<D>(rv, Vs, tid);
        __syncthreads();
        if (t + 1 < ntiles) fetch(t + 1);
        const bool live = !CAUSAL || k0 <= wq0 + 31;
        if (live) {
            const bool edge = (k0 + 63 >= S) || (CAUSAL && k0 + 63 > wq0);
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                f32x16 p, dp;
#pragma unroll
                for (int r = 0; r < 16; ++r) { p[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
                for (int kk = 0; kk < KS; ++kk) {
                    p = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_straight<D>(Ks, kt * 32 + l32, kk, g), qf[kk], p, 0, 0, 0);
                    dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_straight<D>(Vs, kt * 32 + l32, kk, g), of[kk], dp, 0, 0, 0);
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float pv = exp2f(p[r] * c2 - my_lse2);
                    if (edge) {
                        const int key = k0 + kt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                        if (key >= S || (CAUSAL && key > qrow)) pv = 0.f;
                    }
                    dp[r] = pv * (dp[r] - my_dl);
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const bf16x8 dsf = pack8(dp, j * 8);
#pragma unroll
                    for (int t2 = 0; t2 < OT; ++t2)
                        dq[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_trans(Kt, t2 * 32 + l32, kt * 2 + j, g), dsf, dq[t2], 0, 0, 0);
                }
            }
        }
        __syncthreads();
    }
    if (qrow < S) {
        bf16_t* out = dqkv + ((size_t)b * S + qrow) * ld + h * D;
#pragma unroll
        for (int t2 = 0; t2 < OT; ++t2)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                bf16x4 a;
#pragma unroll
                for (int e = 0; e < 4; ++e) a[e] = (bf16_t)(dq[t2][r4 * 4 + e] * scale);
                *reinterpret_cast<bf16x4*>(out + t2 * 32 + 8 * r4 + 4 * g) = a;
            }
    }
}

int check(const AttnArgs& a) {
    if (!attention_mfma_supports(a)) return fail(CHIMERA_EINVAL, "matrix-core attention: unsupported shape (head_dim %d)", a.head_dim);
    return CHIMERA_OK;
}

}  // namespace

bool attention_mfma_supports(const AttnArgs& a) {
    if (a.head_dim != 64 && a.head_dim != 128) return false;
    if (a.batch < 1 || a.seq < 1 || a.heads < 1 || a.batch > 65535 || a.heads > 65535) return false;
    if ((uintptr_t)a.qkv & 15) return false;
    return true;
}

int attention_fwd_mfma(const AttnArgs& a, void* stream) {
    if (int rc = check(a)) return rc;
    if ((uintptr_t)a.ctx & 7) return fail(CHIMERA_EINVAL, "ctx must be 8-byte aligned");
    const dim3 grid((a.seq + 127) / 128, a.heads, a.batch), block(NT);
    const float sl2 = LOG2E / sqrtf((float)a.head_dim);
    hipStream_t s = (hipStream_t)stream;
#define ATTN_FWD(D, C)                                                                                            \
    hipLaunchKernelGGL((attn_fwd_kernel<D, C>), grid, block, 0, s, (const bf16_t*)a.qkv, (bf16_t*)a.ctx, a.lse, a.seq, \
                       a.heads, sl2)
    if (a.head_dim == 64) { if (a.causal) ATTN_FWD(64, true); else ATTN_FWD(64, false); }
    else { if (a.causal) ATTN_FWD(128, true); else ATTN_FWD(128, false); }
#undef ATTN_FWD
    CHIMERA_LAUNCH_CHECK("attention forward");
    return CHIMERA_OK;
}

int attention_bwd_mfma(const AttnArgs& a, void* stream) {
    if (int rc = check(a)) return rc;
    if (((uintptr_t)a.ctx | (uintptr_t)a.dctx | (uintptr_t)a.dqkv) & 15) return fail(CHIMERA_EINVAL, "attention buffers must be 16-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    const int tokens = a.batch * a.seq;
    const dim3 block(NT), tgrid((tokens + NT / WAVE - 1) / (NT / WAVE));
    const dim3 grid((a.seq + 127) / 128, a.heads, a.batch);
    const float scale = 1.0f / sqrtf((float)a.head_dim);
#define ATTN_BWD(D, C)                                                                                              \
    do {                                                                                                            \
        hipLaunchKernelGGL((attn_delta_kernel<D>), tgrid, block, 0, s, (const bf16_t*)a.dctx, (const bf16_t*)a.ctx,   \
                           a.delta, a.batch, a.seq, a.heads);                                                       \
        hipLaunchKernelGGL((attn_bwd_dkv_kernel<D, C>), grid, block, 0, s, (const bf16_t*)a.qkv, (const bf16_t*)a.dctx, \
                           a.lse, a.delta, (bf16_t*)a.dqkv, a.seq, a.heads, scale);                                 \
        hipLaunchKernelGGL((attn_bwd_dq_kernel<D, C>), grid, block, 0, s, (const bf16_t*)a.qkv, (const bf16_t*)a.dctx,  \
                           a.lse, a.delta, (bf16_t*)a.dqkv, a.seq, a.heads, scale);                                 \
    } while (0)
    if (a.head_dim == 64) { if (a.causal) ATTN_BWD(64, true); else ATTN_BWD(64, false); }
    else { if (a.causal) ATTN_BWD(128, true); else ATTN_BWD(128, false); }
#undef ATTN_BWD
    CHIMERA_LAUNCH_CHECK("attention backward");
    return CHIMERA_OK;
}

}  // namespace chimera
