// Fused attention on the CDNA4 matrix cores (bf16 in, float softmax and
// accumulation), forward and backward, for head_dim 64 and 128.
//
//   forward   per (sequence, head, 128 queries): loop over 64-key tiles with an
//             online softmax; writes ctx and the log-sum-exp of every row.
//   backward  two roles that both rebuild P = exp(q k^T / sqrt(d) - lse) from
//             the saved log-sum-exp:
//             dQ    per (sequence, head, 128 queries) looping over 64-key tiles,
//             dK/dV per (sequence, head, 128 keys) looping over 64-query tiles.
//             With many (sequence, head) pairs they are two launches and the dQ
//             one forms delta = rowsum(dctx * ctx) of its queries on the way;
//             with few pairs a small kernel forms delta first and both roles
//             share one launch.  No atomics: every output element has one
//             owner, so results are reproducible bit for bit.
//
// Register/LDS choreography.  v_mfma_f32_32x32x16_bf16 takes, per lane l, 8
// contraction values of row (or column) l%32; which 8 contraction indices a
// lane group l/32 holds is free as long as both operands agree.  Its result
// gives lane l column l%32 and rows 8*(r/4) + 4*(l/32) + r%4 (r = register).
// So a score tile computed TRANSPOSED (keys x queries) leaves each lane with
// one query and 16 keys - exactly an operand of the next product (contraction
// over keys) with keys {4g..4g+3, 8+4g..8+4g+3} (g = l/32) per 16-key step.
// The other operand of that product (V^T, or Q^T, dO^T, K^T in the backward)
// comes from the same LDS tile the tensor arrived in, through the transposing
// LDS read; P never touches LDS, and no transposed tensor exists anywhere.
// The fixed operand of a wavefront (its 32 queries, or its 32 keys and values)
// is loaded straight from global memory into MFMA operand registers.
#include "device.h"

#include <type_traits>

namespace chimera {

namespace {

typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int NT = 256;
constexpr float NEG_BIG = -1.0e30f;
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

__device__ __forceinline__ bf16x8 load_frag(const bf16_t* p, bool ok) {
    bf16x8 z;
#pragma unroll
    for (int i = 0; i < 8; ++i) z[i] = (bf16_t)0.f;
    return ok ? *reinterpret_cast<const bf16x8*>(p) : z;
}

// LDS tiles: one copy [64 rows][D] per tensor serves BOTH operand forms - a straight
// 16-byte read gives a lane 8 consecutive columns of its row (contraction over columns), the
// transposing read gives it 4 consecutive rows of its column (contraction over rows).  The
// 16-byte chunk c of row r sits at c ^ usw(r); usw is chosen so that both read patterns are
// conflict-free on the 64 banks: a straight read touches 16 consecutive rows at one chunk
// index, a transposing read 4 consecutive rows at 4 consecutive chunks.
template <int D> __device__ __forceinline__ int usw(int r) {
    if (D == 64) { const int h = (r >> 1) & 7; return ((h & 1) << 2) | (h & 2) | (h >> 2); }   // 128-byte rows: bit reversal of r/2
    return ((r & 3) << 2) | ((r >> 2) & 3);                                                     // 256-byte rows
}
template <int D>
__device__ __forceinline__ void dma_utile(const bf16_t* __restrict__ g, int ld, int row0, int row_last, unsigned lds_base,
                                          int wave, int lane) {
    constexpr int KB = 64 * D * 2 / 1024, CPR = D / 8;
#pragma unroll
    for (int n0 = 0; n0 < KB; n0 += NT / WAVE) {
        const int n = n0 + wave;
        const int row = n * (64 / CPR) + lane / CPR;
        const int col = ((lane % CPR) ^ usw<D>(row)) << 3;
        lds_dma16(g + (size_t)min(row0 + row, row_last) * ld + col, lds_base + n * 1024);
    }
}
// rows = `row`, contraction step kk over 16 columns
template <int D>
__device__ __forceinline__ bf16x8 frag_us(const bf16_t* tile, int row, int kk, int g) {
    return *reinterpret_cast<const bf16x8*>(tile + row * D + (((kk * 2 + g) ^ usw<D>(row)) << 3));
}
// rows = columns col0 + lane%32 of the tile, contraction over tile rows of 16-step J, in the
// slot order {4g..4g+3, 8+4g..8+4g+3} of a transposed score tile
template <int D>
__device__ __forceinline__ bf16x8 frag_ut(const bf16_t* tile, int col0, int J, int lane) {
    typedef bf16x4 __attribute__((address_space(3))) * lds_v4;
    const int i = lane & 15, g = lane >> 5;
    const int c = (((col0 >> 4) + ((lane >> 4) & 1)) << 1) + ((i >> 1) & 1);
    const int r = 16 * J + 4 * g + (i >> 2);
    const bf16_t* p0 = tile + r * D + ((c ^ usw<D>(r)) << 3) + ((i & 1) << 2);
    const bf16_t* p1 = tile + (r + 8) * D + ((c ^ usw<D>(r + 8)) << 3) + ((i & 1) << 2);
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_v4)p0);
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_v4)p1);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int first) {
    bf16x8 o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (bf16_t)v[first + i];
    return o;
}

__device__ __forceinline__ float xor32(float v) { return __shfl_xor(v, 32, WAVE); }

// ------------------------------------------------------------------- forward
// Which 128-row tile (by rank: 0 = the one with the most work under the causal mask), head and
// sequence a workgroup of the 1-D grid takes; false for the padding workgroups.  Workgroup ids
// go round-robin over the 8 XCDs, so the (sequence, head) pair is chosen by id mod 8 first (the
// pair count is padded to a multiple of 8): all tiles of a pair then run on one XCD and its K, V
// (or Q, dO) are fetched into one L2 instead of up to eight.  Without a mask a group of 8 pairs
// works through its tiles before the next group starts.  With the causal mask a tile's work grows
// with its position, so the longest tiles of ALL pairs are dispatched first (rank slowest).
template <bool CAUSAL>
__device__ __forceinline__ bool attn_tile_of(int bid, int S, int heads, int batch, int& rank, int& h, int& b) {
    const int T = (S + 127) / 128;
    const int pairs = heads * batch, padded = (pairs + 7) & ~7;
    int p;
    if constexpr (CAUSAL) {
        p = bid % padded;
        rank = bid / padded;
    } else {
        const int j = bid >> 3;
        rank = j % T;
        p = (j / T) * 8 + (bid & 7);
    }
    h = p % heads; b = p / heads;
    return p < pairs;
}
inline unsigned attn_grid(const AttnArgs& a) {
    const unsigned T = (a.seq + 127) / 128, pairs = (unsigned)a.heads * a.batch;
    return T * ((pairs + 7) & ~7u);
}

// The forward moves its K and V tiles global -> LDS directly (lds_dma16), one tile ahead of
// the matrix cores, with no staging registers and no transposition work: K is read straight
// (contraction over the head dimension), V with the transposing read (contraction over keys).
// Rows beyond the sequence are fetched from its last row (finite data): their scores are
// masked, so they contribute exact zeros.
template <int D, bool CAUSAL>
__global__ __launch_bounds__(NT) void attn_fwd_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ ctx,
                                                      float* __restrict__ lse, int S, int heads, int batch,
                                                      float scale_log2e) {
    constexpr int KS = D / 16, OT = D / 32;
    __shared__ __attribute__((aligned(16))) bf16_t Ks[2][64 * D];
    __shared__ __attribute__((aligned(16))) bf16_t Vs[2][64 * D];
    const int H = heads * D, ld = 3 * H, bid = (int)blockIdx.x;
    int rank, h, b;
    if (!attn_tile_of<CAUSAL>(bid, S, heads, batch, rank, h, b)) return;
    const int q0 = ((S + 127) / 128 - 1 - rank) * 128;       // longest (causal) tiles first
    const bf16_t* base = qkv + (size_t)b * S * ld + h * D;
    const bf16_t* Kg = base + H;
    const bf16_t* Vg = base + 2 * H;
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wq0 = q0 + wave * 32, qrow = wq0 + l32;
    const unsigned ks0 = lds_address(Ks), vs0 = lds_address(Vs);
    constexpr unsigned TILE_BYTES = 64 * D * 2;

    const int kv_end = CAUSAL ? min(S, q0 + 128) : S;
    const int ntiles = (kv_end + 63) / 64;
    dma_utile<D>(Kg, ld, 0, S - 1, ks0, wave, lane);
    dma_utile<D>(Vg, ld, 0, S - 1, vs0, wave, lane);

    bf16x8 qf[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) qf[kk] = load_frag(base + (size_t)qrow * ld + kk * 16 + g * 8, qrow < S);

    f32x16 o[OT];
#pragma unroll
    for (int t = 0; t < OT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[t][r] = 0.f;
    float m = NEG_BIG, lsum = 0.f;

    // one step of the key loop; the LDS buffer index is a compile-time constant so that every LDS
    // address is the lane's base plus an immediate
    auto step = [&](int t, auto buf_c) {
        constexpr int buf = decltype(buf_c)::value;
        const int k0 = t * 64;
        wait_vmcnt<0>();                   // this wavefront's share of tile t has landed
        __syncthreads();                   // everyone's has; and tile t-1 is consumed, so its buffer is free
        if (t + 1 < ntiles) {
            dma_utile<D>(Kg, ld, k0 + 64, S - 1, ks0 + (buf ^ 1) * TILE_BYTES, wave, lane);
            dma_utile<D>(Vg, ld, k0 + 64, S - 1, vs0 + (buf ^ 1) * TILE_BYTES, wave, lane);
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
                    s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_us<D>(Ks[buf], kt * 32 + l32, kk, g), qf[kk],
                                                                    s[kt], 0, 0, 0);
            }
            // tiles that reach past the sequence or the diagonal mask key by key; the others skip it
            // (wavefront-uniform branch)
            if ((k0 + 63 >= S) || (CAUSAL && k0 + 63 > wq0)) {
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = k0 + kt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                        if (key >= S || (CAUSAL && key > qrow)) s[kt][r] = NEG_BIG;
                    }
            }
            // running maximum in the scaled (log2) domain; the scale is positive, so it commutes with max
            float mx = NEG_BIG;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kt][r]);
            mx = fmaxf(mx, xor32(mx)) * scale_log2e;
            const float m_new = fmaxf(m, mx);
            float rs = 0.f;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    // hardware exp2: arguments are <= 0 here, and flushing tiny results to zero is harmless
                    const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][r], scale_log2e, -m_new));
                    s[kt][r] = p;
                    rs += p;
                }
            rs += xor32(rs);
            // the accumulators only need rescaling when some row's maximum moved
            if (__builtin_amdgcn_ballot_w64(m_new != m)) {
                const float alpha = __builtin_amdgcn_exp2f(m - m_new);
                lsum *= alpha;
#pragma unroll
                for (int t2 = 0; t2 < OT; ++t2)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[t2][r] *= alpha;
            }
            lsum += rs;
            m = m_new;
#pragma unroll
            for (int J = 0; J < 4; ++J) {
                const bf16x8 pf = pack8(s[J >> 1], (J & 1) * 8);
#pragma unroll
                for (int t2 = 0; t2 < OT; ++t2)
                    o[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_ut<D>(Vs[buf], t2 * 32, J, lane), pf, o[t2], 0, 0, 0);
            }
        }
    };
    for (int t = 0; t < ntiles; t += 2) {
        step(t, std::integral_constant<int, 0>{});
        if (t + 1 < ntiles) step(t + 1, std::integral_constant<int, 1>{});
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
// dK, dV of 128 keys (32 per wavefront), looping over 64-query tiles.
//   S  = Q K^T (queries x keys)   P = exp2(S c - lse2)     dP = dO V^T
//   dS = P (dP - delta)           dV^T += dO^T P           dK^T += Q^T dS (then * 1/sqrt(d))
// The Q and dO tiles of the next step travel global -> LDS (lds_dma16) while the matrix cores
// work on the current one; each 32-query half of a tile is finished (scores to dK/dV) before
// the next starts, which keeps the live score registers at 32.  Rows beyond the sequence
// repeat its last row; their P is masked to zero.
// LDS of one backward workgroup: two tensors x two stages of [64][D] tiles, and (dK/dV role) the
// statistics of a tile's 64 queries.
template <int D> struct AttnBwdLds {
    bf16_t t0[2][64 * D], t1[2][64 * D];
    float lse2[2][64], dl[2][64];
};

template <int D, bool CAUSAL>
__device__ __forceinline__ void attn_bwd_dkv_role(AttnBwdLds<D>& sm, int bid, const bf16_t* __restrict__ qkv,
                                                  const bf16_t* __restrict__ dctx, const float* __restrict__ lse,
                                                  const float* __restrict__ delta, bf16_t* __restrict__ dqkv, int S,
                                                  int heads, int batch, float scale) {
    constexpr int KS = D / 16, OT = D / 32;
    constexpr unsigned TILE_BYTES = 64 * D * 2;
    bf16_t (&Qs)[2][64 * D] = sm.t0;
    bf16_t (&Os)[2][64 * D] = sm.t1;
    float (&lse2)[2][64] = sm.lse2;
    float (&dl)[2][64] = sm.dl;
    const int H = heads * D, ld = 3 * H;
    int rank, h, b;
    if (!attn_tile_of<CAUSAL>(bid, S, heads, batch, rank, h, b)) return;
    const int j0 = rank * 128;             // the first keys meet the most queries
    const bf16_t* base = qkv + (size_t)b * S * ld + h * D;
    const bf16_t* dOg = dctx + (size_t)b * S * H + h * D;
    const size_t stat0 = ((size_t)b * heads + h) * S;
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wj0 = j0 + wave * 32, jrow = wj0 + l32;
    const float c2 = scale * LOG2E;
    const unsigned qs0 = lds_address(Qs), os0 = lds_address(Os);

    const int qt0 = CAUSAL ? j0 / 64 : 0;
    const int ntiles = (S + 63) / 64;
    float stat = 0.f;                      // lse (threads 0..63) or delta (threads 64..127) of the next tile
    auto fetch = [&](int t, int buf) {
        const int i0 = t * 64;
        dma_utile<D>(base, ld, i0, S - 1, qs0 + buf * TILE_BYTES, wave, lane);
        dma_utile<D>(dOg, H, i0, S - 1, os0 + buf * TILE_BYTES, wave, lane);
        if (tid < 128) {
            const int i = i0 + (tid & 63);
            stat = i < S ? (tid < 64 ? lse[stat0 + i] * LOG2E : delta[stat0 + i]) : 0.f;
        }
    };
    fetch(qt0, 0);

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

    auto step = [&](int t, auto buf_c) {        // LDS buffer index at compile time: addresses become base + immediate
        constexpr int buf = decltype(buf_c)::value;
        const int i0 = t * 64;
        wait_vmcnt<0>();                   // this wavefront's share of tile t (and its statistics) has arrived
        if (tid < 64) lse2[buf][tid] = stat;
        else if (tid < 128) dl[buf][tid - 64] = stat;
        __syncthreads();                   // tile t complete in LDS; tile t-1 consumed by everyone
        if (t + 1 < ntiles) fetch(t + 1, buf ^ 1);
        const bf16_t* Qt = Qs[buf];
        const bf16_t* Ot = Os[buf];
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
                    p = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_us<D>(Qt, it * 32 + l32, kk, g), kf[kk], p, 0, 0, 0);
                    dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_us<D>(Ot, it * 32 + l32, kk, g), vf[kk], dp, 0, 0, 0);
                }
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int il = it * 32 + 8 * r4 + 4 * g;       // 4 consecutive queries
                    const float4 l4 = *reinterpret_cast<const float4*>(&lse2[buf][il]);
                    const float4 d4 = *reinterpret_cast<const float4*>(&dl[buf][il]);
                    const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int r = r4 * 4 + c;
                        p[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(p[r], c2, -lv[c]));     // hardware exp2
                        dp[r] -= dv4[c];
                    }
                }
                if (edge) {                               // wavefront-uniform: only tiles on an edge mask
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int i = i0 + it * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                        if (i >= S || (CAUSAL && i < jrow)) p[r] = 0.f;
                    }
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) dp[r] *= p[r];
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int J = it * 2 + j;
                    const bf16x8 pf = pack8(p, j * 8);
                    const bf16x8 dsf = pack8(dp, j * 8);
#pragma unroll
                    for (int t2 = 0; t2 < OT; ++t2) {
                        dv[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_ut<D>(Ot, t2 * 32, J, lane), pf, dv[t2], 0, 0, 0);
                        dk[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_ut<D>(Qt, t2 * 32, J, lane), dsf, dk[t2], 0, 0, 0);
                    }
                }
            }
        }
    };
    for (int t = qt0; t < ntiles; t += 2) {
        step(t, std::integral_constant<int, 0>{});
        if (t + 1 < ntiles) step(t + 1, std::integral_constant<int, 1>{});
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
// FORM_DELTA: delta = rowsum(dO * O) of the workgroup's queries is formed here (from the dO
// fragments the wavefront holds anyway and the same pieces of O) and written out for the dK/dV
// kernel that follows; otherwise it is read (attn_delta_kernel has run).
template <int D, bool CAUSAL, bool FORM_DELTA>
__device__ __forceinline__ void attn_bwd_dq_role(AttnBwdLds<D>& sm, int bid, const bf16_t* __restrict__ qkv,
                                                 const bf16_t* __restrict__ dctx, const bf16_t* __restrict__ ctx,
                                                 const float* __restrict__ lse, float* __restrict__ delta,
                                                 bf16_t* __restrict__ dqkv, int S, int heads, int batch, float scale) {
    constexpr int KS = D / 16, OT = D / 32;
    constexpr unsigned TILE_BYTES = 64 * D * 2;
    bf16_t (&Ks)[2][64 * D] = sm.t0;
    bf16_t (&Vs)[2][64 * D] = sm.t1;
    const int H = heads * D, ld = 3 * H;
    int rank, h, b;
    if (!attn_tile_of<CAUSAL>(bid, S, heads, batch, rank, h, b)) return;
    const int q0 = ((S + 127) / 128 - 1 - rank) * 128;
    const bf16_t* base = qkv + (size_t)b * S * ld + h * D;
    const bf16_t* dOg = dctx + (size_t)b * S * H + h * D;
    const size_t stat0 = ((size_t)b * heads + h) * S;
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wq0 = q0 + wave * 32, qrow = wq0 + l32;
    const float c2 = scale * LOG2E;
    const unsigned ks0 = lds_address(Ks), vs0 = lds_address(Vs);

    const int kv_end = CAUSAL ? min(S, q0 + 128) : S;
    const int ntiles = (kv_end + 63) / 64;
    auto fetch = [&](int t, int buf) {
        dma_utile<D>(base + H, ld, t * 64, S - 1, ks0 + buf * TILE_BYTES, wave, lane);
        dma_utile<D>(base + 2 * H, ld, t * 64, S - 1, vs0 + buf * TILE_BYTES, wave, lane);
    };
    fetch(0, 0);

    bf16x8 qf[KS], of[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
        qf[kk] = load_frag(base + (size_t)qrow * ld + kk * 16 + g * 8, qrow < S);
        of[kk] = load_frag(dOg + (size_t)qrow * H + kk * 16 + g * 8, qrow < S);
    }
    const float my_lse2 = qrow < S ? lse[stat0 + qrow] * LOG2E : 0.f;
    float my_dl = 0.f;
    if constexpr (FORM_DELTA) {
        // the lane pair (l, l^32) holds the whole row of dO
        const bf16_t* Og = ctx + (size_t)b * S * H + h * D;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            const bf16x8 cf = load_frag(Og + (size_t)qrow * H + kk * 16 + g * 8, qrow < S);
#pragma unroll
            for (int e = 0; e < 8; ++e) my_dl += (float)of[kk][e] * (float)cf[e];
        }
        my_dl += xor32(my_dl);
        if (g == 0 && qrow < S) delta[stat0 + qrow] = my_dl;
    } else {
        my_dl = qrow < S ? delta[stat0 + qrow] : 0.f;
    }
    f32x16 dq[OT];
#pragma unroll
    for (int t = 0; t < OT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) dq[t][r] = 0.f;

    auto step = [&](int t, auto buf_c) {        // LDS buffer index at compile time
        constexpr int buf = decltype(buf_c)::value;
        const int k0 = t * 64;
        wait_vmcnt<0>();
        __syncthreads();
        if (t + 1 < ntiles) fetch(t + 1, buf ^ 1);
        const bf16_t* Kt = Ks[buf];
        const bf16_t* Vt = Vs[buf];
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
                    p = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_us<D>(Kt, kt * 32 + l32, kk, g), qf[kk], p, 0, 0, 0);
                    dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_us<D>(Vt, kt * 32 + l32, kk, g), of[kk], dp, 0, 0, 0);
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) p[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(p[r], c2, -my_lse2));   // hardware exp2
                if (edge) {                               // wavefront-uniform: only tiles on an edge mask
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = k0 + kt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                        if (key >= S || (CAUSAL && key > qrow)) p[r] = 0.f;
                    }
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) dp[r] = p[r] * (dp[r] - my_dl);
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const bf16x8 dsf = pack8(dp, j * 8);
#pragma unroll
                    for (int t2 = 0; t2 < OT; ++t2)
                        dq[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_ut<D>(Kt, t2 * 32, kt * 2 + j, lane), dsf, dq[t2], 0, 0, 0);
                }
            }
        }
    };
    for (int t = 0; t < ntiles; t += 2) {
        step(t, std::integral_constant<int, 0>{});
        if (t + 1 < ntiles) step(t + 1, std::integral_constant<int, 1>{});
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

// delta[sequence, head, position] = sum over the head dimension of dO * O: one lane per 8 elements
// (16 bytes of each tensor), the D / 8 lanes of a (token, head) pair side by side.
template <int D>
__global__ __launch_bounds__(NT) void attn_delta_kernel(const bf16_t* __restrict__ dctx, const bf16_t* __restrict__ ctx,
                                                        float* __restrict__ delta, int S, int heads, int batch) {
    constexpr int LPH = D / 8;                                   // lanes per (token, head)
    const size_t H = (size_t)heads * D, chunks = (size_t)batch * S * heads * LPH;
    const size_t c = (size_t)blockIdx.x * NT + threadIdx.x;
    float v = 0.f;
    if (c < chunks) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(dctx + c * 8);
        const bf16x8 o = *reinterpret_cast<const bf16x8*>(ctx + c * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) v += (float)a[e] * (float)o[e];
    }
#pragma unroll
    for (int off = LPH / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, WAVE);
    if (c < chunks && (c % LPH) == 0) {
        const size_t th = c / LPH, token = th / heads, h = th % heads;      // token = sequence * S + position
        delta[((token / S) * heads + h) * S + token % S] = v;
    }
    (void)H;
}

// Both backward kernels in one launch: workgroups come in groups of 8 (one per XCD), the groups
// alternate between the dK/dV role and the dQ role, and a workgroup's number within its role keeps
// its id mod 8, so that a (sequence, head) pair's tiles of both roles meet in one L2.  The two
// roles are independent (delta comes from attn_delta_kernel), so with few pairs - where one role
// alone leaves the chip half empty and its longest causal tile sets the time - each fills the
// other's gaps.
template <int D, bool CAUSAL>
__global__ __launch_bounds__(NT) void attn_bwd_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dctx,
                                                      const float* __restrict__ lse, const float* __restrict__ delta,
                                                      bf16_t* __restrict__ dqkv, int S, int heads, int batch, float scale) {
    __shared__ __attribute__((aligned(16))) AttnBwdLds<D> sm;
    const int blk = (int)blockIdx.x;
    const int role = (blk >> 3) & 1, bid = ((blk >> 4) << 3) | (blk & 7);
    if (role == 0) attn_bwd_dkv_role<D, CAUSAL>(sm, bid, qkv, dctx, lse, delta, dqkv, S, heads, batch, scale);
    else attn_bwd_dq_role<D, CAUSAL, false>(sm, bid, qkv, dctx, nullptr, lse, const_cast<float*>(delta), dqkv, S, heads, batch, scale);
}

// The roles as launches of their own, dQ first (it forms delta): for many pairs, where each role
// fills the chip by itself and the merged kernel's register count (that of its larger role) would
// only cost the other role wavefronts per SIMD.
template <int D, bool CAUSAL>
__global__ __launch_bounds__(NT) void attn_bwd_dq_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dctx,
                                                         const bf16_t* __restrict__ ctx, const float* __restrict__ lse,
                                                         float* __restrict__ delta, bf16_t* __restrict__ dqkv, int S,
                                                         int heads, int batch, float scale) {
    __shared__ __attribute__((aligned(16))) AttnBwdLds<D> sm;
    attn_bwd_dq_role<D, CAUSAL, true>(sm, (int)blockIdx.x, qkv, dctx, ctx, lse, delta, dqkv, S, heads, batch, scale);
}
template <int D, bool CAUSAL>
__global__ __launch_bounds__(NT) void attn_bwd_dkv_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dctx,
                                                          const float* __restrict__ lse, const float* __restrict__ delta,
                                                          bf16_t* __restrict__ dqkv, int S, int heads, int batch,
                                                          float scale) {
    __shared__ __attribute__((aligned(16))) AttnBwdLds<D> sm;
    attn_bwd_dkv_role<D, CAUSAL>(sm, (int)blockIdx.x, qkv, dctx, lse, delta, dqkv, S, heads, batch, scale);
}

int check(const AttnArgs& a) {
    if (!attention_mfma_supports(a)) return fail(CHIMERA_EINVAL, "matrix-core attention: unsupported shape (head_dim %d)", a.head_dim);
    return CHIMERA_OK;
}

}  // namespace

bool attention_mfma_supports(const AttnArgs& a) {
    if (a.head_dim != 64 && a.head_dim != 128) return false;
    if (a.batch < 1 || a.seq < 1 || a.heads < 1 || a.batch > 65535 || a.heads > 65535) return false;
    if (((unsigned long long)a.heads * a.batch + 7) * ((a.seq + 127) / 128) >= (1ull << 30)) return false;   // 1-D grid
    if ((uintptr_t)a.qkv & 15) return false;
    return true;
}

int attention_fwd_mfma(const AttnArgs& a, void* stream) {
    if (int rc = check(a)) return rc;
    if ((uintptr_t)a.ctx & 7) return fail(CHIMERA_EINVAL, "ctx must be 8-byte aligned");
    const dim3 grid(attn_grid(a)), block(NT);
    const float sl2 = LOG2E / sqrtf((float)a.head_dim);
    hipStream_t s = (hipStream_t)stream;
#define ATTN_FWD(D, C)                                                                                            \
    hipLaunchKernelGGL((attn_fwd_kernel<D, C>), grid, block, 0, s, (const bf16_t*)a.qkv, (bf16_t*)a.ctx, a.lse, a.seq, \
                       a.heads, a.batch, sl2)
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
    const dim3 block(NT);
    const dim3 grid(attn_grid(a)), grid2(2 * attn_grid(a));    // one role / both roles; attn_grid is a multiple of 8
    const size_t chunks = (size_t)a.batch * a.seq * a.heads * (a.head_dim / 8);
    const dim3 dgrid((unsigned)((chunks + NT - 1) / NT));
    const float scale = 1.0f / sqrtf((float)a.head_dim);
    // Few (sequence, head) pairs: one launch with both roles (measured: 448 workgroups per role
    // 58 -> 53 us, 256 per role at head dim 128 149 -> 119 us; 512 and more per role are faster apart).
    const bool merged = attn_grid(a) <= 480;
#define ATTN_BWD(D, C)                                                                                              \
    do {                                                                                                            \
        if (merged) {                                                                                               \
            hipLaunchKernelGGL((attn_delta_kernel<D>), dgrid, block, 0, s, (const bf16_t*)a.dctx, (const bf16_t*)a.ctx, \
                               a.delta, a.seq, a.heads, a.batch);                                                   \
            hipLaunchKernelGGL((attn_bwd_kernel<D, C>), grid2, block, 0, s, (const bf16_t*)a.qkv, (const bf16_t*)a.dctx, \
                               a.lse, a.delta, (bf16_t*)a.dqkv, a.seq, a.heads, a.batch, scale);                     \
        } else {                                                                                                    \
            hipLaunchKernelGGL((attn_bwd_dq_kernel<D, C>), grid, block, 0, s, (const bf16_t*)a.qkv, (const bf16_t*)a.dctx, \
                               (const bf16_t*)a.ctx, a.lse, a.delta, (bf16_t*)a.dqkv, a.seq, a.heads, a.batch, scale); \
            hipLaunchKernelGGL((attn_bwd_dkv_kernel<D, C>), grid, block, 0, s, (const bf16_t*)a.qkv, (const bf16_t*)a.dctx, \
                               a.lse, a.delta, (bf16_t*)a.dqkv, a.seq, a.heads, a.batch, scale);                    \
        }                                                                                                           \
    } while (0)
    if (a.head_dim == 64) { if (a.causal) ATTN_BWD(64, true); else ATTN_BWD(64, false); }
    else { if (a.causal) ATTN_BWD(128, true); else ATTN_BWD(128, false); }
#undef ATTN_BWD
    CHIMERA_LAUNCH_CHECK("attention backward");
    return CHIMERA_OK;
}

}  // namespace chimera
