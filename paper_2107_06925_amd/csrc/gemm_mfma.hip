// bf16 GEMM on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16), float
// accumulation, for the three products of a linear layer:
//   forward  Y  = X W      A k-contiguous, B stored [k, n]
//   dgrad    dX = dY W^T   A k-contiguous, B k-contiguous
//   wgrad    dW += X^T dY  A stored [k, m], B stored [k, n]  (k = tokens)
//
// One workgroup of 4 or 8 wavefronts computes a BM x BN tile; each wavefront
// owns a 128x64 or 64x64 part of it as a grid of 32x32 MFMA tiles whose
// accumulators never leave the registers.  The k loop moves BK = 64 at a time
// through LDS with two buffers: while the matrix cores work on buffer b, the
// loads of the next k step are already in flight to registers and are written
// to buffer b^1 afterwards, one barrier per step.
//
// An operand that is k-contiguous in memory (X in the forward, both operands of
// dgrad) sits in LDS as [row][k], 128 bytes per row, and lane l reads its MFMA
// operand - row l%32, the 8 consecutive k of chunk 2*kk + l/32 - with one
// 16-byte load.  Chunk c of row r is stored at c ^ (r & 7) ^ ((r >> 3) & 7), so the
// 8 rows a read touches per bank cycle fall on 8 different bank groups.
// An operand whose OTHER index is contiguous in memory (W in the forward, both
// operands of wgrad) is copied to LDS as it lies in memory, [k][row], and the
// transposition is done by the LDS hardware: ds_read_b64_tr_b16 hands lane i of
// each 16-lane group the i-th 16-bit element of the data addressed by lanes
// 4e + i/4 (e = 0..3), i.e. column i of a 4 x 16 block - four consecutive k of one
// row.  Two such reads give the same 8 k values the other flavour gets from one
// 16-byte load.  The 32-byte column blocks of row k are stored at block ^ 2(k & 3):
// one bank cycle serves 32 lanes = two adjacent column blocks x four rows, and this
// puts those eight 32-byte pieces on eight different bank groups (measured: without
// it half of the LDS cycles of the wgrad kernel were bank conflicts).  No transposed
// copy of any activation or weight exists in HBM, and no data is shuffled in
// registers.
//
// Workgroups are renumbered so that each of the 8 XCDs (own L2 each; the
// hardware deals consecutive workgroup ids round-robin over them) works on a
// contiguous range of tiles, and tiles are walked in groups of 8 tile rows so
// that the tiles in flight on one XCD share operand panels in its L2.
#include "device.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <type_traits>

namespace chimera {

namespace {

typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BK = 64;
constexpr int GROUP_M = 8;       // tile rows per raster group
constexpr int NUM_CUS = 256;     // compute units of an MI355X
constexpr size_t SPLITK_COUNTER_BYTES = 4096;

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ (row & 7) ^ ((row >> 3) & 7); }

typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));

// LDS element offset of the 16-byte chunk `ic` (8 rows) of k-row `k` in a [BK][ROWS] tile
template <int ROWS> __device__ __forceinline__ int mc_off(int k, int ic) {
    return k * ROWS + (((ic >> 1) ^ ((k & 3) << 1)) << 4) + ((ic & 1) << 3);
}

template <int ROWS, int NT, bool KC> struct Staged {
    static constexpr int N = ROWS * (BK / 8) / NT;     // 16-byte chunks per thread
    uint4 v[N];
    unsigned ok;     // bit i: v[i] lies inside the matrix (others are zeroed when written to LDS)
};

// global -> registers for one operand tile of ROWS rows x BK k values.
// KC: element (row, k) at base[row * ld + k].  !KC: at base[k * ld + row].
// Loads are unconditional (an out-of-range piece reads element 0 instead and is
// zeroed later), so no branch separates the loads of different k steps.
template <int ROWS, int NT, bool KC>
__device__ __forceinline__ void load_tile(Staged<ROWS, NT, KC>& st, const bf16_t* __restrict__ base, int ld, int row0,
                                          int nrows, int k0, int K, int tid) {
    constexpr int CPT = ROWS * (BK / 8) / NT;
    unsigned okm = 0;
#pragma unroll
    for (int it = 0; it < CPT; ++it) {
        const int c = tid + it * NT;
        bool ok;
        unsigned off;
        if constexpr (KC) {
            const int gr = row0 + (c >> 3), gk = k0 + (c & 7) * 8;
            ok = gr < nrows && gk < K;
            off = (unsigned)gr * (unsigned)ld + (unsigned)gk;
        } else {
            const int gk = k0 + c / (ROWS / 8), gi = row0 + (c % (ROWS / 8)) * 8;
            ok = gk < K && gi < nrows;
            off = (unsigned)gk * (unsigned)ld + (unsigned)gi;
        }
        st.v[it] = *reinterpret_cast<const uint4*>(base + (ok ? off : 0u));
        okm |= (ok ? 1u : 0u) << it;
    }
    st.ok = okm;
}

__device__ __forceinline__ uint4 keep_if(const uint4& q, unsigned mask, int bit) {
    const bool ok = (mask >> bit) & 1u;
    return make_uint4(ok ? q.x : 0u, ok ? q.y : 0u, ok ? q.z : 0u, ok ? q.w : 0u);
}

// registers -> LDS: [ROWS][BK] (KC) or [BK][ROWS] (!KC), swizzled as described above.
template <int ROWS, int NT, bool KC>
__device__ __forceinline__ void store_tile(const Staged<ROWS, NT, KC>& st, bf16_t* lds, int tid) {
    constexpr int CPT = ROWS * (BK / 8) / NT;
#pragma unroll
    for (int it = 0; it < CPT; ++it) {
        const int c = tid + it * NT;
        int off;
        if constexpr (KC) { const int row = c >> 3, kc = c & 7; off = row * BK + swz(row, kc) * 8; }
        else off = mc_off<ROWS>(c / (ROWS / 8), c % (ROWS / 8));
        *reinterpret_cast<uint4*>(lds + off) = keep_if(st.v[it], st.ok, it);
    }
}

// MFMA operand of lane `lane` for the 32 rows starting at r0 and the 16 k values of step kk.
template <int ROWS, bool KC>
__device__ __forceinline__ bf16x8 read_frag(const bf16_t* lds, int r0, int kk, int lane) {
    if constexpr (KC) {
        const int row = r0 + (lane & 31);
        return *reinterpret_cast<const bf16x8*>(lds + row * BK + swz(row, kk * 2 + (lane >> 5)) * 8);
    } else {
        const int i = lane & 15, blk = (r0 >> 4) + ((lane >> 4) & 1);      // 16-row column block of this lane group
        const int k = kk * 16 + (lane >> 5) * 8 + (i >> 2);                // row this lane addresses (first read)
        typedef bf16x4 __attribute__((address_space(3))) * lds_v4;
        const bf16_t* p0 = lds + k * ROWS + ((blk ^ ((k & 3) << 1)) << 4) + ((i & 3) << 2);
        const bf16_t* p1 = p0 + 4 * ROWS;                                  // rows k+4..k+7: same swizzle
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_v4)p0);
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_v4)p1);
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
}

// Epilogue of one wavefront.  Accumulator register r of lane l holds
// C[8*(r/4) + 4*(l/32) + r%4][l%32] of its 32x32 tile: one column per lane, which
// would mean 2-byte global accesses.  So each 32-row band of the wavefront's
// tile goes through a wavefront-private LDS slab ([32][WN + 8] floats, the
// padding keeps the two lane halves on different banks) and comes back as 8
// consecutive columns per lane; bias, residual, GeLU operands and the results
// then move in 16-byte pieces, 128 contiguous bytes per 8 lanes.
template <int TN> struct EpiSlab {
    static constexpr int WN = TN * 32, STRIDE = WN + 8, FLOATS = 32 * STRIDE;
};

__device__ __forceinline__ void load8(const bf16_t* p, float* o) { load_vec<bf16_t>(p, o); }
__device__ __forceinline__ void load8(const float* p, float* o) { load_vec<float>(p, o); load_vec<float>(p + 4, o + 4); }
__device__ __forceinline__ void store8(bf16_t* p, const float* v) { store_vec<bf16_t>(p, v); }
__device__ __forceinline__ void store8(float* p, const float* v) { store_vec<float>(p, v); store_vec<float>(p + 4, v + 4); }

// 8 consecutive elements as they come from memory (one or two 16-byte pieces), widened later:
// what the epilogue requests ahead of time.
template <typename T> struct Raw8;
template <> struct Raw8<bf16_t> {
    uint4 q;
    __device__ __forceinline__ void load(const bf16_t* p) { q = *reinterpret_cast<const uint4*>(p); }
    __device__ __forceinline__ void unpack(float* o) const {
        const unsigned w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) { o[2 * i] = __uint_as_float(w[i] << 16); o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u); }
    }
};
template <> struct Raw8<float> {
    float4 lo, hi;
    __device__ __forceinline__ void load(const float* p) {
        lo = *reinterpret_cast<const float4*>(p); hi = *reinterpret_cast<const float4*>(p + 4);
    }
    __device__ __forceinline__ void unpack(float* o) const {
        o[0] = lo.x; o[1] = lo.y; o[2] = lo.z; o[3] = lo.w; o[4] = hi.x; o[5] = hi.y; o[6] = hi.z; o[7] = hi.w;
    }
};

// The operand an epilogue reads from memory besides the bias: the residual, the GeLU input, or
// the old value of a float accumulator.  Each band of 32 rows needs 32 / RPP pieces per lane, and
// a piece that is only requested when its turn comes costs a full memory round trip per pass
// (16 in a row for a 128-row wavefront tile: as long as a short k loop).  So the pieces of the
// next DEPTH bands are requested before the current band is worked on: all bands when the
// elements have 2 bytes, two bands when they are floats (registers).
template <int EPI, bool RF32, bool CF32, int TM, int TN>
__device__ __forceinline__ void epilogue(const f32x16 (&acc)[TM][TN], float* slab, int row_base, int col_base, int m,
                                         int n, const bf16_t* __restrict__ bias, const bf16_t* __restrict__ R,
                                         void* __restrict__ c, bf16_t* __restrict__ C2, int epi_flag, int lane) {
    constexpr int WN = EpiSlab<TN>::WN, STRIDE = EpiSlab<TN>::STRIDE;
    constexpr int CPR = WN / 8;                // 8-column pieces per row
    constexpr int RPP = 64 / CPR;              // rows covered by the 64 lanes at once
    constexpr int NP = 32 / RPP;               // passes per band of 32 rows
    constexpr bool READS_F32 = EPI == EPI_ACCUM_F32 || (EPI == EPI_BIAS_RESIDUAL && RF32);
    constexpr bool READS = EPI == EPI_BIAS_RESIDUAL || EPI == EPI_DGELU || EPI == EPI_ACCUM_F32;
    using RT = std::conditional_t<READS_F32, float, bf16_t>;
    constexpr int DEPTH = !READS ? 1 : (READS_F32 ? (TM < 2 ? TM : 2) : TM);
    bf16_t* C = (bf16_t*)c;
    float* Cf = (float*)c;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int pr = lane / CPR, pc = (lane % CPR) * 8;
    const int gcol = col_base + pc;
    const bool reads = READS && !(EPI == EPI_ACCUM_F32 && epi_flag);      // an overwriting accumulate reads nothing
    const RT* Rsrc = EPI == EPI_ACCUM_F32 ? reinterpret_cast<const RT*>(c) : reinterpret_cast<const RT*>(R);
    // pieces outside the matrix are requested from its last row / last piece (never used)
    const int lcol = min(gcol, n - 8);
    Raw8<RT> ahead[DEPTH][NP];
    auto request = [&](int a, auto slot_c) {
        constexpr int SLOT = decltype(slot_c)::value;
#pragma unroll
        for (int j = 0; j < NP; ++j) {
            const int grow = min(row_base + a * 32 + j * RPP + pr, m - 1);
            ahead[SLOT][j].load(Rsrc + (size_t)grow * n + lcol);
        }
    };
    float bv[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) bv[e] = 0.f;
    if constexpr (EPI == EPI_BIAS || EPI == EPI_BIAS_GELU || EPI == EPI_BIAS_RESIDUAL)
        if (gcol < n) load8(bias + gcol, bv);
    if constexpr (READS)
        if (reads) {
            request(0, std::integral_constant<int, 0>{});
            if constexpr (DEPTH > 1 && TM > 1) request(1, std::integral_constant<int, 1 % DEPTH>{});
            if constexpr (DEPTH > 2 && TM > 2) request(2, std::integral_constant<int, 2 % DEPTH>{});
            if constexpr (DEPTH > 3 && TM > 3) request(3, std::integral_constant<int, 3 % DEPTH>{});
        }
    static_assert(TM <= 4, "at most four bands per wavefront");
    auto band = [&](auto a_c) {
        constexpr int a = decltype(a_c)::value;
        constexpr int SLOT = a % DEPTH;
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) slab[(8 * (r >> 2) + 4 * lhi + (r & 3)) * STRIDE + b * 32 + l32] = acc[a][b][r];
        __builtin_amdgcn_s_waitcnt(0xc07f);                   // lgkmcnt(0): the slab is written (wavefront-private)
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < NP; ++j) {
            const int lr = j * RPP + pr;
            const int grow = row_base + a * 32 + lr;
            float v[8];
            load_vec<float>(slab + lr * STRIDE + pc, v);
            load_vec<float>(slab + lr * STRIDE + pc + 4, v + 4);
            float rv[8];
            if constexpr (READS) {
                if (reads) ahead[SLOT][j].unpack(rv);
                else
#pragma unroll
                    for (int e = 0; e < 8; ++e) rv[e] = 0.f;
            }
            if (grow >= m || gcol >= n) continue;
            const size_t idx = (size_t)grow * n + gcol;
            if constexpr (EPI == EPI_NONE) {
                store8(C + idx, v);
            } else if constexpr (EPI == EPI_BIAS) {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] += bv[e];
                store8(C + idx, v);
            } else if constexpr (EPI == EPI_BIAS_GELU) {
                float g[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] += bv[e];
                if (epi_flag) {                               // one wavefront-uniform branch per piece, not per element
#pragma unroll
                    for (int e = 0; e < 8; ++e) g[e] = gelu_f(v[e], 1);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) g[e] = gelu_f(v[e], 0);
                }
                store8(C + idx, v);
                store8(C2 + idx, g);
            } else if constexpr (EPI == EPI_BIAS_RESIDUAL) {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] += bv[e] + rv[e];
                if constexpr (CF32) store8(Cf + idx, v); else store8(C + idx, v);
            } else if constexpr (EPI == EPI_DGELU) {
                if (epi_flag) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] *= gelu_grad_f(rv[e], 1);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] *= gelu_grad_f(rv[e], 0);
                }
                store8(C + idx, v);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] += rv[e];    // rv = 0 when the result replaces C
                store8(Cf + idx, v);
            }
        }
        __builtin_amdgcn_wave_barrier();                      // all lanes have read the slab before it is rewritten
        if constexpr (READS && a + DEPTH < TM)
            if (reads) request(a + DEPTH, std::integral_constant<int, SLOT>{});
    };
    band(std::integral_constant<int, 0>{});
    if constexpr (TM > 1) band(std::integral_constant<int, 1>{});
    if constexpr (TM > 2) band(std::integral_constant<int, 2>{});
    if constexpr (TM > 3) band(std::integral_constant<int, 3>{});
}

template <int BM, int BN, int WGM, int WGN, int PF, bool A_KC, bool B_KC>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_bf16_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, const bf16_t* __restrict__ bias,
    const bf16_t* __restrict__ R, void* __restrict__ C, bf16_t* __restrict__ C2, int m, int n, int k, int lda,
    int ldb, int epi, int epi_flag, int res_types, int tiles_m, int tiles_n, int splits, float* __restrict__ slabs,
    unsigned* __restrict__ arrivals) {
    constexpr int NT = WGM * WGN * 64;
    constexpr int WM = BM / WGM, WN = BN / WGN;    // wavefront tile
    constexpr int TM = WM / 32, TN = WN / 32;      // MFMA tiles per wavefront
    __shared__ __attribute__((aligned(16))) bf16_t lds[2][(BM + BN) * BK];

    // workgroup id -> tile, XCD-contiguous then grouped raster
    // With split-K the grid holds `splits` workgroups per tile: split = blockIdx / tiles.
    const int nblk = tiles_m * tiles_n;
    const int split = blockIdx.x / nblk, bid = blockIdx.x % nblk;
    const int xcd = bid & 7, local = bid >> 3;
    const int pid = xcd * (nblk >> 3) + min(xcd, nblk & 7) + local;
    const int width = GROUP_M * tiles_n;
    const int first_m = (pid / width) * GROUP_M;
    const int gsz = min(tiles_m - first_m, GROUP_M);
    const int tile_m = first_m + (pid % width) % gsz;
    const int tile_n = (pid % width) / gsz;
    const int i0 = tile_m * BM, j0 = tile_n * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    // one k step of MFMA work out of LDS buffer `buf`
    auto compute = [&](int buf) {
        const bf16_t* As = lds[buf];
        const bf16_t* Bs = lds[buf] + BM * BK;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 af[TM], bfr[TN];
#pragma unroll
            for (int a = 0; a < TM; ++a) af[a] = read_frag<BM, A_KC>(As, wm0 + a * 32, kk, lane);
#pragma unroll
            for (int b = 0; b < TN; ++b) bfr[b] = read_frag<BN, B_KC>(Bs, wn0 + b * 32, kk, lane);
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bfr[b], acc[a][b], 0, 0, 0);
        }
    };
    auto fetch = [&](Staged<BM, NT, A_KC>& ra, Staged<BN, NT, B_KC>& rb, int kt) {
        load_tile<BM, NT, A_KC>(ra, A, lda, i0, m, kt * BK, k, tid);
        load_tile<BN, NT, B_KC>(rb, B, ldb, j0, n, kt * BK, k, tid);
    };
    auto stash = [&](const Staged<BM, NT, A_KC>& ra, const Staged<BN, NT, B_KC>& rb, int buf) {
        store_tile<BM, NT, A_KC>(ra, lds[buf], tid);
        store_tile<BN, NT, B_KC>(rb, lds[buf] + BM * BK, tid);
    };

    // Software pipeline: global loads run PF k steps ahead of the matrix cores in PF
    // register sets (a ring walked by an unrolled loop, so every index is static),
    // LDS runs one step ahead in two buffers, one barrier per step.
    // This workgroup's share of the k steps: [K0, K1).
    const int KT_all = (k + BK - 1) / BK;
    const int K0 = (int)((long)KT_all * split / splits), K1 = (int)((long)KT_all * (split + 1) / splits);
    const int KT = K1 - K0;
    Staged<BM, NT, A_KC> ra[PF];
    Staged<BN, NT, B_KC> rb[PF];
#pragma unroll
    for (int u = 0; u < PF; ++u)
        if (u < KT) fetch(ra[u], rb[u], K0 + u);
    stash(ra[0], rb[0], 0);
    __syncthreads();
    for (int kt = 0; kt < KT; kt += PF) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int step = kt + u;
            if (step >= KT) break;
            if (step + PF < KT) fetch(ra[u], rb[u], K0 + step + PF);      // set u was stashed one step ago
            compute(step & 1);
            if (step + 1 < KT) stash(ra[(u + 1) % PF], rb[(u + 1) % PF], (step + 1) & 1);
            __syncthreads();
        }
    }

    // Split-K: every workgroup of a tile writes its partial accumulators to its own slab
    // (thread-private order, 16-byte stores), then counts itself in.  Whoever arrives last
    // adds the slabs in split order - so the sum does not depend on who that is - and runs
    // the epilogue.  Nobody waits for anybody.
    if (splits > 1) {
        __shared__ int is_last;
        const size_t tile_elems = (size_t)BM * BN;
        float4* mine = reinterpret_cast<float4*>(slabs + ((size_t)split * nblk + pid) * tile_elems);
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    mine[((a * TN + b) * 4 + q) * NT + tid] =
                        make_float4(acc[a][b][4 * q], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]);
        __threadfence();                       // slab visible device-wide before the arrival count
        __syncthreads();
        if (tid == 0) is_last = atomicAdd(&arrivals[pid], 1u) == (unsigned)(splits - 1);
        __syncthreads();
        if (!is_last) return;
        __threadfence();                       // see the other workgroups' slabs
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
        for (int sp = 0; sp < splits; ++sp) {
            const float4* other = reinterpret_cast<const float4*>(slabs + ((size_t)sp * nblk + pid) * tile_elems);
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float4 v = other[((a * TN + b) * 4 + q) * NT + tid];
                        acc[a][b][4 * q] += v.x; acc[a][b][4 * q + 1] += v.y;
                        acc[a][b][4 * q + 2] += v.z; acc[a][b][4 * q + 3] += v.w;
                    }
        }
        if (tid == 0) arrivals[pid] = 0u;      // ready for the next launch on this stream
    }

    const int rb0 = i0 + wm0, cb0 = j0 + wn0;
    // the operand tiles in LDS are dead once every wavefront has left the k loop; each
    // wavefront then stages its output through its own slab there
    static_assert(sizeof(lds) >= (size_t)WGM * WGN * EpiSlab<TN>::FLOATS * sizeof(float), "LDS too small for the epilogue");
    __syncthreads();
    float* slab = reinterpret_cast<float*>(lds) + (size_t)(tid >> 6) * EpiSlab<TN>::FLOATS;
#define CHIMERA_EPI(E, RF, CF) epilogue<E, RF, CF, TM, TN>(acc, slab, rb0, cb0, m, n, bias, R, C, C2, epi_flag, lane)
    switch (epi) {
        case EPI_NONE: CHIMERA_EPI(EPI_NONE, false, false); break;
        case EPI_BIAS: CHIMERA_EPI(EPI_BIAS, false, false); break;
        case EPI_BIAS_GELU: CHIMERA_EPI(EPI_BIAS_GELU, false, false); break;
        case EPI_BIAS_RESIDUAL:                    // res_types: bit 0 = R is float, bit 1 = C is float
            if (res_types == 0) CHIMERA_EPI(EPI_BIAS_RESIDUAL, false, false);
            else if (res_types == 1) CHIMERA_EPI(EPI_BIAS_RESIDUAL, true, false);
            else if (res_types == 2) CHIMERA_EPI(EPI_BIAS_RESIDUAL, false, true);
            else CHIMERA_EPI(EPI_BIAS_RESIDUAL, true, true);
            break;
        case EPI_DGELU: CHIMERA_EPI(EPI_DGELU, false, false); break;
        default: CHIMERA_EPI(EPI_ACCUM_F32, false, false); break;
    }
#undef CHIMERA_EPI
}

// ---------------------------------------------------------------- async variant
// Same tiles, same LDS layouts, same MFMA loop, but the tiles travel global -> LDS
// without passing through registers (global_load_lds_dwordx4: lane i of a wavefront
// writes 16 bytes at LDS base + 16 i), into a ring of NS stages, so the loads of the
// next NS-1 k steps are in flight while the matrix cores work.  Because the LDS side of
// such a load is fixed, the swizzle is applied on the global side: the lane that owns
// LDS slot (row, position p) fetches the chunk that belongs there.  The instruction is
// issued through inline assembly so that the waits can be counted by hand
// (s_waitcnt vmcnt(n) with the younger stages still outstanding).
// Nothing can be zero-filled on this path: rows beyond the matrix are redirected to a
// valid row (they only feed outputs that are never stored), and k must be a multiple
// of BK (the caller falls back to the register-staged kernel otherwise).

// One output tile; `block_id` numbers the tiles of this product.  ONLY_EPI >= 0 compiles
// that epilogue alone.
template <int BM, int BN, int WGM, int WGN, int WGK, int NS, bool A_KC, bool B_KC, int ONLY_EPI>
__device__ __forceinline__ void gemm_async_tile(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, const bf16_t* __restrict__ bias,
    const bf16_t* __restrict__ R, void* __restrict__ C, bf16_t* __restrict__ C2, int m, int n, int k, int lda,
    int ldb, int epi, int epi_flag, int res_types, int tiles_m, int tiles_n, int group_m, int block_id,
    float* __restrict__ bsum = nullptr, bool xcd_remap = true) {
    constexpr int NT = WGM * WGN * WGK * 64;
    constexpr int KSUB = BK / 16 / WGK;                                   // 16-wide k slices per wavefront and step
    static_assert(KSUB >= 1 && KSUB * WGK * 16 == BK, "k split must divide the step");
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int CA = BM * (BK / 8) / NT, CB = BN * (BK / 8) / NT;      // 16-byte pieces per thread and stage
    constexpr int STAGE = (BM + BN) * BK;                                 // elements
    __shared__ __attribute__((aligned(16))) bf16_t lds[NS * STAGE];

    const int nblk = tiles_m * tiles_n;
    // `block_id` as the hardware deals it (round-robin over the XCDs) or already renumbered
    const int xcd = block_id & 7, local = block_id >> 3;
    const int pid = xcd_remap ? xcd * (nblk >> 3) + min(xcd, nblk & 7) + local : block_id;
    const int width = group_m * tiles_n;
    const int first_m = (pid / width) * group_m;
    const int gsz = min(tiles_m - first_m, group_m);
    const int tile_m = first_m + (pid % width) % gsz;
    const int tile_n = (pid % width) / gsz;
    const int i0 = tile_m * BM, j0 = tile_n * BN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wk = wave / (WGM * WGN), wmn = wave % (WGM * WGN);       // k slice, position in the tile
    const int wm0 = (wmn / WGN) * WM, wn0 = (wmn % WGN) * WN;

    // Per-thread source pointers (advanced by one k step after every issue) for the LDS
    // slots this thread's lane position fills.
    const bf16_t* ga[CA];
    const bf16_t* gb[CB];
    auto source = [&](const bf16_t* base, int ld, int row0, int nrows, int rows_in_tile, bool kc, int slot) {
        if (kc) {
            const int row = slot >> 3, p = slot & 7;
            const int c = p ^ (row & 7) ^ ((row >> 3) & 7);
            const int gr = min(row0 + row, nrows - 1);
            return base + (size_t)gr * ld + c * 8;
        }
        const int per_row = rows_in_tile / 8;
        const int kk = slot / per_row, pc = slot % per_row;
        const int ic = ((((pc >> 1) ^ ((kk & 3) << 1)) << 1) | (pc & 1));
        int gi = row0 + ic * 8;
        if (gi >= nrows) gi = 0;
        return base + (size_t)kk * ld + gi;
    };
#pragma unroll
    for (int it = 0; it < CA; ++it) ga[it] = source(A, lda, i0, m, BM, A_KC, it * NT + tid);
#pragma unroll
    for (int it = 0; it < CB; ++it) gb[it] = source(B, ldb, j0, n, BN, B_KC, it * NT + tid);
    const size_t step_a = A_KC ? (size_t)BK : (size_t)BK * lda;
    const size_t step_b = B_KC ? (size_t)BK : (size_t)BK * ldb;
    // LDS byte address of stage 0 (32-bit pointer in the LDS address space)
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) const void*)lds;

    auto issue = [&](int stage) {
        const unsigned sa = lds0 + (unsigned)(stage * STAGE) * 2u + (unsigned)wave * 1024u;
#pragma unroll
        for (int it = 0; it < CA; ++it) { lds_dma16(ga[it], sa + it * NT * 16); ga[it] += step_a; }
        const unsigned sb = sa + BM * BK * 2;
#pragma unroll
        for (int it = 0; it < CB; ++it) { lds_dma16(gb[it], sb + it * NT * 16); gb[it] += step_b; }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    // Optional by-product: bsum[j] += sum over the contraction index of B(k, j), i.e. an extra
    // all-ones row of A.  The wavefronts at the top edge of the first tile row compute it
    // with one more MFMA per 32 columns (every row of that accumulator is the column sum).
    const bool col_sums = bsum != nullptr && tile_m == 0 && wm0 == 0;
    f32x16 cs[TN];
    bf16x8 ones;
#pragma unroll
    for (int q = 0; q < 8; ++q) ones[q] = (bf16_t)1.0f;
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) cs[b][r] = 0.f;

    const int KT = k / BK;
#pragma unroll
    for (int st = 0; st < NS - 1; ++st)
        if (st < KT) issue(st);
    int cur = 0, nxt = NS - 1;                 // stage computed now / stage the next issue fills
    for (int kt = 0; kt < KT; ++kt) {
        // the oldest outstanding group (step kt) must have landed; up to NS-2 younger ones may fly on
        if (kt + NS - 2 < KT) wait_vmcnt<(NS - 2) * (CA + CB)>(); else wait_vmcnt<0>();
        __syncthreads();                       // every wavefront's part of step kt is in LDS; step kt-1 is consumed
        if (kt + NS - 1 < KT) issue(nxt);
        const bf16_t* As = lds + cur * STAGE;
        const bf16_t* Bs = As + BM * BK;
#pragma unroll
        for (int ks = 0; ks < KSUB; ++ks) {
            const int kk = wk * KSUB + ks;
            bf16x8 af[TM], bfr[TN];
#pragma unroll
            for (int a = 0; a < TM; ++a) af[a] = read_frag<BM, A_KC>(As, wm0 + a * 32, kk, lane);
#pragma unroll
            for (int b = 0; b < TN; ++b) bfr[b] = read_frag<BN, B_KC>(Bs, wn0 + b * 32, kk, lane);
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bfr[b], acc[a][b], 0, 0, 0);
            if constexpr (ONLY_EPI == EPI_ACCUM_F32)
                if (col_sums)
#pragma unroll
                    for (int b = 0; b < TN; ++b) cs[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, bfr[b], cs[b], 0, 0, 0);
        }
        cur = cur + 1 == NS ? 0 : cur + 1;
        nxt = nxt + 1 == NS ? 0 : nxt + 1;
    }

    const int cb0 = j0 + wn0;
    // the operand tiles in LDS are dead once every wavefront has left the k loop; each
    // wavefront then stages its output through its own slab there
    static_assert(sizeof(lds) >= (size_t)(NT / 64) * EpiSlab<TN>::FLOATS * sizeof(float), "LDS too small for the epilogue");
    __syncthreads();
    float* slab = reinterpret_cast<float*>(lds) + (size_t)(tid >> 6) * EpiSlab<TN>::FLOATS;
    auto finish = [&](const auto& out, int rb0) {
#define CHIMERA_EPI(E, RF, CF) epilogue<E, RF, CF>(out, slab, rb0, cb0, m, n, bias, R, C, C2, epi_flag, lane)
        if constexpr (ONLY_EPI == EPI_ACCUM_F32) { CHIMERA_EPI(EPI_ACCUM_F32, false, false); return; }
        switch (epi) {
            case EPI_NONE: CHIMERA_EPI(EPI_NONE, false, false); break;
            case EPI_BIAS: CHIMERA_EPI(EPI_BIAS, false, false); break;
            case EPI_BIAS_GELU: CHIMERA_EPI(EPI_BIAS_GELU, false, false); break;
            case EPI_BIAS_RESIDUAL:
                if (res_types == 0) CHIMERA_EPI(EPI_BIAS_RESIDUAL, false, false);
                else if (res_types == 1) CHIMERA_EPI(EPI_BIAS_RESIDUAL, true, false);
                else if (res_types == 2) CHIMERA_EPI(EPI_BIAS_RESIDUAL, false, true);
                else CHIMERA_EPI(EPI_BIAS_RESIDUAL, true, true);
                break;
            case EPI_DGELU: CHIMERA_EPI(EPI_DGELU, false, false); break;
            default: CHIMERA_EPI(EPI_ACCUM_F32, false, false); break;
        }
#undef CHIMERA_EPI
    };
    // row 0 of a column-sum accumulator: register 0 of lanes 0..31
    auto put_col_sums = [&](const float (&v)[TN]) {
        if (lane < 32)
#pragma unroll
            for (int b = 0; b < TN; ++b) {
                const int col = cb0 + b * 32 + lane;
                if (col < n) bsum[col] = epi_flag ? v[b] : bsum[col] + v[b];
            }
    };
    if constexpr (WGK == 1) {
        if constexpr (ONLY_EPI == EPI_ACCUM_F32)
            if (col_sums) {
                float v[TN];
#pragma unroll
                for (int b = 0; b < TN; ++b) v[b] = cs[b][0];
                put_col_sums(v);
            }
        finish(acc, i0 + wm0);
    } else {
        // Two wavefronts hold partial sums of the same WM x WN block (one per k slice).  Each
        // keeps the upper or lower half of the rows: it hands the other half to its partner
        // through LDS, adds what the partner hands over (one float addition per element, so the
        // result does not depend on which wavefront adds), and finishes its half.
        static_assert(WGK == 2 && TM % 2 == 0, "row halves");
        constexpr int TMO = TM / 2;
        constexpr int PER_WAVE = TMO * TN * 4 * 64;                      // float4 per wavefront
        static_assert(sizeof(lds) >= (size_t)(NT / 64) * PER_WAVE * sizeof(float4), "LDS too small for the exchange");
        float4* xch = reinterpret_cast<float4*>(lds);
        // column sums of the two k slices meet behind the exchange area
        float* xcs = reinterpret_cast<float*>(xch + (size_t)(NT / 64) * PER_WAVE) + wn0;
        static_assert(sizeof(lds) >= (size_t)(NT / 64) * PER_WAVE * sizeof(float4) + BN * sizeof(float), "LDS too small");
        if constexpr (ONLY_EPI == EPI_ACCUM_F32)
            if (col_sums && wk == 1 && lane < 32)
#pragma unroll
                for (int b = 0; b < TN; ++b) xcs[b * 32 + lane] = cs[b][0];
        float4* send = xch + (size_t)wave * PER_WAVE + lane;
        const float4* recv = xch + (size_t)(wave ^ (WGM * WGN)) * PER_WAVE + lane;
        f32x16 own[TMO][TN];
#pragma unroll
        for (int a = 0; a < TMO; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b) {
                const f32x16 give = wk ? acc[a][b] : acc[TMO + a][b];
                own[a][b] = wk ? acc[TMO + a][b] : acc[a][b];
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    send[((a * TN + b) * 4 + q) * 64] = make_float4(give[4 * q], give[4 * q + 1], give[4 * q + 2], give[4 * q + 3]);
            }
        __syncthreads();
#pragma unroll
        for (int a = 0; a < TMO; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 v = recv[((a * TN + b) * 4 + q) * 64];
                    own[a][b][4 * q] += v.x;
                    own[a][b][4 * q + 1] += v.y;
                    own[a][b][4 * q + 2] += v.z;
                    own[a][b][4 * q + 3] += v.w;
                }
        if constexpr (ONLY_EPI == EPI_ACCUM_F32)
            if (col_sums && wk == 0) {
                float v[TN];
#pragma unroll
                for (int b = 0; b < TN; ++b) v[b] = cs[b][0] + (lane < 32 ? xcs[b * 32 + lane] : 0.f);
                put_col_sums(v);
            }
        __syncthreads();                       // the exchange area becomes the slabs
        finish(own, i0 + wm0 + wk * TMO * 32);
    }
}

template <int BM, int BN, int WGM, int WGN, int WGK, int NS, bool A_KC, bool B_KC>
__global__ __launch_bounds__(WGM* WGN * WGK * 64) void gemm_bf16_async_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, const bf16_t* __restrict__ bias,
    const bf16_t* __restrict__ R, void* __restrict__ C, bf16_t* __restrict__ C2, int m, int n, int k, int lda,
    int ldb, int epi, int epi_flag, int res_types, int tiles_m, int tiles_n, int group_m) {
    gemm_async_tile<BM, BN, WGM, WGN, WGK, NS, A_KC, B_KC, -1>(A, B, bias, R, C, C2, m, n, k, lda, ldb, epi, epi_flag,
                                                                res_types, tiles_m, tiles_n, group_m, (int)blockIdx.x);
}

// Several products C_p (float) += A_p B_p of one launch: same contraction length and operand
// layout, each with its own shapes and pointers.  Workgroups [first[p], first[p+1]) work on
// product p, so small products no longer leave most of the chip idle for a launch of their
// own.  (The weight gradients of one Transformer block are such a group.)
constexpr int GROUP_MAX = 4;
struct GemmGroup {
    const bf16_t* a[GROUP_MAX];
    const bf16_t* b[GROUP_MAX];
    float* c[GROUP_MAX];
    float* bsum[GROUP_MAX];      // optional: bsum[j] += sum_k B(k, j)
    int m[GROUP_MAX], n[GROUP_MAX], lda[GROUP_MAX], ldb[GROUP_MAX], tiles_m[GROUP_MAX], tiles_n[GROUP_MAX];
    int group_m[GROUP_MAX];      // tile rows per raster group of each product
    int first[GROUP_MAX + 1];
    int count, k;
    int overwrite;               // results replace C and bsum instead of being added
};

template <int BM, int BN, int WGM, int WGN, int WGK, int NS, bool A_KC, bool B_KC>
__global__ __launch_bounds__(WGM* WGN * WGK * 64) void gemm_bf16_async_group_kernel(GemmGroup grp) {
    // each XCD takes a contiguous range of the group's tiles (products laid end to end), so that
    // its L2 sees few operand panels: one product's tiles are not dealt over all eight XCDs
    const int total = grp.first[grp.count];
    const int xcd = (int)blockIdx.x & 7, local = (int)blockIdx.x >> 3;
    const int gid = xcd * (total >> 3) + min(xcd, total & 7) + local;
    int p = 0;
#pragma unroll
    for (int i = 1; i < GROUP_MAX; ++i)
        if (i < grp.count && gid >= grp.first[i]) p = i;
    gemm_async_tile<BM, BN, WGM, WGN, WGK, NS, A_KC, B_KC, EPI_ACCUM_F32>(
        grp.a[p], grp.b[p], nullptr, nullptr, grp.c[p], nullptr, grp.m[p], grp.n[p], grp.k, grp.lda[p], grp.ldb[p],
        EPI_ACCUM_F32, grp.overwrite, 0, grp.tiles_m[p], grp.tiles_n[p], grp.group_m[p], gid - grp.first[p], grp.bsum[p],
        false);
}

// A launch of 256x256 tiles runs in rounds of NUM_CUS tiles, and a last round with few tiles
// costs as much as a full one.  The products here can be cut along m without touching the data
// (row bands of A and C are just pointer offsets), so the last `b` bands of 256 rows may go to a
// second launch with 128x128 tiles instead.  Cost estimate in units of one 256x256 round: a round
// of 128x128 tiles (quarter of the flops, 1.6x the time per flop) counts 0.45.  Returns the b
// that minimises it (0: leave the product whole); `other` = 256x256 tiles of the launch that do
// not belong to this product.
int bands_to_peel(long other, int tm, int tn, int n) {
    const int tn128 = (n + 127) / 128;
    auto rounds = [](long tiles) { return (double)((tiles + NUM_CUS - 1) / NUM_CUS); };
    const double whole = rounds(other + (long)tm * tn);
    int best_b = 0;
    double best = whole - 0.25;                                  // a split must pay for its second launch
    for (int b = 1; b < tm; ++b) {
        const double est = rounds(other + (long)(tm - b) * tn) + 0.45 * rounds((long)b * 2 * tn128);
        if (est < best) { best = est; best_b = b; }
    }
    return best_b;
}

// Tile rows per raster group.  A launch's tiles are dealt to the 8 XCDs in contiguous ranges of
// `per_xcd` tiles, walked column by column inside groups of g tile rows, so an XCD works on
// about g rows x per_xcd / g columns of tiles and its L2 has to fetch g row panels of A and
// per_xcd / g column panels of B - everything an L2 misses arrives at HBM speed (about 7 TB/s
// for the whole chip, a quarter of what the L2s deliver), whether or not it is in the memory-
// side cache.  Returns the g that minimises the bytes fetched (tile heights bm, widths bn),
// counting the ragged last group at its share of the rows.
int raster_group(int tiles_m, int tiles_n, int per_xcd, int bm, int bn) {
    int best_g = 1;
    double best = 1e300;
    for (int g = 1; g <= std::min(tiles_m, 16); ++g) {
        double cost = 0;
        for (int r0 = 0; r0 < tiles_m; r0 += g) {
            const int rows = std::min(g, tiles_m - r0);
            const int cols = std::min(tiles_n, (per_xcd + rows - 1) / rows);
            cost += ((double)rows * bm + (double)cols * bn) * rows;       // weighted by the group's share of the tiles
        }
        if (cost < best * 0.999) { best = cost; best_g = g; }
    }
    return best_g;
}

struct TileChoice { int bm, bn, splits; };

// The kernels' `epi_flag` argument modifies the epilogue: for the GeLU epilogues 1 selects the
// erf form (0: tanh form); for the float-accumulate epilogue 1 makes the result replace C (and
// the column sums replace bsum) instead of being added, which a single product never asks for.
inline int epilogue_flag(const GemmArgs& g) { return g.epilogue == EPI_ACCUM_F32 ? 0 : g.gelu_erf; }

// Tuning aids, read from the environment once (first use) and changeable through
// chimera_gemm_tuning(): a forced tile ("256x256", "128x128" or "256x256x<splits>" in
// CHIMERA_GEMM_TILE) and the form of the LDS-DMA kernels (CHIMERA_GEMM_ASYNC: "0" = the
// register-staged kernels, "4k" = the k-sliced 128x128 form always, "2" = never).
enum AsyncMode { ASYNC_AUTO = 0, ASYNC_OFF = 1, ASYNC_KSLICED = 2, ASYNC_PLAIN = 3 };
struct Tuning { TileChoice forced{0, 0, 0}; int async_mode = ASYNC_AUTO; };
Tuning& tuning() {
    static Tuning t = [] {
        Tuning v;
        if (const char* e = std::getenv("CHIMERA_GEMM_TILE")) std::sscanf(e, "%dx%dx%d", &v.forced.bm, &v.forced.bn, &v.forced.splits);
        if (const char* e = std::getenv("CHIMERA_GEMM_ASYNC"))
            v.async_mode = e[0] == '0' ? ASYNC_OFF : (!std::strcmp(e, "4k") ? ASYNC_KSLICED : ASYNC_PLAIN);
        return v;
    }();
    return t;
}
TileChoice forced_tile() { return tuning().forced; }

constexpr int MAX_SPLITS = 8;

// 256x256 (8 wavefronts) once the output has enough such tiles for most of the 256 CUs,
// else 128x128 (4 wavefronts, two workgroups per CU); thresholds measured on MI355X.
// A CU fills LDS from L2 at roughly 64 bytes per clock, so a 128x128x64 step (32 KiB for
// 512 clocks of MFMA work) is fed at half the rate the matrix cores could use; 256x256
// halves the bytes per flop, which is why it wins whenever it can occupy the chip.
// Split-K (several workgroups per 256x256 tile, see the kernel) is available on request
// (CHIMERA_GEMM_TILE=256x256x<splits> plus a workspace) but not chosen by default: on
// MI355X the device-wide fences its hand-over needs cost more than the idle CUs.
TileChoice choose_tile(const GemmArgs& g) {
    TileChoice f = forced_tile();
    const long t256 = (long)((g.m + 255) / 256) * ((g.n + 255) / 256);
    if (f.bm) {
        if (f.splits < 1 || f.bm != 256) f.splits = 1;
        f.splits = std::min(f.splits, std::min(MAX_SPLITS, std::max(1, (g.k + BK - 1) / BK)));
        if (f.splits > 1 && (!g.ws || g.ws_bytes < gemm_mfma_workspace_bytes(g.m, g.n, f.splits))) f.splits = 1;
        return f;
    }
    // (measured at 2048 x 4800 x 1600: 152 tiles of 256x256 on 256 CUs take 42 us, 608 of 128x128 48 us)
    if (t256 >= 144) return {256, 256, 1};
    return {128, 128, 1};
}

template <int BM, int BN, int WGM, int WGN, int PF>
int launch_layout(const GemmArgs& g, int splits, hipStream_t s) {
    const int tm = (g.m + BM - 1) / BM, tn = (g.n + BN - 1) / BN;
    const dim3 grid(tm * tn * splits), block(WGM * WGN * 64);
    unsigned* arrivals = (unsigned*)g.ws;                               // [tiles], zero between launches
    float* slabs = g.ws ? (float*)((char*)g.ws + SPLITK_COUNTER_BYTES) : nullptr;
#define CHIMERA_GEMM_LAUNCH(AKC, BKC)                                                                              \
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WGM, WGN, PF, AKC, BKC>), grid, block, 0, s, (const bf16_t*)g.a,  \
                       (const bf16_t*)g.b, (const bf16_t*)g.bias, (const bf16_t*)g.r, g.c, (bf16_t*)g.c2, g.m, g.n, \
                       g.k, g.lda, g.ldb, g.epilogue, epilogue_flag(g), (g.r_f32 ? 1 : 0) | (g.c_f32 ? 2 : 0), tm, tn,    \
                       splits, slabs, arrivals)
    if (g.a_kc && !g.b_kc) CHIMERA_GEMM_LAUNCH(true, false);
    else if (g.a_kc && g.b_kc) CHIMERA_GEMM_LAUNCH(true, true);
    else CHIMERA_GEMM_LAUNCH(false, false);
#undef CHIMERA_GEMM_LAUNCH
    CHIMERA_LAUNCH_CHECK("bf16 gemm");
    return CHIMERA_OK;
}

template <int BM, int BN, int WGM, int WGN, int WGK, int NS>
int launch_async(const GemmArgs& g, hipStream_t s) {
    const int tm = (g.m + BM - 1) / BM, tn = (g.n + BN - 1) / BN;
    const dim3 grid(tm * tn), block(WGM * WGN * WGK * 64);
    const int gm = raster_group(tm, tn, (tm * tn + 7) / 8, BM, BN);
#define CHIMERA_GEMM_LAUNCH(AKC, BKC)                                                                                \
    hipLaunchKernelGGL((gemm_bf16_async_kernel<BM, BN, WGM, WGN, WGK, NS, AKC, BKC>), grid, block, 0, s,                   \
                       (const bf16_t*)g.a, (const bf16_t*)g.b, (const bf16_t*)g.bias, (const bf16_t*)g.r, g.c,        \
                       (bf16_t*)g.c2, g.m, g.n, g.k, g.lda, g.ldb, g.epilogue, epilogue_flag(g),                            \
                       (g.r_f32 ? 1 : 0) | (g.c_f32 ? 2 : 0), tm, tn, gm)
    if (g.a_kc && !g.b_kc) CHIMERA_GEMM_LAUNCH(true, false);
    else if (g.a_kc && g.b_kc) CHIMERA_GEMM_LAUNCH(true, true);
    else CHIMERA_GEMM_LAUNCH(false, false);
#undef CHIMERA_GEMM_LAUNCH
    CHIMERA_LAUNCH_CHECK("bf16 gemm (async)");
    return CHIMERA_OK;
}

// Name of the kernel instantiation(s) the last grouped launch on this thread went to (for reports).
thread_local char g_last_group_kernel[192] = "";
void note_group_kernel(bool first, const char* name) {
    char* dst = g_last_group_kernel;
    const size_t used = first ? 0 : std::strlen(dst);
    std::snprintf(dst + used, sizeof g_last_group_kernel - used, "%s%s", used ? " + " : "", name);
}

template <int BM, int BN, int WGM, int WGN, int WGK, int NS>
int launch_group(const GemmGroup& grp, hipStream_t s, bool first = true) {
    char name[96];
    std::snprintf(name, sizeof name, "gemm_bf16_async_group_kernel<%d,%d,%d,%d,%d,%d,false,false>", BM, BN, WGM, WGN, WGK, NS);
    note_group_kernel(first, name);
    const dim3 grid(grp.first[grp.count]), block(WGM * WGN * WGK * 64);
    hipLaunchKernelGGL((gemm_bf16_async_group_kernel<BM, BN, WGM, WGN, WGK, NS, false, false>), grid, block, 0, s, grp);
    CHIMERA_LAUNCH_CHECK("bf16 gemm group");
    return CHIMERA_OK;
}

}  // namespace

bool gemm_mfma_supports(const GemmArgs& g) {
    if (!g.a_kc && g.b_kc) return false;                       // layout no linear layer needs
    if ((g.k % 8) || (g.n % 8) || (g.lda % 8) || (g.ldb % 8)) return false;
    if (!g.a_kc && (g.m % 8)) return false;
    if (((uintptr_t)g.a | (uintptr_t)g.b) & 15) return false;  // 16-byte vector loads
    // operand elements are addressed with 32-bit offsets
    const unsigned long long ea = (unsigned long long)(g.a_kc ? g.m : g.k) * g.lda, eb = (unsigned long long)(g.b_kc ? g.n : g.k) * g.ldb;
    if (ea >= (1ull << 32) || eb >= (1ull << 32)) return false;
    return g.m >= 1 && g.n >= 1 && g.k >= 1;
}

// Workspace of a split-K launch: arrival counters (zero before the first launch, left zero
// by every launch) followed by one float slab per (split, 256x256 tile).
size_t gemm_mfma_workspace_bytes(int m, int n, int splits) {
    const size_t tiles = (size_t)((m + 255) / 256) * ((n + 255) / 256);
    return SPLITK_COUNTER_BYTES + (size_t)splits * tiles * 256 * 256 * sizeof(float);
}
// Workspace that allows any split count up to MAX_SPLITS for an m x n output.
size_t gemm_mfma_workspace_need(int m, int n, int k) {
    if (m < 1 || n < 1 || k < 1) return 0;
    return gemm_mfma_workspace_bytes(m, n, MAX_SPLITS);
}

int gemm_mfma_bf16(const GemmArgs& g, void* stream) {
    if (!gemm_mfma_supports(g)) return fail(CHIMERA_EINVAL, "bf16 matrix-core gemm: unsupported shape or layout");
    if (g.epilogue < EPI_NONE || g.epilogue > EPI_ACCUM_F32) return fail(CHIMERA_EINVAL, "unknown epilogue %d", g.epilogue);
    hipStream_t s = (hipStream_t)stream;
    const TileChoice t = choose_tile(g);
    if (t.splits > 1 && (size_t)((g.m + 255) / 256) * ((g.n + 255) / 256) * sizeof(unsigned) > SPLITK_COUNTER_BYTES)
        return fail(CHIMERA_EINVAL, "too many tiles for split-K");
    // the async kernels cannot zero-fill: whole k steps only, and at least 8 rows on each side.
    // 128x128 tiles: with one workgroup per CU, a workgroup of 4 wavefronts leaves one wavefront
    // per SIMD, and nothing covers its LDS latency and the barrier of every k step; then 8
    // wavefronts share the tile, two per 64x64 block, each taking half of every k step (their
    // partial sums meet in LDS at the end), over a 3-stage ring of 96 KiB - one such workgroup
    // per CU, so more than NUM_CUS tiles would take it two rounds.  Beyond that the 4-wavefront
    // form with its 2-stage ring (64 KiB of LDS, two workgroups per CU) is faster: 416 tiles of a
    // 4096 x 1600 x 6400 product take 109 us against 124 us, 208 tiles (2048 rows) 89 against 62.
    const int mode = tuning().async_mode;
    const bool can_async = g.k % BK == 0 && g.m >= 8 && g.n >= 8 && t.splits == 1 && mode != ASYNC_OFF;
    if (can_async) {
        if (t.bm == 256 && t.bn == 256) {
            const int tm = (g.m + 255) / 256, tn = (g.n + 255) / 256;
            const int b = forced_tile().bm ? 0 : bands_to_peel(0, tm, tn, g.n);
            if (b > 0 && g.m - (tm - b) * 256 >= 8) {
                // rows [0, m0) with 256x256 tiles, rows [m0, m) with 128x128 tiles
                const size_t m0 = (size_t)(tm - b) * 256;
                const size_t csz = (g.epilogue == EPI_ACCUM_F32 || g.c_f32) ? 4 : 2;
                GemmArgs head = g, tail = g;
                head.m = (int)m0;
                tail.m = g.m - (int)m0;
                tail.a = (const char*)g.a + (g.a_kc ? m0 * g.lda : m0) * 2;
                tail.c = (char*)g.c + m0 * g.n * csz;
                if (g.c2) tail.c2 = (char*)g.c2 + m0 * g.n * 2;
                if (g.r) tail.r = (const char*)g.r + m0 * g.n * (g.r_f32 ? 4 : 2);
                if (int rc = launch_async<256, 256, 2, 4, 1, 2>(head, s)) return rc;
                const long t128 = (long)((tail.m + 127) / 128) * ((tail.n + 127) / 128);
                if (t128 <= NUM_CUS) return launch_async<128, 128, 2, 2, 2, 3>(tail, s);
                return launch_async<128, 128, 2, 2, 1, 2>(tail, s);
            }
            return launch_async<256, 256, 2, 4, 1, 2>(g, s);
        }
        if (t.bm == 128 && t.bn == 128) {
            const long t128 = (long)((g.m + 127) / 128) * ((g.n + 127) / 128);
            const bool ksplit = mode != ASYNC_AUTO ? mode == ASYNC_KSLICED : t128 <= NUM_CUS;
            if (ksplit) return launch_async<128, 128, 2, 2, 2, 3>(g, s);
            return launch_async<128, 128, 2, 2, 1, 2>(g, s);
        }
    }
    if (t.bm == 256 && t.bn == 256) return launch_layout<256, 256, 2, 4, 1>(g, t.splits, s);
    if (t.bm == 128 && t.bn == 128) return launch_layout<128, 128, 2, 2, 1>(g, 1, s);
    return fail(CHIMERA_EINVAL, "no %dx%d gemm tile", t.bm, t.bn);
}

bool gemm_mfma_group_supports(int count, const GemmArgs* g) {
    if (count < 1 || count > GROUP_MAX || !g) return false;
    for (int i = 0; i < count; ++i) {
        if (g[i].a_kc || g[i].b_kc || g[i].epilogue != EPI_ACCUM_F32 || !gemm_mfma_supports(g[i])) return false;
        if (g[i].k != g[0].k || g[i].k % BK || g[i].m < 8 || g[i].n < 8) return false;
        if ((uintptr_t)g[i].c & 15) return false;
    }
    return true;
}

namespace {
int launch_group_tiled(int count, const GemmArgs* g, float* const* bsum, int overwrite, int tile, hipStream_t stream,
                       bool first = true) {
    GemmGroup grp{};
    grp.count = count; grp.k = g[0].k; grp.overwrite = overwrite ? 1 : 0;
    int tiles = 0;
    for (int i = 0; i < count; ++i) {
        grp.a[i] = (const bf16_t*)g[i].a; grp.b[i] = (const bf16_t*)g[i].b; grp.c[i] = (float*)g[i].c;
        grp.bsum[i] = bsum ? bsum[i] : nullptr;
        grp.m[i] = g[i].m; grp.n[i] = g[i].n; grp.lda[i] = g[i].lda; grp.ldb[i] = g[i].ldb;
        grp.tiles_m[i] = (g[i].m + tile - 1) / tile; grp.tiles_n[i] = (g[i].n + tile - 1) / tile;
        grp.first[i] = tiles;
        tiles += grp.tiles_m[i] * grp.tiles_n[i];
    }
    for (int i = 0; i < count; ++i) grp.group_m[i] = raster_group(grp.tiles_m[i], grp.tiles_n[i], (tiles + 7) / 8, tile, tile);
    for (int i = count; i <= GROUP_MAX; ++i) grp.first[i] = tiles;
    if (tile == 256) return launch_group<256, 256, 2, 4, 1, 2>(grp, stream, first);
    // two workgroups per CU or the k-sliced 8-wavefront form
    const int mode = tuning().async_mode;
    const bool ksplit = mode != ASYNC_AUTO ? mode == ASYNC_KSLICED : tiles <= NUM_CUS;
    if (ksplit) return launch_group<128, 128, 2, 2, 2, 3>(grp, stream, first);
    return launch_group<128, 128, 2, 2, 1, 2>(grp, stream, first);
}
}  // namespace

// Decides how a group goes out: tile size, and whether the last row bands of one product leave
// as a second launch with 128x128 tiles (a nearly empty last round of 256x256 tiles).
int gemm_mfma_group_plan(int count, const GemmArgs* g, GemmGroupPlan* plan) {
    if (!plan) return fail(CHIMERA_EINVAL, "plan is NULL");
    if (!gemm_mfma_group_supports(count, g))
        return fail(CHIMERA_EINVAL, "bf16 gemm group: 1..%d float-accumulating products with index-contiguous operands, "
                    "one contraction length (a multiple of %d)", GROUP_MAX, BK);
    static_assert(GROUP_MAX == sizeof(plan->head) / sizeof(plan->head[0]), "plan size");
    plan->count = count; plan->has_tail = 0; plan->tail_of = -1;
    for (int i = 0; i < count; ++i) plan->head[i] = g[i];
    // tile choice as for single products: 256x256 once such tiles occupy most of the chip, else
    // 128x128.  (192 tiles of 256x256 on 256 CUs beat 768 tiles of 128x128: they pull half the
    // bytes from L2 into LDS, which is what limits these kernels, and the CUs they leave free
    // serve the launches of the other stream.)
    long t256 = 0;
    for (int i = 0; i < count; ++i) t256 += (long)((g[i].m + 255) / 256) * ((g[i].n + 255) / 256);
    const TileChoice forced = forced_tile();
    plan->tile = forced.bm == 256 || forced.bm == 128 ? forced.bm : (t256 >= 160 ? 256 : 128);
    if (plan->tile != 256 || forced.bm) return CHIMERA_OK;
    // a nearly empty last round: the last row bands of one product go to a 128x128 launch
    int best_p = -1, best_b = 0;
    double best_rounds = 1e30;
    for (int p = 0; p < count; ++p) {
        const int tm = (g[p].m + 255) / 256, tn = (g[p].n + 255) / 256;
        const int b = bands_to_peel(t256 - (long)tm * tn, tm, tn, g[p].n);
        if (!b || g[p].m - (tm - b) * 256 < 8) continue;
        const double est = (double)((t256 - (long)b * tn + NUM_CUS - 1) / NUM_CUS) + 0.45 * (double)(((long)b * 2 * ((g[p].n + 127) / 128) + NUM_CUS - 1) / NUM_CUS);
        if (est < best_rounds) { best_rounds = est; best_p = p; best_b = b; }
    }
    if (best_p < 0) return CHIMERA_OK;
    const size_t m0 = (size_t)((g[best_p].m + 255) / 256 - best_b) * 256;
    plan->head[best_p].m = (int)m0;
    plan->tail = g[best_p];
    plan->tail.m = g[best_p].m - (int)m0;
    plan->tail.a = (const char*)plan->tail.a + m0 * 2;                      // A is [k, m]: the band starts m0 columns in
    plan->tail.c = (char*)plan->tail.c + m0 * plan->tail.n * sizeof(float);
    plan->has_tail = 1; plan->tail_of = best_p;
    return CHIMERA_OK;
}

int gemm_mfma_group_launch_head(const GemmGroupPlan& plan, float* const* bsum, int overwrite, void* stream) {
    return launch_group_tiled(plan.count, plan.head, bsum, overwrite, plan.tile, (hipStream_t)stream);
}

int gemm_mfma_group_launch_tail(const GemmGroupPlan& plan, int overwrite, void* stream) {
    if (!plan.has_tail) return CHIMERA_OK;
    return launch_group_tiled(1, &plan.tail, nullptr, overwrite, 128, (hipStream_t)stream, false);   // the column sums come from the head
}

int gemm_mfma_bf16_group(int count, const GemmArgs* g, float* const* bsum, int overwrite, void* stream) {
    GemmGroupPlan plan;
    if (int rc = gemm_mfma_group_plan(count, g, &plan)) return rc;
    if (int rc = gemm_mfma_group_launch_head(plan, bsum, overwrite, stream)) return rc;
    return gemm_mfma_group_launch_tail(plan, overwrite, stream);
}

const char* gemm_mfma_last_group_kernel() { return g_last_group_kernel; }

int gemm_mfma_set_tuning(int bm, int bn, int splits, int async_mode) {
    if (!((bm == 0 && bn == 0) || (bm == 128 && bn == 128) || (bm == 256 && bn == 256)))
        return fail(CHIMERA_EINVAL, "forced tile %dx%d: 0x0 (automatic), 128x128 or 256x256", bm, bn);
    if (splits < 0 || splits > MAX_SPLITS) return fail(CHIMERA_EINVAL, "splits=%d outside [0,%d]", splits, MAX_SPLITS);
    if (async_mode < ASYNC_AUTO || async_mode > ASYNC_PLAIN) return fail(CHIMERA_EINVAL, "async_mode=%d outside [0,3]", async_mode);
    Tuning& t = tuning();
    t.forced = TileChoice{bm, bn, splits};
    t.async_mode = async_mode;
    return CHIMERA_OK;
}

}  // namespace chimera
