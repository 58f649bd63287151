// Device-side helpers shared by the HIP kernels: element types, 16-byte
// vector access, wavefront reductions (64 lanes) and the GeLU forms.
#pragma once

#include <hip/hip_runtime.h>

#include "internal.h"

namespace chimera {

typedef __bf16 bf16_t;

constexpr float LN_EPS = 1e-5f;
constexpr int WAVE = 64;

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int VEC = 4;   // elements per 16-byte access
    static __device__ __forceinline__ float to_f(float v) { return v; }
    static __device__ __forceinline__ float from_f(float v) { return v; }
};
template <> struct Elem<bf16_t> {
    static constexpr int VEC = 8;
    static __device__ __forceinline__ float to_f(bf16_t v) { return (float)v; }
    static __device__ __forceinline__ bf16_t from_f(float v) { return (bf16_t)v; }   // nearest even
};

// 16-byte load of Elem<T>::VEC consecutive elements, widened to float.
template <typename T> __device__ __forceinline__ void load_vec(const T* p, float* out);
template <> __device__ __forceinline__ void load_vec<float>(const float* p, float* out) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
}
template <> __device__ __forceinline__ void load_vec<bf16_t>(const bf16_t* p, float* out) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        out[2 * i] = __uint_as_float(w[i] << 16);
        out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}
template <typename T> __device__ __forceinline__ void store_vec(T* p, const float* in);
template <> __device__ __forceinline__ void store_vec<float>(float* p, const float* in) {
    *reinterpret_cast<float4*>(p) = make_float4(in[0], in[1], in[2], in[3]);
}
template <> __device__ __forceinline__ void store_vec<bf16_t>(bf16_t* p, const float* in) {
    typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
    bf16x8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (bf16_t)in[i];
    *reinterpret_cast<bf16x8*>(p) = v;
}

// V consecutive elements of type T (V = 4 or 8), widened to float / narrowed from float.
template <typename T, int V> __device__ __forceinline__ void load_elems(const T* p, float* out) {
    constexpr int PER = Elem<T>::VEC;
#pragma unroll
    for (int i = 0; i < V; i += PER) load_vec<T>(p + i, out + i);
}
template <typename T, int V> __device__ __forceinline__ void store_elems(T* p, const float* in) {
    constexpr int PER = Elem<T>::VEC;
#pragma unroll
    for (int i = 0; i < V; i += PER) store_vec<T>(p + i, in + i);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
    return v;
}

// GeLU, tanh form: 0.5 u (1 + tanh z), z = sqrt(2/pi) (u + 0.044715 u^3); erf form: u Phi(u).
// 0.5 (1 + tanh z) is the logistic function of 2z, which needs one hardware exp2 and one
// reciprocal: s = 1 / (1 + exp(-2z)).  Large |z| saturate exactly (exp2 -> inf gives s = 0,
// exp2 -> 0 gives s = 1).
__device__ __forceinline__ float gelu_logistic(float u) {
    const float u2 = u * u;
    const float m2z = u * __builtin_fmaf(u2, -2.0f * 0.79788456080286536f * 0.044715f * 1.4426950408889634f,
                                         -2.0f * 0.79788456080286536f * 1.4426950408889634f);    // -2 z log2(e)
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(m2z));
}
__device__ __forceinline__ float gelu_f(float u, int erf_form) {
    if (erf_form) return 0.5f * u * (1.0f + erff(u * 0.70710678118654752f));
    return u * gelu_logistic(u);
}
// d/du [u s(2z)] = s + u s (1 - s) 2 z'(u),  z'(u) = sqrt(2/pi) (1 + 3 * 0.044715 u^2)
__device__ __forceinline__ float gelu_grad_f(float u, int erf_form) {
    if (erf_form)
        return 0.5f * (1.0f + erff(u * 0.70710678118654752f)) + u * __expf(-0.5f * u * u) * 0.39894228040143268f;
    const float s = gelu_logistic(u);
    const float dz2 = __builtin_fmaf(u * u, 2.0f * 0.79788456080286536f * 3.0f * 0.044715f, 2.0f * 0.79788456080286536f);
    return __builtin_fmaf(u * dz2, s - s * s, s);
}

// Global -> LDS without passing through registers: lane i of the wavefront writes the 16
// bytes it fetches from `gptr` to LDS byte address lds_base + 16 i (lds_base must be the
// same for the whole wavefront).  Issued through inline assembly so that the wait can be
// counted by hand (wait_vmcnt) instead of draining every outstanding load.  The LDS base
// travels in M0, named as a register operand: the compiler loads M0 itself and knows that
// the statement depends on it, so its own uses of M0 cannot collide with this one.
__device__ __forceinline__ void lds_dma16(const void* gptr, unsigned lds_base) {
    asm volatile("global_load_lds_dwordx4 %0, off" ::"v"(gptr), "{m0}"(lds_base) : "memory");
}
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
    __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));     // expcnt, lgkmcnt untouched
}
// LDS byte address (32-bit pointer in the LDS address space) of a __shared__ object
__device__ __forceinline__ unsigned lds_address(const void* p) {
    return (unsigned)(size_t)(__attribute__((address_space(3))) const void*)p;
}

#define CHIMERA_LAUNCH_CHECK(what)                                                           \
    do {                                                                                     \
        hipError_t e__ = hipGetLastError();                                                  \
        if (e__ != hipSuccess) return fail(CHIMERA_EDEVICE, "%s: %s", what, hipGetErrorString(e__)); \
    } while (0)

}  // namespace chimera
