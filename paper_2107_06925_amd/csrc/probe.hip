// Measured ceilings of the device the library runs on: a register-resident MFMA loop
// (no memory traffic at all) and a streaming copy.  They put the achieved rates of the
// stage kernels next to what this chip sustains, beside the published peaks.
#include <hip/hip_runtime.h>

#include "device.h"
#include "internal.h"

namespace chimera {
namespace {

typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int PROBE_CUS = 256;          // compute units of an MI355X
constexpr int PROBE_WAVES = 8;          // wavefronts per workgroup: two per SIMD
constexpr int PROBE_UNROLL = 16;

// Every wavefront issues iters x 16 independent-accumulator-chained 32x32x16 bf16 MFMAs on
// operands that never leave registers.
__global__ __launch_bounds__(PROBE_WAVES * 64) void mfma_loop_kernel(int iters, float* sink) {
    const int lane = threadIdx.x & 63;
    bf16x8 a, b;
#pragma unroll
    for (int q = 0; q < 8; ++q) { a[q] = (bf16_t)(float)((lane + q) & 3); b[q] = (bf16_t)(float)((lane - q) & 3); }
    f32x16 c0 = {0}, c1 = {0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < PROBE_UNROLL / 2; ++u) {
            c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, c1, 0, 0, 0);
        }
    }
    float r = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) r += c0[q] + c1[q];
    if (r == -1.f) *sink = r;           // never true (all terms are non-negative); keeps the loop alive
}

__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

template <typename F> int timed(hipStream_t s, int reps, float* ms, const F& launch) {
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) return fail(CHIMERA_EDEVICE, "hipEventCreate failed");
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return fail(CHIMERA_EDEVICE, "hipEventCreate failed"); }
    launch();                           // warm-up
    (void)hipEventRecord(a, s);
    for (int i = 0; i < reps; ++i) launch();
    (void)hipEventRecord(b, s);
    hipError_t e = hipEventSynchronize(b);
    if (e == hipSuccess) e = hipEventElapsedTime(ms, a, b);
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    if (e != hipSuccess) return fail(CHIMERA_EDEVICE, "probe: %s", hipGetErrorString(e));
    return CHIMERA_OK;
}

}  // namespace
}  // namespace chimera

using namespace chimera;

extern "C" {

int chimera_probe_mfma_bf16(float* d_sink, int iters, double* h_tflops, void* hip_stream) {
    if (!d_sink || !h_tflops) return fail(CHIMERA_EINVAL, "NULL argument");
    if (iters < 1 || iters > (1 << 20)) return fail(CHIMERA_EINVAL, "iters out of range");
    hipStream_t s = (hipStream_t)hip_stream;
    const int blocks = PROBE_CUS * 2, reps = 3;
    float ms = 0.f;
    int rc = timed(s, reps, &ms, [&] { hipLaunchKernelGGL(mfma_loop_kernel, dim3(blocks), dim3(PROBE_WAVES * 64), 0, s, iters, d_sink); });
    if (rc) return rc;
    CHIMERA_LAUNCH_CHECK("mfma probe");
    const double flop = 2.0 * 32 * 32 * 16 * PROBE_UNROLL * (double)iters * PROBE_WAVES * blocks * reps;
    *h_tflops = flop / (ms * 1e-3) / 1e12;
    return CHIMERA_OK;
}

int chimera_probe_copy(const void* d_src, void* d_dst, size_t bytes, double* h_gbs, void* hip_stream) {
    if (!d_src || !d_dst || !h_gbs) return fail(CHIMERA_EINVAL, "NULL argument");
    if (bytes < 16 || (bytes % 16) || (((uintptr_t)d_src | (uintptr_t)d_dst) & 15)) return fail(CHIMERA_EINVAL, "copy probe needs 16-byte multiples");
    hipStream_t s = (hipStream_t)hip_stream;
    const int reps = 5;
    float ms = 0.f;
    int rc = timed(s, reps, &ms, [&] {
        hipLaunchKernelGGL(copy_kernel, dim3(PROBE_CUS * 16), dim3(256), 0, s, (const uint4*)d_src, (uint4*)d_dst, bytes / 16);
    });
    if (rc) return rc;
    CHIMERA_LAUNCH_CHECK("copy probe");
    *h_gbs = 2.0 * (double)bytes * reps / (ms * 1e-3) / 1e9;      // bytes read + bytes written
    return CHIMERA_OK;
}

}  // extern "C"
