// Diagnostics: what the INT8 matrix cores of the device deliver on their own, with no
// memory traffic at all -- the ceiling against which the batched GEMM of Algorithm 1
// line 6 is read.  The published peak assumes the boost clock; the clock that the chip
// sustains depends on how many operand bits toggle, so the probe runs either on constant
// operands or on pseudo-random ones (residues are close to uniform over [-128, 127]).
#include <hip/hip_runtime.h>

#include "../../include/oz2.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kProbeThreads = 256;     // one wavefront per SIMD
constexpr int kProbeAcc = 8;           // independent accumulators per wavefront
constexpr int kProbeOps = 8;           // distinct operand registers per side

__device__ inline uint32_t mix(uint32_t x) {      // integer hash (xorshift-multiply rounds)
    x ^= x >> 16; x *= 0x7feb352du;
    x ^= x >> 15; x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

// Every wavefront issues iters * kProbeAcc * kProbeOps v_mfma_i32_32x32x32_i8 back to back.
// Consecutive instructions of the pipeline see different operand registers, so with
// random contents the multiplier inputs toggle the way a stream of residues makes them.
__global__ __launch_bounds__(kProbeThreads) void k_mfma_probe(int *out, int iters, int random_operands) {
    v4i a[kProbeOps], b[kProbeOps];
    const uint32_t id = blockIdx.x * kProbeThreads + threadIdx.x;
#pragma unroll
    for (int i = 0; i < kProbeOps; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            a[i][c] = random_operands ? (int)mix(id * 64u + i * 8u + c) : 0x01010101;
            b[i][c] = random_operands ? (int)mix(id * 64u + i * 8u + c + 4u) : 0x01010101;
        }
    v16i acc[kProbeAcc];
#pragma unroll
    for (int i = 0; i < kProbeAcc; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int o = 0; o < kProbeOps; ++o)
#pragma unroll
            for (int i = 0; i < kProbeAcc; ++i)
                acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[(o + i) % kProbeOps], b[o], acc[i], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < kProbeAcc; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[id] = s;
}

}  // namespace

extern "C" oz2_status oz2_mfma_probe(int random_operands, double seconds, double *tops, int *compute_units,
                                     int *clock_mhz) {
    if (!tops || !(seconds > 0.0) || seconds > 5.0) return OZ2_INVALID_ARG;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return OZ2_HIP_ERROR;
    if (compute_units) *compute_units = prop.multiProcessorCount;
    if (clock_mhz) *clock_mhz = prop.clockRate / 1000;
    // Two workgroups per compute unit: two wavefronts per SIMD, as in the GEMM.
    const int blocks = 2 * prop.multiProcessorCount;
    int *out = nullptr;
    if (hipMalloc(&out, sizeof(int) * (size_t)blocks * kProbeThreads) != hipSuccess) return OZ2_WORKSPACE;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    oz2_status st = OZ2_HIP_ERROR;
    float ms = 0.f;
    const double ops_per_iter = (double)blocks * (kProbeThreads / 64) * kProbeAcc * kProbeOps * 65536.0;
    // One short launch sizes the timed one (the sustained clock is what is being measured,
    // so the timed launch has to last long enough for the power management to settle).
    int iters = 2000;
    if (hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess) {
        for (int pass = 0; pass < 2; ++pass) {
            (void)hipEventRecord(e0, nullptr);
            hipLaunchKernelGGL(k_mfma_probe, dim3(blocks), dim3(kProbeThreads), 0, nullptr, out, iters, random_operands);
            (void)hipEventRecord(e1, nullptr);
            if (hipGetLastError() != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                hipEventElapsedTime(&ms, e0, e1) != hipSuccess || !(ms > 0.f)) {
                ms = 0.f;
                break;
            }
            if (pass == 0) {
                double want = iters * (seconds * 1e3 / ms);
                iters = want > 2e8 ? 200000000 : (want < 2000 ? 2000 : (int)want);
            }
        }
        if (ms > 0.f) {
            *tops = ops_per_iter * iters / (ms * 1e-3) / 1e12;
            st = OZ2_OK;
        }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(out);
    return st;
}
