// Two measurement probes for the benchmark: what this chip sustains on a register-resident MFMA loop and on a
// large streaming copy.  The benchmark prices its kernels against the published peaks and against these.
#include "rrm_internal.h"

namespace rrm {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr int PROBE_ACC = 4;  // independent accumulator chains per wavefront (covers the issue-to-use latency)

// every wavefront: iters x PROBE_ACC products of 32x32x32 (int8) tiles, operands and sums in registers
__global__ __launch_bounds__(256) void probe_mfma_i8_kernel(int* __restrict__ sink, int iters) {
    v4i a, b;
    for (int k = 0; k < 4; ++k) {
        a[k] = (int)threadIdx.x * 0x01010101 + k;
        b[k] = (int)blockIdx.x + k;
    }
    v16i acc[PROBE_ACC];
    for (int j = 0; j < PROBE_ACC; ++j)
        for (int k = 0; k < 16; ++k) acc[j][k] = 0;
    for (int i = 0; i < iters; ++i)
        for (int j = 0; j < PROBE_ACC; ++j) acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[j], 0, 0, 0);
    int s = 0;
    for (int j = 0; j < PROBE_ACC; ++j)
        for (int k = 0; k < 16; ++k) s += acc[j][k];
    if (s == 0x7fffffff) sink[0] = s;  // (keeps the loop alive; practically never taken)
}

__global__ __launch_bounds__(256) void probe_mfma_bf16_kernel(float* __restrict__ sink, int iters) {
    v8bf a, b;
    for (int k = 0; k < 8; ++k) {
        a[k] = (__bf16)(float)((threadIdx.x + k) & 7);
        b[k] = (__bf16)(float)((blockIdx.x + k) & 3);
    }
    v16f acc[PROBE_ACC];
    for (int j = 0; j < PROBE_ACC; ++j)
        for (int k = 0; k < 16; ++k) acc[j][k] = 0.0f;
    for (int i = 0; i < iters; ++i)
        for (int j = 0; j < PROBE_ACC; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    float s = 0.0f;
    for (int j = 0; j < PROBE_ACC; ++j)
        for (int k = 0; k < 16; ++k) s += acc[j][k];
    if (s == -1.0f) sink[0] = s;
}

// grid-stride copy of 16-byte vectors, four loads in flight per lane: every byte read once and written once
__global__ __launch_bounds__(256) void probe_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t nvec) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < nvec; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        dst[i] = a;
        dst[i + stride] = b;
        dst[i + 2 * stride] = c;
        dst[i + 3 * stride] = d;
    }
    for (; i < nvec; i += stride) dst[i] = src[i];
}

}  // namespace

hipError_t launch_probe_mfma(int is_bf16, void* sink, int iters, int workgroups, hipStream_t s) {
    if (is_bf16)
        hipLaunchKernelGGL(probe_mfma_bf16_kernel, dim3((unsigned int)workgroups), dim3(256), 0, s, (float*)sink, iters);
    else
        hipLaunchKernelGGL(probe_mfma_i8_kernel, dim3((unsigned int)workgroups), dim3(256), 0, s, (int*)sink, iters);
    return hipGetLastError();
}

hipError_t launch_probe_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
    const size_t nvec = bytes / 16;
    if (nvec == 0) return hipSuccess;
    const size_t want = (nvec + 255) / 256;
    const unsigned int grid = (unsigned int)(want < (size_t)NUM_CU * 32 ? want : (size_t)NUM_CU * 32);
    hipLaunchKernelGGL(probe_copy_kernel, dim3(grid), dim3(256), 0, s, (uint4*)dst, (const uint4*)src, nvec);
    return hipGetLastError();
}

}  // namespace rrm
