// Small utility kernels: fills and copies that stay kernels (no memset nodes, so every per-frame
// call of the library can be captured into a HIP graph), and the int8 harness nonlinearity.
#include "rrm_internal.h"

namespace rrm {

namespace {

template <typename T>
__global__ void fill_bias_kernel(T* __restrict__ y, const T* __restrict__ bias, long long total, int c_out) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < total) y[i] = bias ? bias[i % c_out] : (T)0;
}

__global__ void fill_zero_kernel(uint4* __restrict__ p, long long nvec) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nvec) p[i] = make_uint4(0, 0, 0, 0);
}

__global__ void copy_kernel(uint4* __restrict__ dst, const unsigned char* __restrict__ src, long long nvec,
                            long long bytes) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nvec) return;
    if (i * 16 + 16 <= bytes) {
        dst[i] = *reinterpret_cast<const uint4*>(src + i * 16);
    } else {
        unsigned int w[4] = {0, 0, 0, 0};
        for (int k = 0; k < 16; ++k)
            if (i * 16 + k < bytes) w[k >> 2] |= (unsigned int)src[i * 16 + k] << (8 * (k & 3));
        dst[i] = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// out[n][ho][wo][c] = max over the 3x3/2 window (or identity) of min(127, max(0, y) >> shift)
__global__ void relu_requant_pool_kernel(const int* __restrict__ y, signed char* __restrict__ out, int n, int h, int w,
                                         int c, int ho, int wo, int shift, int pool) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long total = (long long)n * ho * wo * c;
    if (i >= total) return;
    const int ch = (int)(i % c);
    long long r = i / c;
    const int ox = (int)(r % wo);
    r /= wo;
    const int oy = (int)(r % ho);
    const int b = (int)(r / ho);
    int best = 0;
    if (pool) {
        for (int dy = 0; dy < 3; ++dy)
            for (int dx = 0; dx < 3; ++dx) {
                const int v = y[(((long long)b * h + 2 * oy + dy) * w + 2 * ox + dx) * c + ch];
                best = max(best, v);
            }
    } else {
        best = max(0, y[i]);
    }
    // max commutes with the monotone map v -> min(127, max(0, v) >> shift)
    best = min(127, best >> shift);
    out[i] = (signed char)best;
}

}  // namespace

hipError_t launch_fill_bias(int is_float, void* y, const void* bias, long long rows, int c_out, hipStream_t s) {
    const long long total = rows * c_out;
    if (total <= 0) return hipSuccess;
    dim3 grid((unsigned int)((total + 255) / 256)), block(256);
    if (is_float)
        hipLaunchKernelGGL(fill_bias_kernel<float>, grid, block, 0, s, (float*)y, (const float*)bias, total, c_out);
    else
        hipLaunchKernelGGL(fill_bias_kernel<int>, grid, block, 0, s, (int*)y, (const int*)bias, total, c_out);
    return hipGetLastError();
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
    const long long nvec = (long long)(bytes / 16);  // buffers are allocated in 16-byte multiples
    if (nvec <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned int)((nvec + 255) / 256)), dim3(256), 0, s, (uint4*)p, nvec);
    return hipGetLastError();
}

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
    const long long nvec = (long long)((bytes + 15) / 16);  // dst is allocated in 16-byte multiples
    if (nvec <= 0) return hipSuccess;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned int)((nvec + 255) / 256)), dim3(256), 0, s, (uint4*)dst,
                       (const unsigned char*)src, nvec, (long long)bytes);
    return hipGetLastError();
}

hipError_t launch_relu_requant_pool(const void* y, void* out, int n, int h, int w, int c, int shift, int pool,
                                    hipStream_t s) {
    const int ho = pool ? (h - 3) / 2 + 1 : h, wo = pool ? (w - 3) / 2 + 1 : w;
    const long long total = (long long)n * ho * wo * c;
    if (total <= 0) return hipSuccess;
    hipLaunchKernelGGL(relu_requant_pool_kernel, dim3((unsigned int)((total + 255) / 256)), dim3(256), 0, s,
                       (const int*)y, (signed char*)out, n, h, w, c, ho, wo, shift, pool);
    return hipGetLastError();
}

}  // namespace rrm
