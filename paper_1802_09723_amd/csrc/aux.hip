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

__global__ void fill_word_kernel(uint4* __restrict__ p, long long nvec, unsigned int word) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nvec) p[i] = make_uint4(word, word, word, word);
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

// The same map, four channels per thread (16-byte loads of y), one workgroup row per output row.  With
// CHANGED, an output is recomputed only if one of the blocks of y under its window was written by the layer's
// last step (byte flags `touched`, one per block of (1 << tshift)^2 positions); the rest of `out` keeps its value
// from the previous call.
template <bool CHANGED>
__global__ __launch_bounds__(256) void relu_requant_pool4_kernel(const int4* __restrict__ y, unsigned int* __restrict__ out,
                                                                 const unsigned char* __restrict__ touched,
                                                                 const unsigned int* __restrict__ touched_all, int tshift,
                                                                 int h, int w, int c4, int ho, int wo, int shift, int pool,
                                                                 unsigned int magic_c4, unsigned int magic_ho) {
    const int row = (int)blockIdx.x;  // b*ho + oy
    const int idx = (int)(blockIdx.y * blockDim.x + threadIdx.x);
    if (idx >= wo * c4) return;
    const int b = (int)udiv_magic((unsigned int)row, (unsigned int)ho, magic_ho);
    const int oy = row - b * ho;
    const int ox = (int)udiv_magic((unsigned int)idx, (unsigned int)c4, magic_c4);
    const int cv = idx - ox * c4;
    const int y0 = pool ? 2 * oy : oy, x0 = pool ? 2 * ox : ox;
    const int span = pool ? 2 : 0;
    if (CHANGED && touched_all[0] == 0u) {
        const int rnd = (1 << tshift) - 1;
        const int sty = (h + rnd) >> tshift, stx = (w + rnd) >> tshift;
        const unsigned char* t = touched + (size_t)b * sty * stx;
        const int sy0 = y0 >> tshift, sy1 = (y0 + span) >> tshift, sx0 = x0 >> tshift, sx1 = (x0 + span) >> tshift;
        unsigned int any = 0;
        for (int sy = sy0; sy <= sy1; ++sy)
            for (int sx = sx0; sx <= sx1; ++sx) any |= t[sy * stx + sx];
        if (!any) return;
    }
    int4 best = make_int4(0, 0, 0, 0);
    const int4* yb = y + ((size_t)(b * h + y0) * w + x0) * c4 + cv;
    for (int dy = 0; dy <= span; ++dy)
        for (int dx = 0; dx <= span; ++dx) {
            const int4 v = yb[(size_t)(dy * w + dx) * c4];
            best.x = max(best.x, v.x);
            best.y = max(best.y, v.y);
            best.z = max(best.z, v.z);
            best.w = max(best.w, v.w);
        }
    // max commutes with the monotone map v -> min(127, max(0, v) >> shift)
    const unsigned int o = (unsigned int)min(127, best.x >> shift) | (unsigned int)min(127, best.y >> shift) << 8 |
                           (unsigned int)min(127, best.z >> shift) << 16 | (unsigned int)min(127, best.w >> shift) << 24;
    out[(size_t)(row * wo + ox) * c4 + cv] = o;
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

hipError_t launch_fill_word(void* p, size_t bytes, unsigned int word, hipStream_t s) {
    const long long nvec = (long long)(bytes / 16);  // buffers are allocated in 16-byte multiples
    if (nvec <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_word_kernel, dim3((unsigned int)((nvec + 255) / 256)), dim3(256), 0, s, (uint4*)p, nvec, word);
    return hipGetLastError();
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) { return launch_fill_word(p, bytes, 0u, s); }

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
    const long long nvec = (long long)((bytes + 15) / 16);  // dst is allocated in 16-byte multiples
    if (nvec <= 0) return hipSuccess;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned int)((nvec + 255) / 256)), dim3(256), 0, s, (uint4*)dst,
                       (const unsigned char*)src, nvec, (long long)bytes);
    return hipGetLastError();
}

hipError_t launch_relu_requant_pool(const void* y, void* out, const void* touched, const unsigned int* touched_all,
                                    int tshift, int n, int h, int w, int c, int shift, int pool, hipStream_t s) {
    const int ho = pool ? (h - 3) / 2 + 1 : h, wo = pool ? (w - 3) / 2 + 1 : w;
    const long long total = (long long)n * ho * wo * c;
    if (total <= 0) return hipSuccess;
    if (c % 4 == 0 && (reinterpret_cast<uintptr_t>(y) & 15) == 0 && (reinterpret_cast<uintptr_t>(out) & 3) == 0) {
        const int c4 = c / 4;
        auto magic = [](int d) { return d <= 1 ? 0u : (unsigned int)((1ull << 32) / (unsigned long long)d + 1ull); };
        dim3 grid((unsigned int)(n * ho), (unsigned int)((wo * c4 + 255) / 256));
        if (touched)
            hipLaunchKernelGGL(relu_requant_pool4_kernel<true>, grid, dim3(256), 0, s, (const int4*)y, (unsigned int*)out,
                               (const unsigned char*)touched, touched_all, tshift, h, w, c4, ho, wo, shift, pool, magic(c4), magic(ho));
        else
            hipLaunchKernelGGL(relu_requant_pool4_kernel<false>, grid, dim3(256), 0, s, (const int4*)y, (unsigned int*)out,
                               (const unsigned char*)nullptr, (const unsigned int*)nullptr, 0, h, w, c4, ho, wo, shift, pool, magic(c4), magic(ho));
        return hipGetLastError();
    }
    if (touched) return hipErrorInvalidValue;  // the incremental form needs channel counts in fours
    hipLaunchKernelGGL(relu_requant_pool_kernel, dim3((unsigned int)((total + 255) / 256)), dim3(256), 0, s,
                       (const int*)y, (signed char*)out, n, h, w, c, ho, wo, shift, pool);
    return hipGetLastError();
}

}  // namespace rrm
