// Fully-connected layers with many streams: the layer is a skinny matrix product, W [c_out x c_in] times the
// streams' vectors [c_in x n], and it runs on the matrix cores with W read once for all streams.
//
// Dense layer (Eq. 3, FC form):      Y = b + W X^T
// Delta step (Algorithm 1, FC branch), int8: Y += W D^T with D = X_t - X_{t-1} for all streams, in two launches:
//   fc_diff_kernel     writes D (the byte differences), commits the stored input and counts the changes;
//   fc_batched_kernel  multiplies.  With tens of streams the union of the changed columns is most of the matrix
//                      (64 streams at 1 % each already touch half of the columns), so the product runs over all of
//                      W: its cost is one pass over W whatever the density, a tenth of what n separate column walks
//                      cost at 64 streams.
// bf16: the fp32 difference of two bf16 values needs two bf16 terms (hi and lo), so the delta product would be two
// passes of matrix instructions for the same pass over W that the layer itself takes; the step therefore commits,
// counts and recomputes Y = b + W X_t^T (which is also free of the step-to-step rounding of an accumulated sum).
// Shapes: v_mfma_i32_16x16x64_i8 / v_mfma_f32_16x16x32_bf16.  Lane l of a wavefront supplies 16 bytes of A (row
// l % 16 of a 16-row block of W, k-group l / 16: contiguous in W's own row-major layout) and 16 bytes of B (stream
// l % 16 of a 16-stream tile, same k-group: contiguous in a stream's vector), and receives rows 4 (l / 16) .. + 3
// of column l % 16: four consecutive output channels of one stream, one 16-byte store.
// Workgroup = one 16-row block of W, eight (four) wavefronts on interleaved 64-byte k-steps; their sums are added through
// LDS in a fixed order (bit-reproducible fp32), so c_out / 16 workgroups each read their rows of W exactly once and
// the streams' vectors (a few hundred KB, resident in L2) once each.
#include <type_traits>

#include "rrm_internal.h"

namespace rrm {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));


// D = x_t - x_snap for every stream, x_snap <- x_t, change counts.  One thread per 16-byte unit.  !WRITE_D: the commit
// and the counts only (the step recomputes the layer from x_t).
template <int DT, bool WRITE_D>
__global__ __launch_bounds__(256) void fc_diff_kernel(const uint4* __restrict__ x_t, uint4* __restrict__ x_snap,
                                                      uint4* __restrict__ d0, uint4* __restrict__ d1, long long nvec,
                                                      unsigned long long n_cin, DevStats* __restrict__ stats) {
    const long long v = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    unsigned int nchanged = 0;
    if (v < nvec) {
        const uint4 a = x_t[v], s = x_snap[v];
        uint4 hi = make_uint4(0, 0, 0, 0), lo = hi;
        if ((a.x ^ s.x) | (a.y ^ s.y) | (a.z ^ s.z) | (a.w ^ s.w)) {
            const unsigned int aw[4] = {a.x, a.y, a.z, a.w}, sw[4] = {s.x, s.y, s.z, s.w};
            unsigned int hw[4], lw[4] = {0u, 0u, 0u, 0u};
            if (DT == RRM_I8_I32) {
                const unsigned int H = 0x80808080u;
                unsigned int ovf = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    // byte-wise wrapping subtraction and its signed-overflow mask
                    const unsigned int d = ((aw[i] | H) - (sw[i] & ~H)) ^ ((aw[i] ^ ~sw[i]) & H);
                    ovf |= (aw[i] ^ sw[i]) & (aw[i] ^ d) & H;
                    hw[i] = d;
                    const unsigned int z = aw[i] ^ sw[i];
                    nchanged += __popc((((z & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | z) & H);
                }
                if (ovf) atomicOr(&stats->range_error, 1u);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    unsigned int h2 = 0, l2 = 0;
#pragma unroll
                    for (int k = 0; k < 2; ++k) {
                        const unsigned int xa = (aw[i] >> (16 * k)) & 0xFFFFu, xb = (sw[i] >> (16 * k)) & 0xFFFFu;
                        if (xa == xb) continue;
                        ++nchanged;
                        if (!WRITE_D) continue;
                        const float d = __uint_as_float(xa << 16) - __uint_as_float(xb << 16);
                        // round-to-nearest-even bf16 of d, and of what is left
                        auto to_bf16 = [](float f) {
                            const unsigned int u = __float_as_uint(f);
                            return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
                        };
                        const unsigned int h = to_bf16(d);
                        const unsigned int l = to_bf16(d - __uint_as_float(h << 16));
                        h2 |= (h & 0xFFFFu) << (16 * k);
                        l2 |= (l & 0xFFFFu) << (16 * k);
                    }
                    hw[i] = h2;
                    lw[i] = l2;
                }
            }
            hi = make_uint4(hw[0], hw[1], hw[2], hw[3]);
            lo = make_uint4(lw[0], lw[1], lw[2], lw[3]);
            x_snap[v] = a;
        }
        if (WRITE_D) {
            d0[v] = hi;
            if (DT == RRM_BF16_F32) d1[v] = lo;
        }
    }
    // counts: wavefront, then workgroup, then one set of atomics
    __shared__ unsigned int s_n[4];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) nchanged += __shfl_xor(nchanged, o);
    if ((threadIdx.x & 63) == 0) s_n[threadIdx.x >> 6] = nchanged;
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int tot = s_n[0] + s_n[1] + s_n[2] + s_n[3];
        if (tot) {
            atomicAdd(&stats->changed_elems, (unsigned long long)tot);
            atomicAdd(&stats->changed_units, (unsigned long long)tot);
            atomicAdd(&stats->active_tiles, (unsigned long long)tot);
        }
        if (blockIdx.x == 0) {  // one launch = one delta step
            atomicAdd(&stats->delta_steps, 1ull);
            atomicAdd(&stats->total_tiles, n_cin);
        }
    }
}

// Y (+)= W B^T.  w: [c_out][c_in] row-major; b0 (b1): [n][c_in] (the streams' vectors, or the difference's terms);
// y: [n][c_out].  DELTA: y is read and added to (TERMS planes of B); else y = bias + product.
// TMAX bounds the 16-stream tiles (accumulators), WAVES wavefronts share the k-steps of the rows, and every
// wavefront issues the loads of U steps before it multiplies the first: the loop is bound by memory latency otherwise
// (a step is one 64-byte piece of a row and of every stream's vector).
template <int DT, bool DELTA, int TERMS, int TMAX, int WAVES, int U>
__global__ __launch_bounds__(WAVES * 64) void fc_batched_kernel(const unsigned char* __restrict__ w,
                                                                const unsigned char* __restrict__ b0,
                                                                const unsigned char* __restrict__ b1,
                                                                const void* __restrict__ bias_v, void* y_v, FcGeom g,
                                                                int ntiles) {
    constexpr int ESIZE = DT == RRM_I8_I32 ? 1 : 2;
    constexpr int KSTEP = 64 / ESIZE;  // elements per MFMA step: 64 int8 / 32 bf16 (64 bytes of a row)
    typedef typename std::conditional<DT == RRM_I8_I32, int, float>::type val_t;
    typedef typename std::conditional<DT == RRM_I8_I32, v4i, v4f>::type acc_t;
    __shared__ acc_t red[WAVES - 1][TMAX][64];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int o0 = (int)blockIdx.x * 16;
    const int row = o0 + (lane & 15);  // (c_out is a multiple of 16: every row exists)
    const int kg = lane >> 4;          // k-group: bytes 16 kg .. 16 kg + 15 of a 64-byte step
    const long long row_bytes = (long long)g.c_in * ESIZE;
    const unsigned char* wp = w + (long long)row * row_bytes + kg * 16;
    const int nsteps = g.c_in / KSTEP;
    // this lane's stream in tile t is 16 t + lane % 16; streams beyond n read stream n - 1 (their columns are not stored)
    const unsigned char* bp0[TMAX];
    const unsigned char* bp1[TMAX];
#pragma unroll
    for (int t = 0; t < TMAX; ++t) {
        int s = 16 * t + (lane & 15);
        s = s < g.n ? s : g.n - 1;
        bp0[t] = b0 + (long long)s * row_bytes + kg * 16;
        bp1[t] = TERMS == 2 ? b1 + (long long)s * row_bytes + kg * 16 : nullptr;
    }

    acc_t acc[TMAX];
#pragma unroll
    for (int t = 0; t < TMAX; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[t][i] = 0;

    auto mma = [&](const uint4& a, const uint4& b, acc_t c) {
        if constexpr (DT == RRM_I8_I32)
            return __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(v4i, a), __builtin_bit_cast(v4i, b), c, 0, 0, 0);
        else
            return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
    };
    // two register sets: the loads of the next U steps are issued before the current U steps are multiplied
    struct Ops {
        uint4 a[U], bh[U][TMAX], bl[U][TERMS == 2 ? TMAX : 1];
    };
    auto load = [&](int st0, Ops& o) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int st = st0 + u * WAVES;
            const long long off = (long long)(st < nsteps ? st : wave) * 64;  // (a step beyond the end re-reads the first: not used)
            o.a[u] = *reinterpret_cast<const uint4*>(wp + off);
#pragma unroll
            for (int t = 0; t < TMAX; ++t)
                if (t < ntiles) {
                    o.bh[u][t] = *reinterpret_cast<const uint4*>(bp0[t] + off);
                    if (TERMS == 2) o.bl[u][t] = *reinterpret_cast<const uint4*>(bp1[t] + off);
                }
        }
    };
    auto multiply = [&](int st0, const Ops& o) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (st0 + u * WAVES >= nsteps) break;
#pragma unroll
            for (int t = 0; t < TMAX; ++t)
                if (t < ntiles) {
                    acc[t] = mma(o.a[u], o.bh[u][t], acc[t]);
                    if (TERMS == 2) acc[t] = mma(o.a[u], o.bl[u][t], acc[t]);
                }
        }
    };
    Ops ra, rb;
    constexpr int STRIDE = WAVES * U;
    load(wave, ra);
    for (int st0 = wave; st0 < nsteps; st0 += 2 * STRIDE) {
        if (st0 + STRIDE < nsteps) load(st0 + STRIDE, rb);
        multiply(st0, ra);
        if (st0 + STRIDE < nsteps) {
            if (st0 + 2 * STRIDE < nsteps) load(st0 + 2 * STRIDE, ra);
            multiply(st0 + STRIDE, rb);
        }
    }
    // ---- the wavefronts' sums, added in a fixed order ---------------------------------------------------------
    if (wave > 0) {
#pragma unroll
        for (int t = 0; t < TMAX; ++t)
            if (t < ntiles) red[wave - 1][t][lane] = acc[t];
    }
    __syncthreads();
    if (wave == 0) {
        val_t* y = static_cast<val_t*>(y_v);
        const val_t* bias = static_cast<const val_t*>(bias_v);
        const int oc = o0 + 4 * (lane >> 4);  // this lane's four consecutive output channels
#pragma unroll
        for (int t = 0; t < TMAX; ++t) {
            if (t >= ntiles) continue;
            acc_t sum = acc[t];
#pragma unroll
            for (int q = 0; q < WAVES - 1; ++q) {
                const acc_t o = red[q][t][lane];
#pragma unroll
                for (int i = 0; i < 4; ++i) sum[i] += o[i];
            }
            const int s = 16 * t + (lane & 15);
            if (s >= g.n) continue;
            acc_t* yp = reinterpret_cast<acc_t*>(y + (long long)s * g.c_out + oc);  // (c_out % 16 == 0: 16-byte aligned)
            acc_t base;
            if (DELTA) {
                base = *yp;
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) base[i] = bias ? bias[oc + i] : (val_t)0;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) base[i] += sum[i];
            *yp = base;
        }
    }
}

template <int DT, bool DELTA, int TERMS>
void launch_batched(const void* w_rm, const void* b0, const void* b1, const void* bias, void* y, const FcGeom& g,
                    hipStream_t s) {
    const int ntiles = (g.n + 15) / 16;
    dim3 grid((unsigned int)(g.c_out / 16));
    const unsigned char* w = static_cast<const unsigned char*>(w_rm);
    const unsigned char* p0 = static_cast<const unsigned char*>(b0);
    const unsigned char* p1 = static_cast<const unsigned char*>(b1);
    // (two-term products hold twice the operands: half the steps in flight)
    if (ntiles <= 4)
        hipLaunchKernelGGL((fc_batched_kernel<DT, DELTA, TERMS, 4, 8, TERMS == 2 ? 1 : 2>), grid, dim3(512), 0, s, w, p0, p1, bias, y, g, ntiles);
    else if (ntiles <= 8)
        hipLaunchKernelGGL((fc_batched_kernel<DT, DELTA, TERMS, 8, 8, 1>), grid, dim3(512), 0, s, w, p0, p1, bias, y, g, ntiles);
    else
        hipLaunchKernelGGL((fc_batched_kernel<DT, DELTA, TERMS, 16, 4, 1>), grid, dim3(256), 0, s, w, p0, p1, bias, y, g, ntiles);
}

}  // namespace

bool fc_batched_ok(int dtype, const FcGeom& g) {
    const int esize = dtype == RRM_I8_I32 ? 1 : 2;
    return g.n >= FC_BATCH_MIN_STREAMS && g.n <= FC_BATCH_MAX_STREAMS && g.c_out % 16 == 0 && (g.c_in * esize) % 64 == 0;
}

hipError_t launch_fc_batched_dense(int dtype, const void* w_rm, const void* x, const void* bias, void* y, const FcGeom& g,
                                   hipStream_t s) {
    if (!fc_batched_ok(dtype, g)) return hipErrorInvalidValue;
    if (dtype == RRM_I8_I32)
        launch_batched<RRM_I8_I32, false, 1>(w_rm, x, nullptr, bias, y, g, s);
    else
        launch_batched<RRM_BF16_F32, false, 1>(w_rm, x, nullptr, bias, y, g, s);
    return hipGetLastError();
}

hipError_t launch_fc_batched_delta(int dtype, const void* w_rm, const void* x_t, void* x_snap, void* d0, void* d1,
                                   const void* bias, void* y, const FcGeom& g, DevStats* stats, hipStream_t s) {
    if (!fc_batched_ok(dtype, g) || g.eps != 0.0f) return hipErrorInvalidValue;
    const int esize = dtype == RRM_I8_I32 ? 1 : 2;
    const long long nvec = (long long)g.n * g.c_in * esize / 16;
    const unsigned long long n_cin = (unsigned long long)g.n * (unsigned long long)g.c_in;
    dim3 dgrid((unsigned int)((nvec + 255) / 256)), dblock(256);
    if (dtype == RRM_I8_I32) {
        hipLaunchKernelGGL((fc_diff_kernel<RRM_I8_I32, true>), dgrid, dblock, 0, s, (const uint4*)x_t, (uint4*)x_snap, (uint4*)d0,
                           (uint4*)d1, nvec, n_cin, stats);
        launch_batched<RRM_I8_I32, true, 1>(w_rm, d0, nullptr, nullptr, y, g, s);
    } else {
        // bf16: the difference needs two bf16 terms, i.e. two products over all of W, while the layer itself (Eq. 3)
        // is one -- and it does not accumulate rounding from step to step.  The step commits, counts and recomputes.
        hipLaunchKernelGGL((fc_diff_kernel<RRM_BF16_F32, false>), dgrid, dblock, 0, s, (const uint4*)x_t, (uint4*)x_snap,
                           (uint4*)nullptr, (uint4*)nullptr, nvec, n_cin, stats);
        launch_batched<RRM_BF16_F32, false, 1>(w_rm, x_t, nullptr, bias, y, g, s);
    }
    return hipGetLastError();
}

}  // namespace rrm
