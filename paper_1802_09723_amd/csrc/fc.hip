// Fully-connected sparse-delta path: P_t = P_{t-1} + W (I_t - I_{t-1})  (Algorithm 1, FC branch).
//
// The engine the paper relies on (Sec. 3.5) scans the activation vector for non-zero entries,
// broadcasts (a_j, j) and multiplies the weight column W_j, summing into row accumulators.  Here:
//   fc_scan     one workgroup per stream compares x_t with the snapshot, commits changes, and
//               compacts the changed entries (index j, difference a_j) into an ordered list with a
//               wavefront popcount + LDS prefix sum.
//   fc_scatter  streams only the listed columns.  The weights are stored input-major
//               (W^T [c_in][c_out], every column of W contiguous), each lane owns 16 bytes worth of
//               output channels, and the list is split over workgroups so that enough loads are in
//               flight to stream at memory speed; every split writes its partial sums to scratch.
//   fc_reduce   adds the partial sums of the splits, in split order, into the stored projection
//               (no atomics: exact for int32, and bit-reproducible run to run for fp32).
// The layer is memory-bound: bytes moved are (changed columns) x c_out x element size.
#include <type_traits>

#include "rrm_internal.h"

namespace rrm {

namespace {

constexpr int FC_SCAN_THREADS = 1024;
constexpr int FC_MIN_COLS = 8;  // columns per active workgroup before the list is split further

__device__ __forceinline__ float bf16_to_f32(unsigned int h) { return __uint_as_float(h << 16); }

template <int DT>
__global__ __launch_bounds__(FC_SCAN_THREADS) void fc_scan_kernel(const unsigned char* __restrict__ x_t,
                                                                  unsigned char* __restrict__ x_snap,
                                                                  int* __restrict__ idx, void* __restrict__ val_v,
                                                                  int* __restrict__ count, FcGeom g,
                                                                  DevStats* __restrict__ stats) {
    constexpr int PV = DT == RRM_I8_I32 ? 16 : 8;
    constexpr int ESIZE = DT == RRM_I8_I32 ? 1 : 2;
    typedef typename std::conditional<DT == RRM_I8_I32, int, float>::type val_t;
    val_t* val = static_cast<val_t*>(val_v);
    __shared__ int wave_tot[FC_SCAN_THREADS / 64];
    __shared__ int running;
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long row = (long long)b * g.c_in;
    const int nunits = (g.c_in + PV - 1) / PV;
    if (tid == 0) running = 0;
    __syncthreads();
    for (int u0 = 0; u0 < nunits; u0 += FC_SCAN_THREADS) {
        const int u = u0 + tid;
        val_t dv[PV];
        unsigned int mask = 0;
        const int e0 = u * PV;
        if (u < nunits) {
            if (g.vec_ok) {
                const uint4 a = *reinterpret_cast<const uint4*>(x_t + (row + e0) * ESIZE);
                uint4* sp = reinterpret_cast<uint4*>(x_snap + (row + e0) * ESIZE);
                const uint4 s = *sp;
                if ((a.x ^ s.x) | (a.y ^ s.y) | (a.z ^ s.z) | (a.w ^ s.w)) {
                    const unsigned int aw[4] = {a.x, a.y, a.z, a.w}, sw[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
                    for (int e = 0; e < PV; ++e) {
                        if (DT == RRM_I8_I32) {
                            const int xa = (int)(signed char)(aw[e >> 2] >> (8 * (e & 3)));
                            const int xb = (int)(signed char)(sw[e >> 2] >> (8 * (e & 3)));
                            dv[e] = (val_t)(xa - xb);
                            if (xa != xb) mask |= 1u << e;
                        } else {
                            const unsigned int xa = (aw[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                            const unsigned int xb = (sw[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                            dv[e] = (val_t)(bf16_to_f32(xa) - bf16_to_f32(xb));
                            if (xa != xb) mask |= 1u << e;
                        }
                    }
                    *sp = a;
                }
            } else {
                for (int e = 0; e < PV; ++e) {
                    dv[e] = 0;
                    if (e0 + e >= g.c_in) continue;
                    if (DT == RRM_I8_I32) {
                        const signed char xa = (signed char)x_t[row + e0 + e];
                        const signed char xb = (signed char)x_snap[row + e0 + e];
                        if (xa != xb) {
                            mask |= 1u << e;
                            dv[e] = (val_t)((int)xa - (int)xb);
                            x_snap[row + e0 + e] = (unsigned char)xa;
                        }
                    } else {
                        const unsigned short xa = reinterpret_cast<const unsigned short*>(x_t)[row + e0 + e];
                        unsigned short* sp = reinterpret_cast<unsigned short*>(x_snap) + row + e0 + e;
                        if (xa != *sp) {
                            mask |= 1u << e;
                            dv[e] = (val_t)(bf16_to_f32(xa) - bf16_to_f32(*sp));
                            *sp = xa;
                        }
                    }
                }
            }
        }
        // ---- ordered compaction: wave inclusive scan of the counts, then across waves in LDS -----
        const int cnt = __popc(mask);
        int incl = cnt;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(incl, o);
            if (lane >= o) incl += t;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        int wbase = 0, btot = 0;
        for (int w = 0; w < FC_SCAN_THREADS / 64; ++w) {
            const int t = wave_tot[w];
            if (w < wave) wbase += t;
            btot += t;
        }
        int pos = running + wbase + incl - cnt;
        if (mask) {
#pragma unroll
            for (int e = 0; e < PV; ++e)
                if (mask & (1u << e)) {
                    idx[row + pos] = e0 + e;
                    val[row + pos] = dv[e];
                    ++pos;
                }
        }
        __syncthreads();
        if (tid == 0) running += btot;
        __syncthreads();
    }
    if (tid == 0) {
        const int total = running;
        count[b] = total;
        if (total) {
            atomicAdd(&stats->changed_elems, (unsigned long long)total);
            atomicAdd(&stats->changed_units, (unsigned long long)total);
            atomicAdd(&stats->active_tiles, (unsigned long long)total);
        }
    }
}

// number of workgroups the column list is split over, from the list length (same in both kernels)
__device__ __forceinline__ int fc_active_splits(int cnt, int splits) {
    int s_eff = (cnt + FC_MIN_COLS - 1) / FC_MIN_COLS;
    return s_eff > splits ? splits : s_eff;
}

template <int DT, int DENSE>
__global__ __launch_bounds__(256) void fc_scatter_kernel(const unsigned char* __restrict__ wT,
                                                         const int* __restrict__ idx, const void* __restrict__ val_v,
                                                         const int* __restrict__ count,
                                                         const unsigned char* __restrict__ x, void* __restrict__ part_v,
                                                         FcGeom g, int splits) {
    constexpr int PV = DT == RRM_I8_I32 ? 16 : 8;
    constexpr int ESIZE = DT == RRM_I8_I32 ? 1 : 2;
    constexpr int UN = 8;  // columns in flight per lane
    typedef typename std::conditional<DT == RRM_I8_I32, int, float>::type val_t;
    const val_t* val = static_cast<const val_t*>(val_v);
    const int b = blockIdx.z, s = blockIdx.y;
    const int cnt = DENSE ? g.c_in : count[b];
    const int s_eff = fc_active_splits(cnt, splits);
    if (s >= s_eff) return;
    const int co0 = (blockIdx.x * 256 + threadIdx.x) * PV;
    if (co0 >= g.c_out_p) return;
    const long long row = (long long)b * g.c_in;
    val_t acc[PV];
#pragma unroll
    for (int e = 0; e < PV; ++e) acc[e] = 0;
    const unsigned char* wcol = wT + (long long)co0 * ESIZE;
    const long long pitch = (long long)g.c_out_p * ESIZE;

    auto column = [&](int k, int& j, val_t& d) {
        if (DENSE) {
            j = k;
            if (DT == RRM_I8_I32)
                d = (val_t)(int)(signed char)x[row + k];
            else
                d = (val_t)bf16_to_f32(reinterpret_cast<const unsigned short*>(x)[row + k]);
        } else {
            j = idx[row + k];
            d = val[row + k];
        }
    };
    auto fma16 = [&](const uint4& w, val_t d) {
        const unsigned int ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int e = 0; e < PV; ++e) {
            if (DT == RRM_I8_I32)
                acc[e] += d * (val_t)(int)(signed char)(ww[e >> 2] >> (8 * (e & 3)));
            else
                acc[e] += d * (val_t)__uint_as_float((e & 1) ? (ww[e >> 1] & 0xFFFF0000u) : (ww[e >> 1] << 16));
        }
    };

    int k = s;
    for (; k + (UN - 1) * s_eff < cnt; k += UN * s_eff) {
        int j[UN];
        val_t d[UN];
        uint4 w[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) column(k + u * s_eff, j[u], d[u]);
#pragma unroll
        for (int u = 0; u < UN; ++u) w[u] = *reinterpret_cast<const uint4*>(wcol + j[u] * pitch);
#pragma unroll
        for (int u = 0; u < UN; ++u) fma16(w[u], d[u]);
    }
    for (; k < cnt; k += s_eff) {
        int j0;
        val_t d0;
        column(k, j0, d0);
        fma16(*reinterpret_cast<const uint4*>(wcol + j0 * pitch), d0);
    }
    // partial sums of this split: scratch [stream][split][c_out_p]
    val_t* part = static_cast<val_t*>(part_v) + ((long long)b * splits + s) * g.c_out_p + co0;
#pragma unroll
    for (int e = 0; e < PV; e += 4) {
        typedef typename std::conditional<DT == RRM_I8_I32, int4, float4>::type vec_t;
        vec_t o;
        o.x = acc[e]; o.y = acc[e + 1]; o.z = acc[e + 2]; o.w = acc[e + 3];
        *reinterpret_cast<vec_t*>(part + e) = o;
    }
}

template <int DT, int DENSE>
__global__ __launch_bounds__(256) void fc_reduce_kernel(const void* __restrict__ part_v, const int* __restrict__ count,
                                                        const void* __restrict__ bias_v, void* __restrict__ y_v, FcGeom g,
                                                        int splits) {
    typedef typename std::conditional<DT == RRM_I8_I32, int, float>::type val_t;
    const int b = blockIdx.y;
    const int co = blockIdx.x * 256 + threadIdx.x;
    if (co >= g.c_out) return;
    const int cnt = DENSE ? g.c_in : count[b];
    const int s_eff = fc_active_splits(cnt, splits);
    const val_t* part = static_cast<const val_t*>(part_v) + (long long)b * splits * g.c_out_p + co;
    val_t sum = 0;
    int s = 0;
    for (; s + 3 < s_eff; s += 4) {  // four loads in flight, added in split order
        const val_t p0 = part[(long long)s * g.c_out_p], p1 = part[(long long)(s + 1) * g.c_out_p];
        const val_t p2 = part[(long long)(s + 2) * g.c_out_p], p3 = part[(long long)(s + 3) * g.c_out_p];
        sum += p0;
        sum += p1;
        sum += p2;
        sum += p3;
    }
    for (; s < s_eff; ++s) sum += part[(long long)s * g.c_out_p];
    val_t* y = static_cast<val_t*>(y_v) + (long long)b * g.c_out + co;
    if (DENSE) {
        const val_t* bias = static_cast<const val_t*>(bias_v);
        *y = (bias ? bias[co] : (val_t)0) + sum;
    } else if (sum != (val_t)0) {
        *y += sum;
    }
}

}  // namespace

hipError_t launch_fc_scan(int dtype, const void* x_t, void* x_snap, int* idx, void* val, int* count,
                          const FcGeom& g, DevStats* stats, hipStream_t s) {
    dim3 grid((unsigned int)g.n), block(FC_SCAN_THREADS);
    if (dtype == RRM_I8_I32)
        hipLaunchKernelGGL(fc_scan_kernel<RRM_I8_I32>, grid, block, 0, s, (const unsigned char*)x_t,
                           (unsigned char*)x_snap, idx, val, count, g, stats);
    else
        hipLaunchKernelGGL(fc_scan_kernel<RRM_BF16_F32>, grid, block, 0, s, (const unsigned char*)x_t,
                           (unsigned char*)x_snap, idx, val, count, g, stats);
    return hipGetLastError();
}

hipError_t launch_fc_scatter(int dtype, int dense, int splits, const void* wT, const int* idx, const void* val,
                             const int* count, const void* x, void* part, const void* bias, void* y, const FcGeom& g,
                             hipStream_t s) {
    dim3 grid((unsigned int)g.slices, (unsigned int)splits, (unsigned int)g.n), block(256);
    dim3 rgrid((unsigned int)((g.c_out + 255) / 256), (unsigned int)g.n);
    const unsigned char* w = static_cast<const unsigned char*>(wT);
    const unsigned char* xx = static_cast<const unsigned char*>(x);
#define RRM_FC(DTV, DV)                                                                                              \
    do {                                                                                                            \
        hipLaunchKernelGGL((fc_scatter_kernel<DTV, DV>), grid, block, 0, s, w, idx, val, count, xx, part, g, splits); \
        hipLaunchKernelGGL((fc_reduce_kernel<DTV, DV>), rgrid, block, 0, s, part, count, bias, y, g, splits);        \
    } while (0)
    if (dtype == RRM_I8_I32) {
        if (dense) RRM_FC(RRM_I8_I32, 1); else RRM_FC(RRM_I8_I32, 0);
    } else {
        if (dense) RRM_FC(RRM_BF16_F32, 1); else RRM_FC(RRM_BF16_F32, 0);
    }
#undef RRM_FC
    return hipGetLastError();
}

}  // namespace rrm
