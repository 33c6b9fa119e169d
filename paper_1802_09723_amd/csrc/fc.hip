// Fully-connected sparse-delta path: P_t = P_{t-1} + W (I_t - I_{t-1})  (Algorithm 1, FC branch).
//
// The engine the paper relies on (Sec. 3.5) scans the activation vector for non-zero entries,
// broadcasts (a_j, j) and multiplies the weight column W_j, summing into row accumulators.  Here:
//   fc_scan     one workgroup per stream compares x_t with the snapshot, commits changes, and
//               compacts the changed entries (index j, difference a_j) into an ordered list with a
//               wavefront popcount + LDS prefix sum.
//   fc_scatter  streams only the listed columns.  The weights are stored input-major
//               (W^T [c_in][c_out], every column of W contiguous), each lane owns 16 bytes worth of
//               output channels, and the list is split over workgroups (and over four column groups
//               inside a workgroup, combined through LDS) so that enough loads are in flight to stream
//               at memory speed; every split writes its partial sums to scratch.
//   fc_reduce   adds the partial sums of the splits, in a fixed order, into the stored projection
//               (no atomics: exact for int32, and bit-reproducible run to run for fp32).
// The layer is memory-bound: bytes moved are (changed columns) x c_out x element size.
#include <type_traits>

#include "rrm_internal.h"

namespace rrm {

namespace {

constexpr int FC_SCAN_THREADS = 1024;
constexpr int FC_MIN_COLS = 2;  // columns per active workgroup before the list is split further

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
    unsigned int ntrunc = 0;  // truncated differences of this thread (bf16 with a threshold) and their squares
    float tsq = 0.f;
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
                    unsigned int nw[4] = {a.x, a.y, a.z, a.w};  // the unit's new snapshot
#pragma unroll
                    for (int e = 0; e < PV; ++e) {
                        if (DT == RRM_I8_I32) {
                            const int xa = (int)(signed char)(aw[e >> 2] >> (8 * (e & 3)));
                            const int xb = (int)(signed char)(sw[e >> 2] >> (8 * (e & 3)));
                            dv[e] = (val_t)(xa - xb);
                            if (xa != xb) mask |= 1u << e;
                        } else {
                            // (truncation threshold, Sec. 3.3 "Improving sparsity": a difference below g.eps is
                            // neither listed nor committed; eps = 0 is the exact method)
                            const unsigned int xa = (aw[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                            const unsigned int xb = (sw[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                            const float d = bf16_to_f32(xa) - bf16_to_f32(xb);
                            dv[e] = (val_t)d;
                            if (xa != xb) {
                                if (fabsf(d) < g.eps) {
                                    ++ntrunc;
                                    tsq += d * d;
                                    nw[e >> 1] = (nw[e >> 1] & ~(0xFFFFu << (16 * (e & 1)))) | (xb << (16 * (e & 1)));
                                } else {
                                    mask |= 1u << e;
                                }
                            }
                        }
                    }
                    if (mask) *sp = make_uint4(nw[0], nw[1], nw[2], nw[3]);
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
                            const float d = bf16_to_f32(xa) - bf16_to_f32(*sp);
                            if (fabsf(d) < g.eps) {
                                ++ntrunc;
                                tsq += d * d;
                            } else {
                                mask |= 1u << e;
                                dv[e] = (val_t)d;
                                *sp = xa;
                            }
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
    if (DT == RRM_BF16_F32) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            ntrunc += __shfl_xor(ntrunc, o);
            tsq += __shfl_xor(tsq, o);
        }
        if (lane == 0 && ntrunc) {
            atomicAdd(&stats->truncated_elems, (unsigned long long)ntrunc);
            atomicAdd(&stats->truncated_sumsq, (double)tsq);
        }
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

constexpr int FC_KG = 4;          // column groups of a scatter workgroup (1024 threads = 4 x 256 lanes)
constexpr int FC_RG = 8;          // split groups of a reduce workgroup (1024 threads = 8 x 128 lanes)
constexpr int FC_MAX_SPLITS = 64;

// number of workgroups the column list is split over, from the list length (same in both kernels)
__device__ __forceinline__ int fc_active_splits(int cnt, int splits) {
    int s_eff = (cnt + FC_KG * FC_MIN_COLS - 1) / (FC_KG * FC_MIN_COLS);
    if (s_eff < 1) s_eff = 1;
    return s_eff > splits ? splits : s_eff;
}

// Workgroup (slice, split s, stream): 256 lanes of 16 bytes of output channels each, times FC_KG column
// groups; column group kg of split s takes columns s*FC_KG + kg, + s_eff*FC_KG, ... of the list.  The four
// groups' sums are added through LDS, so a split leaves one row of partial sums.
template <int DT, int DENSE>
__global__ __launch_bounds__(FC_KG * 256) void fc_scatter_kernel(const unsigned char* __restrict__ wT,
                                                                 const int* __restrict__ idx, const void* __restrict__ val_v,
                                                                 const int* __restrict__ count,
                                                                 const unsigned char* __restrict__ x,
                                                                 void* __restrict__ part_v, FcGeom g, int splits) {
    constexpr int PV = DT == RRM_I8_I32 ? 16 : 8;
    constexpr int ESIZE = DT == RRM_I8_I32 ? 1 : 2;
    constexpr int UN = 8;  // columns in flight per lane
    typedef typename std::conditional<DT == RRM_I8_I32, int, float>::type val_t;
    typedef typename std::conditional<DT == RRM_I8_I32, int4, float4>::type vec_t;
    __shared__ vec_t red[FC_KG - 1][PV / 4][256];
    const val_t* val = static_cast<const val_t*>(val_v);
    const int b = blockIdx.z, s = blockIdx.y;
    const int cnt = DENSE ? g.c_in : count[b];
    const int s_eff = fc_active_splits(cnt, splits);
    if (s >= s_eff) return;  // (the whole workgroup)
    const int lane = threadIdx.x & 255, kg = threadIdx.x >> 8;
    const int co0 = (blockIdx.x * 256 + lane) * PV;
    const bool live = co0 < g.c_out_p;
    const long long row = (long long)b * g.c_in;
    val_t acc[PV];
#pragma unroll
    for (int e = 0; e < PV; ++e) acc[e] = 0;
    const unsigned char* wcol = wT + (long long)(live ? co0 : 0) * ESIZE;
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

    if (live) {
        const int step = s_eff * FC_KG;
        int k = s * FC_KG + kg;
        for (; k + (UN - 1) * step < cnt; k += UN * step) {
            int j[UN];
            val_t d[UN];
            uint4 w[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) column(k + u * step, j[u], d[u]);
#pragma unroll
            for (int u = 0; u < UN; ++u) w[u] = *reinterpret_cast<const uint4*>(wcol + j[u] * pitch);
#pragma unroll
            for (int u = 0; u < UN; ++u) fma16(w[u], d[u]);
        }
        {   // the rest of this group's columns (fewer than UN), in flight together
            int j[UN];
            val_t d[UN];
            uint4 w[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                j[u] = 0;
                d[u] = 0;
                if (k + u * step < cnt) column(k + u * step, j[u], d[u]);
            }
#pragma unroll
            for (int u = 0; u < UN; ++u)
                w[u] = k + u * step < cnt ? *reinterpret_cast<const uint4*>(wcol + j[u] * pitch) : uint4{0u, 0u, 0u, 0u};
#pragma unroll
            for (int u = 0; u < UN; ++u) fma16(w[u], d[u]);
        }
    }
    // column groups 1.. hand their sums to group 0 (added in group order: the result does not depend on timing)
    if (kg > 0) {
#pragma unroll
        for (int e = 0; e < PV; e += 4) {
            vec_t o;
            o.x = acc[e]; o.y = acc[e + 1]; o.z = acc[e + 2]; o.w = acc[e + 3];
            red[kg - 1][e >> 2][lane] = o;
        }
    }
    __syncthreads();
    if (kg == 0 && live) {
#pragma unroll
        for (int q = 0; q < FC_KG - 1; ++q)
#pragma unroll
            for (int e = 0; e < PV; e += 4) {
                const vec_t o = red[q][e >> 2][lane];
                acc[e] += o.x; acc[e + 1] += o.y; acc[e + 2] += o.z; acc[e + 3] += o.w;
            }
        // partial sums of this split: scratch [stream][split][c_out_p]
        val_t* part = static_cast<val_t*>(part_v) + ((long long)b * splits + s) * g.c_out_p + co0;
#pragma unroll
        for (int e = 0; e < PV; e += 4) {
            vec_t o;
            o.x = acc[e]; o.y = acc[e + 1]; o.z = acc[e + 2]; o.w = acc[e + 3];
            *reinterpret_cast<vec_t*>(part + e) = o;
        }
    }
}

// Workgroup (block of 512 channels, stream): 128 lanes of 4 channels each, times FC_RG split groups; group
// rg adds the partial rows rg, rg + FC_RG, ... (all loads in flight together), the groups' sums are added
// through LDS in group order, and group 0 applies the result: y += sum (delta), y = bias + sum (dense).
template <int DT, int DENSE>
__global__ __launch_bounds__(FC_RG * 128) void fc_reduce_kernel(const void* __restrict__ part_v,
                                                                const int* __restrict__ count,
                                                                const void* __restrict__ bias_v, void* __restrict__ y_v,
                                                                FcGeom g, int splits) {
    typedef typename std::conditional<DT == RRM_I8_I32, int, float>::type val_t;
    typedef typename std::conditional<DT == RRM_I8_I32, int4, float4>::type vec_t;
    constexpr int PER = FC_MAX_SPLITS / FC_RG;  // partial rows per thread at most
    __shared__ vec_t red[FC_RG - 1][128];
    const int b = blockIdx.y;
    const int lane = threadIdx.x & 127, rg = threadIdx.x >> 7;
    const int co = (blockIdx.x * 128 + lane) * 4;
    const bool live = co < g.c_out_p;  // (c_out_p is a multiple of 4)
    const int cnt = DENSE ? g.c_in : count[b];
    const int s_eff = fc_active_splits(cnt, splits);
    const val_t* part = static_cast<const val_t*>(part_v) + (long long)b * splits * g.c_out_p + (live ? co : 0);
    vec_t v[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int s = rg + i * FC_RG;
        v[i] = (live && s < s_eff) ? *reinterpret_cast<const vec_t*>(part + (long long)s * g.c_out_p) : vec_t{0, 0, 0, 0};
    }
    vec_t sum = v[0];
#pragma unroll
    for (int i = 1; i < PER; ++i) {
        sum.x += v[i].x; sum.y += v[i].y; sum.z += v[i].z; sum.w += v[i].w;
    }
    if (rg > 0) red[rg - 1][lane] = sum;
    __syncthreads();
    if (rg != 0 || !live) return;
#pragma unroll
    for (int q = 0; q < FC_RG - 1; ++q) {
        const vec_t o = red[q][lane];
        sum.x += o.x; sum.y += o.y; sum.z += o.z; sum.w += o.w;
    }
    val_t* y = static_cast<val_t*>(y_v) + (long long)b * g.c_out;
    const val_t* bias = static_cast<const val_t*>(bias_v);
    const val_t r[4] = {sum.x, sum.y, sum.z, sum.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        if (co + k >= g.c_out) break;
        if (DENSE)
            y[co + k] = (bias ? bias[co + k] : (val_t)0) + r[k];
        else if (r[k] != (val_t)0)
            y[co + k] += r[k];
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
    if (splits < 1 || splits > FC_MAX_SPLITS) return hipErrorInvalidValue;
    dim3 grid((unsigned int)g.slices, (unsigned int)splits, (unsigned int)g.n), block(FC_KG * 256);
    dim3 rgrid((unsigned int)((g.c_out_p / 4 + 127) / 128), (unsigned int)g.n), rblock(FC_RG * 128);
    const unsigned char* w = static_cast<const unsigned char*>(wT);
    const unsigned char* xx = static_cast<const unsigned char*>(x);
#define RRM_FC(DTV, DV)                                                                                              \
    do {                                                                                                            \
        hipLaunchKernelGGL((fc_scatter_kernel<DTV, DV>), grid, block, 0, s, w, idx, val, count, xx, part, g, splits); \
        hipLaunchKernelGGL((fc_reduce_kernel<DTV, DV>), rgrid, rblock, 0, s, part, count, bias, y, g, splits);       \
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
