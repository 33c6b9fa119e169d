// Input-stationary ("scatter") delta convolution in ONE launch per step, for low change densities and for layers
// with too few positions to fill the chip otherwise (int8 -> int32, bf16 -> fp32).
//
// Algorithm 1's inner loop as the sparse engine of Sec. 3.5 walks it: the activations are scanned for non-zero
// entries of the difference, and every such entry multiplies the weights that see it and is summed into the
// outputs it touches.  Here a workgroup owns a block of consecutive input positions (and a share of the output
// channels).  It compares x_t with the stored input for its positions (first statement of the loop), keeps the
// difference in LDS, compacts the changed positions with one ballot, and multiplies them, as the columns of a
// matrix product per filter tap,
//     Z_tap [c_out x changed positions] = W_tap [c_out x c_in] * dI [c_in x changed positions]
// (v_mfma_i32_32x32x32_i8 / v_mfma_f32_32x32x16_bf16; weight fragments straight from memory in per-lane order, each
// used once per workgroup), and adds column p of Z_tap into the stored projection at the output position that sees
// input position p under that tap, with atomic adds: several input positions meet in one output, and integer adds
// commute (bit-exact); fp32 adds are applied in arrival order (within the layer's tolerance, not bit-reproducible).
// The work is exactly proportional to the number of changed input positions (Table 1 / Eq. 6 at position
// granularity), there is no change map, no work list in memory and no second launch.
//
// The stored input is committed by the workgroup's own threads from registers; when several workgroups share a
// position block (output-channel splits) the one that finishes its compare last does it (arrival counter per block,
// rearmed by that workgroup), because the others still read the old values until then.
#include <algorithm>
#include <mutex>
#include <type_traits>

#include "rrm_internal.h"

namespace rrm {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

__device__ __forceinline__ v16i mma(const uint4& a, const uint4& b, v16i c) {
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(v4i, a), __builtin_bit_cast(v4i, b), c, 0, 0, 0);
}
__device__ __forceinline__ v16f mma(const uint4& a, const uint4& b, v16f c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0,
                                                   0);
}

__device__ __forceinline__ float bf16_to_f32(unsigned int h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ unsigned int f32_to_bf16(float f) {  // round to nearest even (finite inputs)
    unsigned int u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

constexpr int ST = 256;  // threads

template <int DT, int TERMS>
__global__ __launch_bounds__(ST) void conv_scatter_kernel(const uint4* __restrict__ x_t, uint4* x_snap,
                                                          const uint4* __restrict__ wsc, void* y_v, ScatGeom g,
                                                          DevStats* __restrict__ stats_base) {
    typedef typename std::conditional<DT == RRM_I8_I32, v16i, v16f>::type acc_t;
    typedef typename std::conditional<DT == RRM_I8_I32, int, float>::type sc_t;
    constexpr int UPT = SCAT_UPT;  // 16-byte units per thread at most
    // LDS: difference planes [TERMS][PB][U] x 16 bytes, then one 16-byte block of zeros
    extern __shared__ uint4 smem[];
    uint4* dl = smem;
    const int plane = g.PB * g.U;  // units per plane
    uint4* zero_unit = dl + TERMS * plane;
    __shared__ unsigned int s_flag[64];
    __shared__ int s_list[64];
    __shared__ int s_cnt;
    __shared__ unsigned int s_prev;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const long long p0 = (long long)blockIdx.x * g.PB;             // first position of the block
    const int npos = (int)min((long long)g.PB, g.npos_total - p0);  // positions in it
    const int nunits = npos * g.U;
    const long long u0 = p0 * g.U;  // first 16-byte unit of the block (positions are contiguous in x)
    DevStats* stats = stats_base + (blockIdx.x & (STAT_SLOTS - 1));
    sc_t* y = static_cast<sc_t*>(y_v);

    if (tid < 64) s_flag[tid] = 0u;
    if (tid == 0) *zero_unit = make_uint4(0, 0, 0, 0);
    __syncthreads();

    // ---- difference with the stored input (Algorithm 1), kept in LDS; new snapshot values in registers -----------
    uint4 keep[UPT];
    unsigned int keep_mask = 0;
    unsigned int nelem = 0, nunit = 0, ntrunc = 0;
    float tsq = 0.f;
#pragma unroll
    for (int i = 0; i < UPT; ++i) {
        const int v = tid + ST * i;
        if (v >= nunits) break;
        const uint4 a = x_t[u0 + v], b = x_snap[u0 + v];
        uint4 d0v = make_uint4(0, 0, 0, 0), d1v = d0v;
        bool changed = ((a.x ^ b.x) | (a.y ^ b.y) | (a.z ^ b.z) | (a.w ^ b.w)) != 0u;
        if (changed) {
            const unsigned int aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
            unsigned int dw[4], lw[4] = {0u, 0u, 0u, 0u}, sw[4] = {a.x, a.y, a.z, a.w};
            if (DT == RRM_I8_I32) {
                const unsigned int H = 0x80808080u;
                unsigned int ovf = 0;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    // byte-wise wrapping subtraction and its signed-overflow mask
                    const unsigned int d = ((aw[k] | H) - (bw[k] & ~H)) ^ ((aw[k] ^ ~bw[k]) & H);
                    ovf |= (aw[k] ^ bw[k]) & (aw[k] ^ d) & H;
                    dw[k] = d;
                    const unsigned int z = aw[k] ^ bw[k];
                    nelem += __popc((((z & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | z) & H);
                }
                if (ovf) atomicOr(&stats->range_error, 1u);
            } else {
                // (truncation threshold, Sec. 3.4 "Improving sparsity": an entry whose difference is below g.eps is
                // neither applied nor committed; eps = 0 is the exact method.)  The difference is formed in fp32 and
                // carried as a bf16 head and a bf16 tail.
                bool any_pass = false;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    unsigned int hi2 = 0, lo2 = 0, sn2 = 0;
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const unsigned int xa = (aw[k] >> (16 * e)) & 0xFFFFu, xb = (bw[k] >> (16 * e)) & 0xFFFFu;
                        const float d = bf16_to_f32(xa) - bf16_to_f32(xb);
                        const bool differ = xa != xb;
                        const bool trunc = differ && fabsf(d) < g.eps;
                        const bool pass = differ && !trunc;
                        any_pass |= pass;
                        nelem += pass ? 1u : 0u;
                        ntrunc += trunc ? 1u : 0u;
                        tsq += trunc ? d * d : 0.f;
                        const unsigned int hi = pass ? f32_to_bf16(d) : 0u;
                        const unsigned int lo = pass && TERMS == 2 ? f32_to_bf16(d - bf16_to_f32(hi)) : 0u;
                        hi2 |= hi << (16 * e);
                        lo2 |= lo << (16 * e);
                        sn2 |= (pass ? xa : xb) << (16 * e);
                    }
                    dw[k] = hi2;
                    lw[k] = lo2;
                    sw[k] = sn2;
                }
                changed = any_pass;
            }
            if (changed) {
                d0v = make_uint4(dw[0], dw[1], dw[2], dw[3]);
                d1v = make_uint4(lw[0], lw[1], lw[2], lw[3]);
                keep[i] = make_uint4(sw[0], sw[1], sw[2], sw[3]);
                keep_mask |= 1u << i;
                ++nunit;
                s_flag[v / g.U] = 1u;  // (every writer stores the same value)
            }
        }
        dl[v] = d0v;
        if (TERMS == 2) dl[plane + v] = d1v;
    }
    __syncthreads();
    // every read of the stored input by this workgroup is done
    const bool shared_block = gridDim.y > 1;
    if (shared_block && tid == 0) s_prev = atomicAdd(&g.arrive[blockIdx.x], 1u);

    // ---- changed positions of the block -> column list (one ballot: a block has at most 64 positions) -----------
    if (wave == 0) {
        const bool f = lane < npos && s_flag[lane] != 0u;
        const unsigned long long m = __ballot(f);
        if (f) s_list[__popcll(m & ((1ull << lane) - 1ull))] = lane;
        if (lane == 0) s_cnt = (int)__popcll(m);
    }
    __syncthreads();
    const int cnt = s_cnt;

    // ---- statistics (one workgroup per position block) --------------------------------------------------------------
    if (blockIdx.y == 0) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            nelem += __shfl_xor(nelem, o);
            nunit += __shfl_xor(nunit, o);
            if (DT == RRM_BF16_F32) {
                ntrunc += __shfl_xor(ntrunc, o);
                tsq += __shfl_xor(tsq, o);
            }
        }
        if (lane == 0) {
            if (nunit) {
                atomicAdd(&stats->changed_elems, (unsigned long long)nelem);
                atomicAdd(&stats->changed_units, (unsigned long long)nunit);
            }
            if (DT == RRM_BF16_F32 && ntrunc) {
                atomicAdd(&stats->truncated_elems, (unsigned long long)ntrunc);
                atomicAdd(&stats->truncated_sumsq, (double)tsq);
            }
        }
        if (tid == 0) {
            if (cnt) atomicAdd(&stats->active_tiles, (unsigned long long)cnt);
            if (blockIdx.x == 0) {  // one launch = one delta step
                atomicAdd(&stats_base->delta_steps, 1ull);
                atomicAdd(&stats_base->total_tiles, (unsigned long long)g.npos_total);
                if (g.touched_all) g.touched_all[0] = 1u;  // this path keeps no flags of what it wrote: "everything"
            }
        }
    }

    // ---- the products: work items (channel block of a group, tap, part of the K range of at most 8 steps).  A
    // workgroup takes items blockIdx.y, + gridDim.y, ... and deals them to its wavefronts; a wavefront has an item's
    // (at most 8) weight fragments in flight together, multiplies, and applies its columns.
    if (cnt > 0) {
        const int n = lane & 31, khalf = lane >> 5;
        const int ntile = (cnt + 31) >> 5;  // 1 or 2
        // this lane's columns: block-local position, stream, image coordinates
        int pl[2], cbs[2], ciy[2], cix[2];
        bool cok[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int ci = t * 32 + n;
            cok[t] = t < ntile && ci < cnt;
            pl[t] = cok[t] ? s_list[ci] : 0;
            const long long P = p0 + pl[t];
            cbs[t] = (int)(P / ((long long)g.h * g.w));
            const int r = (int)(P - (long long)cbs[t] * g.h * g.w);
            ciy[t] = r / g.w;
            cix[t] = r - ciy[t] * g.w;
        }
        const int nitems = g.npair * g.ntaps * g.nkp;
        for (int item = (int)blockIdx.y + wave * (int)gridDim.y; item < nitems; item += (ST / 64) * (int)gridDim.y) {
            const int pt = item / g.nkp, kp = item - pt * g.nkp;
            const int pair = pt / g.ntaps, tap = pt - pair * g.ntaps;
            const int grp = pair / g.ncb, cb = pair - grp * g.ncb;
            const int ky = tap / g.kw, kx = tap - ky * g.kw;
            acc_t acc[2];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[t][r] = 0;
            const int k0 = kp * 8;
            const uint4* wp = wsc + ((size_t)(pair * g.ntaps + tap) * g.nk + k0) * 64 + lane;
            const int ub = grp * g.ug;  // first unit of the group within a position
            uint4 a[8];
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (k0 + k < g.nk) a[k] = wp[(size_t)k * 64];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                if (k0 + k >= g.nk) break;
                const int chunk = 2 * (k0 + k) + khalf;
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    if (t >= ntile) break;
                    const uint4* bp = chunk < g.ug ? dl + (pl[t] * g.U + ub + chunk) : zero_unit;
                    acc[t] = mma(a[k], *bp, acc[t]);
                    if (TERMS == 2) acc[t] = mma(a[k], chunk < g.ug ? bp[plane] : *zero_unit, acc[t]);
                }
            }
            // column p of this tap's product belongs to the output position that sees input position p under the tap
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                if (!cok[t]) continue;
                const int ty = ciy[t] + g.pad - ky, tx = cix[t] + g.pad - kx;
                if (ty < 0 || tx < 0) continue;
                const int oy = ty / g.stride, ox = tx / g.stride;
                if (oy * g.stride != ty || ox * g.stride != tx || oy >= g.ho || ox >= g.wo) continue;
                sc_t* yp = y + ((size_t)((cbs[t] * g.ho + oy) * g.wo + ox)) * g.c_out + grp * g.og + cb * 32;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int c = 8 * (r >> 2) + 4 * khalf + (r & 3);
                    const sc_t v = acc[t][r];
                    if (cb * 32 + c < g.og && v != (sc_t)0) atomicAdd(yp + c, v);
                }
            }
        }
    }

    // ---- commit the stored input (only where a difference was applied) ---------------------------------------------
    if (shared_block) {
        __syncthreads();  // (s_prev is visible to every thread)
        if (s_prev != gridDim.y - 1u) return;
        if (tid == 0) g.arrive[blockIdx.x] = 0u;
    }
#pragma unroll
    for (int i = 0; i < UPT; ++i)
        if (keep_mask & (1u << i)) x_snap[u0 + tid + ST * i] = keep[i];
}

}  // namespace

hipError_t launch_conv_scatter(int dtype, int terms, const void* x_t, void* x_snap, const void* wsc, void* y,
                               const ScatGeom& g, DevStats* stats, hipStream_t s) {
    const long long nblk = (g.npos_total + g.PB - 1) / g.PB;
    dim3 grid((unsigned int)nblk, (unsigned int)g.cs);
    const int t = dtype == RRM_BF16_F32 ? terms : 1;
    const size_t lds = ((size_t)t * g.PB * g.U + 1) * 16;
    const uint4* xt = static_cast<const uint4*>(x_t);
    uint4* xs = static_cast<uint4*>(x_snap);
    const uint4* w = static_cast<const uint4*>(wsc);
    if (lds > 64 * 1024) {
        static std::mutex mu;  // shared by every handle and thread of the process
        static bool granted = false;
        std::lock_guard<std::mutex> lock(mu);
        if (!granted) {
            const int cap = 96 * 1024;
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(conv_scatter_kernel<RRM_I8_I32, 1>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, cap);
            if (e == hipSuccess)
                e = hipFuncSetAttribute(reinterpret_cast<const void*>(conv_scatter_kernel<RRM_BF16_F32, 1>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, cap);
            if (e == hipSuccess)
                e = hipFuncSetAttribute(reinterpret_cast<const void*>(conv_scatter_kernel<RRM_BF16_F32, 2>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, cap);
            if (e != hipSuccess) return e;
            granted = true;
        }
    }
    if (dtype == RRM_I8_I32)
        hipLaunchKernelGGL((conv_scatter_kernel<RRM_I8_I32, 1>), grid, dim3(ST), lds, s, xt, xs, w, y, g, stats);
    else if (t == 2)
        hipLaunchKernelGGL((conv_scatter_kernel<RRM_BF16_F32, 2>), grid, dim3(ST), lds, s, xt, xs, w, y, g, stats);
    else
        hipLaunchKernelGGL((conv_scatter_kernel<RRM_BF16_F32, 1>), grid, dim3(ST), lds, s, xt, xs, w, y, g, stats);
    return hipGetLastError();
}

}  // namespace rrm
