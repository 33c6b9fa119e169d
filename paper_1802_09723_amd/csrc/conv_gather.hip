// Gather-tile implicit-GEMM convolution on the gfx950 matrix cores (int8 -> int32, bf16 -> fp32).
//
// Delta mode computes the second term of Eq. 5, F * (I_t - I_{t-1}), only where it is non-zero, and
// adds it in place into the stored projection (Algorithm 1: P_t = P_{t-1} + F * dI).  Dense mode
// computes Eq. 3, y = b + F * x, everywhere.
//
// Unit of work: a 4x4 block of output positions (a "sub-tile", 16 positions = one MFMA column
// block).  The scan kernel sets one bit per sub-tile whose receptive field contains a changed input.
// Every workgroup of this kernel reads that bit array (a few hundred bytes), ranks the set bits with
// a popcount prefix sum, and takes its share of the ranked list: up to NT active sub-tiles from
// anywhere in the batch.  They become the N dimension of one GEMM per workgroup:
//     M = output channels (WM blocks of 16, one wavefront each)
//     N = 16 x (gathered sub-tiles)
//     K = (filter tap, 16-byte channel chunk) pairs, four per MFMA
//         (v_mfma_i32_16x16x64_i8 / v_mfma_f32_16x16x32_bf16; lane l supplies row/column l%16 and the
//          16 bytes of pair 4q + l/16).
// The weight operand is read from a copy of the filters packed at create time in that per-lane order
// (one coalesced 1 KiB read per wavefront and K step, prefetched PF steps ahead in registers) and is
// reused for all gathered sub-tiles; the activation operand comes from the sub-tiles' input windows
// staged in LDS (slab by slab over the channel chunks, the next slab's loads in flight during the
// current K loop).  In delta mode the staged data is the difference buffer, zero where nothing changed.
// The number of sub-tiles per workgroup adapts on the device: few active sub-tiles are spread one per
// workgroup (latency), many are packed NT per workgroup (weight reuse).
// Every output element has exactly one owner: no atomics on y, results reproducible run to run.
// The last workgroup to finish clears the bit array and the arrival counter, so nothing on the host
// changes between steps (HIP-graph replay safe).
#include "rrm_internal.h"

namespace rrm {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr int PF = 4;        // weight fragments in flight per wavefront; nq is a multiple of PF

template <int DT>
struct Acc;
template <>
struct Acc<RRM_I8_I32> {
    typedef v4i type;
    typedef int4 vec;
    typedef int scalar;
};
template <>
struct Acc<RRM_BF16_F32> {
    typedef v4f type;
    typedef float4 vec;
    typedef float scalar;
};

__device__ __forceinline__ v4i mma(const uint4& a, const uint4& b, v4i c) {
    return __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(v4i, a), __builtin_bit_cast(v4i, b), c, 0, 0, 0);
}
__device__ __forceinline__ v4f mma(const uint4& a, const uint4& b, v4f c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0,
                                                   0);
}

// u / d for small u through a precomputed reciprocal (magic == 0 means d == 1)
__device__ __forceinline__ int fdiv(int u, unsigned int magic) {
    return magic ? (int)__umulhi((unsigned int)u, magic) : u;
}

template <int DT, int MODE, int WM, int NT, int TERMS>
__global__ __launch_bounds__(CONV_THREADS) void conv_gather_kernel(
    const unsigned char* __restrict__ src0, const unsigned char* __restrict__ src1, unsigned int* subbits,
    unsigned int* ctrl, const uint4* __restrict__ wpack, const int* __restrict__ offtab,
    const void* __restrict__ bias_v, void* y_v, ConvGeom g, DevStats* __restrict__ stats) {
    typedef typename Acc<DT>::type acc_t;
    typedef typename Acc<DT>::vec vec_t;
    typedef typename Acc<DT>::scalar sc_t;
    constexpr int ESIZE = DT == RRM_I8_I32 ? 1 : 2;
    constexpr int WN = 4 / WM;      // wavefronts along N
    constexpr int NA = NT / WN;     // accumulators (sub-tiles) per wavefront
    constexpr bool PREFETCH_Y = MODE == MODE_DELTA && NA <= 8;
    constexpr int MAXU = TERMS == 2 ? CONV_MAX_STAGE_UNITS / 2 : CONV_MAX_STAGE_UNITS;  // per thread and slab
    static_assert(NT % WN == 0 && NA >= 1, "bad tile shape");

    extern __shared__ uint4 smem[];
    unsigned char* tile0 = reinterpret_cast<unsigned char*>(smem);
    unsigned char* tile1 = tile0 + (size_t)NT * g.slot_bytes;
    int* tab = reinterpret_cast<int*>(tile0 + (size_t)TERMS * NT * g.slot_bytes);
    __shared__ int s_sub[NT];          // gathered sub-tile ids
    __shared__ int s_scan[CONV_THREADS / WAVE];
    __shared__ int s_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;

    // ---- which sub-tiles does this workgroup own? ----------------------------------------------------
    int count, excl = 0;
    const int wpt = (g.n_words + CONV_THREADS - 1) / CONV_THREADS;  // bit-array words per thread
    const int w_lo = tid * wpt, w_hi = min(w_lo + wpt, g.n_words);
    if (MODE == MODE_DELTA) {
        // popcount prefix sum over the bit array (every workgroup does the same small scan)
        int mine = 0;
        for (int w = w_lo; w < w_hi; ++w) mine += __popc(subbits[w]);
        int incl = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(incl, o);
            if (lane >= o) incl += t;
        }
        if (lane == 63) s_scan[wave] = incl;
        __syncthreads();
        count = s_scan[0] + s_scan[1] + s_scan[2] + s_scan[3];
        excl = incl - mine;
        for (int w = 0; w < wave; ++w) excl += s_scan[w];
    } else {
        count = g.n_sub;
    }
    // few active sub-tiles are spread one per workgroup, many are packed up to NT per workgroup
    int per = (count + (int)gridDim.x - 1) / (int)gridDim.x;
    if (per < 1) per = 1;
    if (per > NT) per = NT;  // cannot bind: gridDim.x * NT >= n_sub >= count
    const int first = (int)blockIdx.x * per;
    int mycount = count - first;
    if (mycount > per) mycount = per;

    if (MODE == MODE_DELTA) {
        if (mycount > 0) {
            // the rank of a set bit is the number of set bits before it; keep ranks first .. first+mycount-1
            int rank = excl;
            for (int w = w_lo; w < w_hi; ++w) {
                unsigned int bits = subbits[w];
                while (bits) {
                    const int bpos = __ffs(bits) - 1;
                    bits &= bits - 1;
                    const int r = rank - first;
                    if (r >= 0 && r < mycount) s_sub[r] = w * 32 + bpos;
                    ++rank;
                }
            }
        }
        // arrival: after this workgroup's last read of the bit array
        __syncthreads();
        if (tid == 0) {
            __threadfence();
            const unsigned int total = gridDim.x * gridDim.y;
            const unsigned int old = atomicAdd(&ctrl[0], 1u);
            s_last = (old == total - 1u) ? 1 : 0;
        }
        __syncthreads();
        if (s_last) {
            // every workgroup has read the bits: clear them for the next step
            for (int w = tid; w < g.n_words; w += CONV_THREADS) subbits[w] = 0u;
            if (tid == 0) {
                ctrl[0] = 0u;
                if (count) atomicAdd(&stats[0].active_tiles, (unsigned long long)count);
            }
        }
        if (mycount <= 0) return;
    } else {
        if (mycount <= 0) return;
        if (tid < mycount) s_sub[tid] = first + tid;
        __syncthreads();
    }

    const int nbg = (g.ncb + WM - 1) / WM;
    const int grp = blockIdx.y / nbg;
    const int bg = blockIdx.y - grp * nbg;
    const int j = lane & 15, kgrp = lane >> 4;
    const int wm_i = wave % WM, wn_i = wave / WM;
    const int cb = bg * WM + wm_i;
    const bool has_mma = cb < g.ncb;
    const int co0 = cb * 16 + 4 * kgrp;  // first of this lane's 4 output channels, within the group
    const bool vec_ok = g.vec_store && co0 + 3 < g.og;
    const int subs_per_img = g.sty * g.stx;

    // lane-constant offset of its output position inside a sub-tile's input window
    const int posbase = (((j >> 2) * g.stride) * g.ww + (j & 3) * g.stride) * g.pitch;

    long long ybase[NA];
    bool ok[NA];
    vec_t yold[PREFETCH_Y ? NA : 1];
    acc_t acc[NA];
#pragma unroll
    for (int a = 0; a < NA; ++a) {
        const int slot = wn_i + a * WN;
        acc[a] = acc_t{0, 0, 0, 0};
        ok[a] = false;
        ybase[a] = 0;
        if (slot < mycount) {
            const int id = s_sub[slot];
            const int b = fdiv(id, g.magic_sub);
            const int r = id - b * subs_per_img;
            const int sy = fdiv(r, g.magic_stx), sx = r - sy * g.stx;
            const int oy = 4 * sy + (j >> 2), ox = 4 * sx + (j & 3);
            ok[a] = has_mma && oy < g.ho && ox < g.wo && co0 < g.og;
            ybase[a] = (((long long)b * g.ho + oy) * g.wo + ox) * g.c_out + (long long)grp * g.og + co0;
            if (PREFETCH_Y && ok[a] && vec_ok)
                yold[PREFETCH_Y ? a : 0] = *reinterpret_cast<const vec_t*>(static_cast<const sc_t*>(y_v) + ybase[a]);
        }
    }

    const int ntab = g.nq * 4;
    const int ktotal = g.nslab * g.nq;
    const uint4* wp = wpack + (((long long)grp * g.ncb + (has_mma ? cb : 0)) * ktotal) * 64 + lane;
    uint4 abuf[PF];
#pragma unroll
    for (int i = 0; i < PF; ++i) abuf[i] = wp[(long long)min(i, ktotal - 1) * 64];
    int kk = 0;

    // ---- staging: global -> registers -> LDS, one slab of channel chunks at a time ---------------------
    uint4 st0[MAXU], st1[TERMS == 2 ? MAXU : 1];
    // value(s) of staged unit u of a slab: 16 bytes of one (sub-tile, window position, chunk)
    auto fetch_unit = [&](int u, int slab, bool last, int sc_eff, int per_slot, uint4& v0, uint4& v1, int& lds_off) {
        const int slot = fdiv(u, g.magic_wsc[last ? 1 : 0]);
        const int r = u - slot * per_slot;
        const int hp = fdiv(r, g.magic_sc[last ? 1 : 0]), cc = r - hp * sc_eff;
        lds_off = slot * g.slot_bytes + hp * g.pitch + cc * 16;
        const int hy = fdiv(hp, g.magic_ww), hx = hp - hy * g.ww;
        const int id = s_sub[slot];
        const int b = fdiv(id, g.magic_sub);
        const int rr = id - b * subs_per_img;
        const int sy = fdiv(rr, g.magic_stx), sx = rr - sy * g.stx;
        const int iy = 4 * sy * g.stride - g.pad + hy, ix = 4 * sx * g.stride - g.pad + hx;
        v0 = make_uint4(0, 0, 0, 0);
        v1 = make_uint4(0, 0, 0, 0);
        if (iy >= 0 && iy < g.h && ix >= 0 && ix < g.w) {
            const long long ebase = ((((long long)b * g.h + iy) * g.w + ix) * g.c_in) + (long long)grp * g.cg +
                                    (long long)(slab * g.sc + cc) * g.per_vec;
            if (g.fast_stage) {
                v0 = *reinterpret_cast<const uint4*>(src0 + ebase * ESIZE);
                if (TERMS == 2) v1 = *reinterpret_cast<const uint4*>(src1 + ebase * ESIZE);
            } else {
                unsigned int w0[4] = {0, 0, 0, 0}, w1[4] = {0, 0, 0, 0};
                const int c0 = (slab * g.sc + cc) * g.per_vec;
                for (int e = 0; e < g.per_vec; ++e) {
                    if (c0 + e >= g.cg) break;
                    const long long ei = ebase + e;
                    if (ESIZE == 1) {
                        w0[e >> 2] |= (unsigned int)src0[ei] << (8 * (e & 3));
                    } else {
                        w0[e >> 1] |= (unsigned int)reinterpret_cast<const unsigned short*>(src0)[ei] << (16 * (e & 1));
                        if (TERMS == 2)
                            w1[e >> 1] |= (unsigned int)reinterpret_cast<const unsigned short*>(src1)[ei] << (16 * (e & 1));
                    }
                }
                v0 = make_uint4(w0[0], w0[1], w0[2], w0[3]);
                v1 = make_uint4(w1[0], w1[1], w1[2], w1[3]);
            }
        }
    };
    // Register-buffered staging (loads of the next slab overlap the current K loop) when a slab is at
    // most MAXU units per thread; otherwise global -> LDS directly at store time.
    const bool reg_stage = (long long)NT * g.wpos * g.sc <= (long long)MAXU * CONV_THREADS;
    auto stage_load = [&](int slab) {
        if (!reg_stage) return;
        const bool last = slab == g.nslab - 1;
        const int sc_eff = last ? g.chunks - slab * g.sc : g.sc;
        const int per_slot = g.wpos * sc_eff;
        const int units = mycount * per_slot;
#pragma unroll
        for (int i = 0; i < MAXU; ++i) {
            const int u = tid + i * CONV_THREADS;
            uint4 v0 = make_uint4(0, 0, 0, 0), v1 = make_uint4(0, 0, 0, 0);
            int o;
            if (u < units) fetch_unit(u, slab, last, sc_eff, per_slot, v0, v1, o);
            st0[i] = v0;
            if (TERMS == 2) st1[i] = v1;
        }
    };
    auto stage_store = [&](int slab) {
        const bool last = slab == g.nslab - 1;
        const int sc_eff = last ? g.chunks - slab * g.sc : g.sc;
        const int per_slot = g.wpos * sc_eff;
        const int units = mycount * per_slot;
        if (reg_stage) {
#pragma unroll
            for (int i = 0; i < MAXU; ++i) {
                const int u = tid + i * CONV_THREADS;
                if (u < units) {
                    const int slot = fdiv(u, g.magic_wsc[last ? 1 : 0]);
                    const int r = u - slot * per_slot;
                    const int hp = fdiv(r, g.magic_sc[last ? 1 : 0]), cc = r - hp * sc_eff;
                    const int o = slot * g.slot_bytes + hp * g.pitch + cc * 16;
                    *reinterpret_cast<uint4*>(tile0 + o) = st0[i];
                    if (TERMS == 2) *reinterpret_cast<uint4*>(tile1 + o) = st1[i];
                }
            }
        } else {
            for (int u = tid; u < units; u += CONV_THREADS) {
                uint4 v0, v1;
                int o;
                fetch_unit(u, slab, last, sc_eff, per_slot, v0, v1, o);
                *reinterpret_cast<uint4*>(tile0 + o) = v0;
                if (TERMS == 2) *reinterpret_cast<uint4*>(tile1 + o) = v1;
            }
        }
        for (int e = tid; e < ntab; e += CONV_THREADS) tab[e] = offtab[slab * ntab + e];
    };

    stage_load(0);
    for (int slab = 0; slab < g.nslab; ++slab) {
        if (slab) __syncthreads();  // everyone is done reading the previous slab
        stage_store(slab);
        __syncthreads();
        if (slab + 1 < g.nslab) stage_load(slab + 1);  // in flight during this slab's K loop
        if (has_mma) {
            for (int q = 0; q < g.nq; q += PF) {
#pragma unroll
                for (int p = 0; p < PF; ++p) {
                    const uint4 a = abuf[p];
                    abuf[p] = wp[(long long)min(kk + PF, ktotal - 1) * 64];  // refill PF steps ahead
                    ++kk;
                    const int off = tab[4 * (q + p) + kgrp] + posbase;
#pragma unroll
                    for (int s = 0; s < NA; ++s) {
                        const int slot = wn_i + s * WN;
                        if (slot < mycount) {  // wave-uniform
                            const uint4 b0 = *reinterpret_cast<const uint4*>(tile0 + slot * g.slot_bytes + off);
                            acc[s] = mma(a, b0, acc[s]);
                            if (TERMS == 2) {
                                const uint4 b1 = *reinterpret_cast<const uint4*>(tile1 + slot * g.slot_bytes + off);
                                acc[s] = mma(a, b1, acc[s]);
                            }
                        }
                    }
                }
            }
        }
    }

    // ---- epilogue: lane holds 4 consecutive output channels of one position ----------------------------
    sc_t* y = static_cast<sc_t*>(y_v);
    const sc_t* bias = static_cast<const sc_t*>(bias_v);
#pragma unroll
    for (int a = 0; a < NA; ++a) {
        if (!ok[a]) continue;
        const sc_t r[4] = {acc[a][0], acc[a][1], acc[a][2], acc[a][3]};
        if (MODE == MODE_DELTA) {
            if (r[0] == (sc_t)0 && r[1] == (sc_t)0 && r[2] == (sc_t)0 && r[3] == (sc_t)0) continue;
            if (vec_ok) {
                vec_t o;
                if (PREFETCH_Y)
                    o = yold[PREFETCH_Y ? a : 0];
                else
                    o = *reinterpret_cast<const vec_t*>(y + ybase[a]);
                o.x += r[0]; o.y += r[1]; o.z += r[2]; o.w += r[3];
                *reinterpret_cast<vec_t*>(y + ybase[a]) = o;
            } else {
                for (int k = 0; k < 4 && co0 + k < g.og; ++k) y[ybase[a] + k] += r[k];
            }
        } else {
            const int bo = grp * g.og + co0;
            if (vec_ok) {
                vec_t o;
                o.x = r[0] + (bias ? bias[bo] : (sc_t)0);
                o.y = r[1] + (bias ? bias[bo + 1] : (sc_t)0);
                o.z = r[2] + (bias ? bias[bo + 2] : (sc_t)0);
                o.w = r[3] + (bias ? bias[bo + 3] : (sc_t)0);
                *reinterpret_cast<vec_t*>(y + ybase[a]) = o;
            } else {
                for (int k = 0; k < 4 && co0 + k < g.og; ++k) y[ybase[a] + k] = r[k] + (bias ? bias[bo + k] : (sc_t)0);
            }
        }
    }
}

template <int DT, int MODE, int WM, int NT, int TERMS>
hipError_t launch_one(const void* src0, const void* src1, unsigned int* subbits, unsigned int* ctrl,
                      const void* wpack, const int* offtab, const void* bias, void* y, const ConvGeom& g,
                      DevStats* stats, hipStream_t s) {
    const int nbg = (g.ncb + WM - 1) / WM;
    dim3 grid((unsigned int)((g.n_sub + NT - 1) / NT), (unsigned int)(g.groups * nbg));
    const size_t lds = (size_t)TERMS * NT * g.slot_bytes + (size_t)g.nq * 4 * sizeof(int);
    hipLaunchKernelGGL((conv_gather_kernel<DT, MODE, WM, NT, TERMS>), grid, dim3(CONV_THREADS), lds, s,
                       static_cast<const unsigned char*>(src0), static_cast<const unsigned char*>(src1), subbits,
                       ctrl, static_cast<const uint4*>(wpack), offtab, bias, y, g, stats);
    return hipGetLastError();
}

template <int DT, int MODE, int TERMS>
hipError_t launch_shape(int wm, int nt, const void* src0, const void* src1, unsigned int* subbits,
                        unsigned int* ctrl, const void* wpack, const int* offtab, const void* bias, void* y,
                        const ConvGeom& g, DevStats* stats, hipStream_t s) {
#define RRM_CASE(WMV, NTV)                                                                                          \
    if (wm == WMV && nt == NTV)                                                                                      \
        return launch_one<DT, MODE, WMV, NTV, TERMS>(src0, src1, subbits, ctrl, wpack, offtab, bias, y, g, stats, s);
    RRM_CASE(4, 1) RRM_CASE(4, 2) RRM_CASE(4, 4) RRM_CASE(4, 8) RRM_CASE(4, 16) RRM_CASE(1, 4) RRM_CASE(1, 8) RRM_CASE(1, 16)
#undef RRM_CASE
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_conv(int dtype, int mode, int wm, int nt, int terms, const void* src0, const void* src1,
                       unsigned int* subbits, unsigned int* ctrl, const void* wpack, const int* offtab,
                       const void* bias, void* y, const ConvGeom& g, DevStats* stats, hipStream_t s) {
    if (dtype == RRM_I8_I32) {
        if (mode == MODE_DELTA)
            return launch_shape<RRM_I8_I32, MODE_DELTA, 1>(wm, nt, src0, src1, subbits, ctrl, wpack, offtab, bias, y, g, stats, s);
        return launch_shape<RRM_I8_I32, MODE_DENSE, 1>(wm, nt, src0, src1, subbits, ctrl, wpack, offtab, bias, y, g, stats, s);
    }
    if (mode == MODE_DENSE)
        return launch_shape<RRM_BF16_F32, MODE_DENSE, 1>(wm, nt, src0, src1, subbits, ctrl, wpack, offtab, bias, y, g, stats, s);
    if (terms == 2)
        return launch_shape<RRM_BF16_F32, MODE_DELTA, 2>(wm, nt, src0, src1, subbits, ctrl, wpack, offtab, bias, y, g, stats, s);
    return launch_shape<RRM_BF16_F32, MODE_DELTA, 1>(wm, nt, src0, src1, subbits, ctrl, wpack, offtab, bias, y, g, stats, s);
}

}  // namespace rrm
