// Gather-tile implicit-GEMM convolution on the gfx950 matrix cores (int8 -> int32, bf16 -> fp32).
//
// Delta mode computes the second term of Eq. 5, F * (I_t - I_{t-1}), only on the 8x8 output tiles
// whose receptive field contains a change, and adds it in place into the stored projection
// (Algorithm 1: P_t = P_{t-1} + F * dI).  Dense mode computes Eq. 3, y = b + F * x, on every tile.
//
// GEMM view per workgroup: M = output channels (16 per MFMA row block), N = 64 positions of one
// 8x8 output tile (four 4x4 sub-tiles of 16), K = (tap, 16-byte channel chunk) pairs.  One MFMA
// (v_mfma_i32_16x16x64_i8 / v_mfma_f32_16x16x32_bf16) consumes four K pairs: lane l supplies
// row/column l%16 and the 16 bytes of pair 4q + l/16.  The weight operand comes from a copy of the
// filters packed at create time in exactly that per-lane order (one coalesced 1 KiB read per
// wavefront and MFMA, prefetched PF steps ahead in registers); the activation operand comes from the
// tile's input window staged in LDS.  In delta mode the staged data is the difference buffer, which
// is zero wherever nothing changed.
// Each output element has exactly one owner, so the in-place accumulation needs no atomics and is
// reproducible run to run.
#include "rrm_internal.h"

namespace rrm {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr int PF = 4;  // weight fragments in flight per wavefront; nq is a multiple of PF

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
__device__ __forceinline__ unsigned int fdiv(unsigned int u, unsigned int magic) {
    return magic ? __umulhi(u, magic) : u;
}

template <int DT, int MODE, int WM, int TERMS>
__global__ __launch_bounds__(CONV_THREADS) void conv_tile_kernel(
    const unsigned char* __restrict__ src0, const unsigned char* __restrict__ src1, unsigned int* tileflag,
    const uint4* __restrict__ wpack, const int* __restrict__ offtab, const void* __restrict__ bias_v, void* y_v,
    ConvGeom g, DevStats* __restrict__ stats) {
    typedef typename Acc<DT>::type acc_t;
    typedef typename Acc<DT>::vec vec_t;
    typedef typename Acc<DT>::scalar sc_t;
    constexpr int ESIZE = DT == RRM_I8_I32 ? 1 : 2;
    extern __shared__ uint4 smem[];
    unsigned char* tile0 = reinterpret_cast<unsigned char*>(smem);
    unsigned char* tile1 = tile0 + g.lds_tile_bytes;
    int* tab = reinterpret_cast<int*>(tile0 + (size_t)TERMS * g.lds_tile_bytes);
    __shared__ unsigned int s_flag;

    const int tid = threadIdx.x;
    const int tile = blockIdx.x;
    if (MODE == MODE_DELTA) {
        // The stamp counts the workgroups that still have to consume this tile.  It can only reach
        // zero after every consumer has read it, because each takes its own count off after reading.
        if (tid == 0) {
            const unsigned int f = tileflag[tile];
            if (f) {
                atomicSub(&tileflag[tile], 1u);
                if (blockIdx.y == 0) atomicAdd(&stats[tile & (STAT_SLOTS - 1)].active_tiles, 1ull);
            }
            s_flag = f;
        }
        __syncthreads();
        if (s_flag == 0) return;  // nothing in this tile's receptive field changed
    }
    const int tiles_per_img = g.tiles_y * g.tiles_x;
    const int b = tile / tiles_per_img;
    const int trem = tile - b * tiles_per_img;
    const int ty = trem / g.tiles_x, tx = trem - ty * g.tiles_x;
    const int nbg = (g.ncb + WM - 1) / WM;
    const int grp = blockIdx.y / nbg;
    const int bg = blockIdx.y - grp * nbg;

    const int lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, kgrp = lane >> 4;
    const int cbw = wave % WM, nset = wave / WM;
    const int cb = bg * WM + cbw;
    const bool has_mma = cb < g.ncb;
    const int co0 = cb * 16 + 4 * kgrp;  // first of this lane's 4 output channels, within the group
    const bool vec_ok = g.vec_store && co0 + 3 < g.og;

    const int iy0 = ty * TILE * g.stride - g.pad, ix0 = tx * TILE * g.stride - g.pad;

    int posbase[WM];
    long long ybase[WM];
    bool pos_ok[WM];
    vec_t yold[WM];
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const int st = nset * WM + i;
        const int py = 4 * (st >> 1) + (j >> 2), px = 4 * (st & 1) + (j & 3);
        posbase[i] = ((py * g.stride) * g.tw_in + px * g.stride) * g.pitch;
        const int oy = ty * TILE + py, ox = tx * TILE + px;
        pos_ok[i] = has_mma && oy < g.ho && ox < g.wo && co0 < g.og;
        ybase[i] = (((long long)b * g.ho + oy) * g.wo + ox) * g.c_out + (long long)grp * g.og + co0;
        // the stored projection is fetched now so that its latency overlaps the K loop
        if (MODE == MODE_DELTA && pos_ok[i] && vec_ok)
            yold[i] = *reinterpret_cast<const vec_t*>(static_cast<const sc_t*>(y_v) + ybase[i]);
    }
    acc_t acc[WM];
#pragma unroll
    for (int i = 0; i < WM; ++i) acc[i] = acc_t{0, 0, 0, 0};

    const int ntab = g.nq * 4;
    const long long img_base = (long long)b * g.h * g.w;
    const int ktotal = g.nslab * g.nq;
    const uint4* wp = wpack + (((long long)grp * g.ncb + (has_mma ? cb : 0)) * ktotal) * 64 + lane;
    uint4 abuf[PF];
#pragma unroll
    for (int i = 0; i < PF; ++i) abuf[i] = wp[(long long)min(i, ktotal - 1) * 64];
    int kk = 0;

    for (int slab = 0; slab < g.nslab; ++slab) {
        const bool last = slab == g.nslab - 1;
        const int sc_eff = last ? g.chunks - slab * g.sc : g.sc;
        const unsigned int magic = g.magic_sc[last ? 1 : 0];
        if (slab) __syncthreads();
        // ---- stage this slab of the input window into LDS --------------------------------------
        const int units = g.th_in * g.tw_in * sc_eff;
        for (int u = tid; u < units; u += CONV_THREADS) {
            const int hp = (int)fdiv((unsigned int)u, magic), cc = u - hp * sc_eff;
            const int hy = (int)fdiv((unsigned int)hp, g.magic_tw), hx = hp - hy * g.tw_in;
            const int iy = iy0 + hy, ix = ix0 + hx;
            uint4 v0 = make_uint4(0, 0, 0, 0), v1 = make_uint4(0, 0, 0, 0);
            if (iy >= 0 && iy < g.h && ix >= 0 && ix < g.w) {
                const long long ebase = ((img_base + (long long)iy * g.w + ix) * g.c_in) + (long long)grp * g.cg +
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
                                w1[e >> 1] |= (unsigned int)reinterpret_cast<const unsigned short*>(src1)[ei]
                                              << (16 * (e & 1));
                        }
                    }
                    v0 = make_uint4(w0[0], w0[1], w0[2], w0[3]);
                    v1 = make_uint4(w1[0], w1[1], w1[2], w1[3]);
                }
            }
            *reinterpret_cast<uint4*>(tile0 + hp * g.pitch + cc * 16) = v0;
            if (TERMS == 2) *reinterpret_cast<uint4*>(tile1 + hp * g.pitch + cc * 16) = v1;
        }
        for (int e = tid; e < ntab; e += CONV_THREADS) tab[e] = offtab[slab * ntab + e];
        __syncthreads();
        // ---- K loop over (tap, chunk) pairs of this slab ----------------------------------------
        if (has_mma) {
            for (int q = 0; q < g.nq; q += PF) {
#pragma unroll
                for (int p = 0; p < PF; ++p) {
                    const uint4 a = abuf[p];
                    abuf[p] = wp[(long long)min(kk + PF, ktotal - 1) * 64];  // refill PF steps ahead
                    ++kk;
                    const int off = tab[4 * (q + p) + kgrp];
#pragma unroll
                    for (int i = 0; i < WM; ++i) {
                        const uint4 b0 = *reinterpret_cast<const uint4*>(tile0 + posbase[i] + off);
                        acc[i] = mma(a, b0, acc[i]);
                        if (TERMS == 2) {
                            const uint4 b1 = *reinterpret_cast<const uint4*>(tile1 + posbase[i] + off);
                            acc[i] = mma(a, b1, acc[i]);
                        }
                    }
                }
            }
        }
    }

    // ---- epilogue: lane holds 4 consecutive output channels of one position ----------------------
    sc_t* y = static_cast<sc_t*>(y_v);
    const sc_t* bias = static_cast<const sc_t*>(bias_v);
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        if (!pos_ok[i]) continue;
        const sc_t r[4] = {acc[i][0], acc[i][1], acc[i][2], acc[i][3]};
        if (MODE == MODE_DELTA) {
            if (r[0] == (sc_t)0 && r[1] == (sc_t)0 && r[2] == (sc_t)0 && r[3] == (sc_t)0) continue;
            if (vec_ok) {
                vec_t o = yold[i];
                o.x += r[0]; o.y += r[1]; o.z += r[2]; o.w += r[3];
                *reinterpret_cast<vec_t*>(y + ybase[i]) = o;
            } else {
                for (int k = 0; k < 4 && co0 + k < g.og; ++k) y[ybase[i] + k] += r[k];
            }
        } else {
            const int bo = grp * g.og + co0;
            if (vec_ok) {
                vec_t o;
                o.x = r[0] + (bias ? bias[bo] : (sc_t)0);
                o.y = r[1] + (bias ? bias[bo + 1] : (sc_t)0);
                o.z = r[2] + (bias ? bias[bo + 2] : (sc_t)0);
                o.w = r[3] + (bias ? bias[bo + 3] : (sc_t)0);
                *reinterpret_cast<vec_t*>(y + ybase[i]) = o;
            } else {
                for (int k = 0; k < 4 && co0 + k < g.og; ++k) y[ybase[i] + k] = r[k] + (bias ? bias[bo + k] : (sc_t)0);
            }
        }
    }
}

template <int DT, int MODE, int WM, int TERMS>
hipError_t launch_one(const void* src0, const void* src1, unsigned int* tileflag, const void* wpack,
                      const int* offtab, const void* bias, void* y, const ConvGeom& g, DevStats* stats,
                      hipStream_t s) {
    const int nbg = (g.ncb + WM - 1) / WM;
    dim3 grid((unsigned int)(g.n * g.tiles_y * g.tiles_x), (unsigned int)(g.groups * nbg));
    const size_t lds = (size_t)TERMS * g.lds_tile_bytes + (size_t)g.nq * 4 * sizeof(int);
    hipLaunchKernelGGL((conv_tile_kernel<DT, MODE, WM, TERMS>), grid, dim3(CONV_THREADS), lds, s,
                       static_cast<const unsigned char*>(src0), static_cast<const unsigned char*>(src1), tileflag,
                       static_cast<const uint4*>(wpack), offtab, bias, y, g, stats);
    return hipGetLastError();
}

template <int DT, int MODE, int TERMS>
hipError_t launch_wm(int wm, const void* src0, const void* src1, unsigned int* tileflag, const void* wpack,
                     const int* offtab, const void* bias, void* y, const ConvGeom& g, DevStats* stats,
                     hipStream_t s) {
    switch (wm) {
        case 1: return launch_one<DT, MODE, 1, TERMS>(src0, src1, tileflag, wpack, offtab, bias, y, g, stats, s);
        case 2: return launch_one<DT, MODE, 2, TERMS>(src0, src1, tileflag, wpack, offtab, bias, y, g, stats, s);
        default: return launch_one<DT, MODE, 4, TERMS>(src0, src1, tileflag, wpack, offtab, bias, y, g, stats, s);
    }
}

}  // namespace

int conv_consumers(int wm, const ConvGeom& g) { return g.groups * ((g.ncb + wm - 1) / wm); }

hipError_t launch_conv(int dtype, int mode, int wm, int terms, const void* src0, const void* src1,
                       unsigned int* tileflag, const void* wpack, const int* offtab, const void* bias, void* y,
                       const ConvGeom& g, DevStats* stats, hipStream_t s) {
    if (dtype == RRM_I8_I32) {
        if (mode == MODE_DELTA)
            return launch_wm<RRM_I8_I32, MODE_DELTA, 1>(wm, src0, src1, tileflag, wpack, offtab, bias, y, g, stats, s);
        return launch_wm<RRM_I8_I32, MODE_DENSE, 1>(wm, src0, src1, tileflag, wpack, offtab, bias, y, g, stats, s);
    }
    if (mode == MODE_DENSE)
        return launch_wm<RRM_BF16_F32, MODE_DENSE, 1>(wm, src0, src1, tileflag, wpack, offtab, bias, y, g, stats, s);
    if (terms == 2)
        return launch_wm<RRM_BF16_F32, MODE_DELTA, 2>(wm, src0, src1, tileflag, wpack, offtab, bias, y, g, stats, s);
    return launch_wm<RRM_BF16_F32, MODE_DELTA, 1>(wm, src0, src1, tileflag, wpack, offtab, bias, y, g, stats, s);
}

}  // namespace rrm
