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
// wavefront and MFMA); the activation operand comes from the tile's input window staged in LDS,
// where in delta mode only units whose change-map bit is set are fetched at all.
// Each output element has exactly one owner, so the in-place accumulation needs no atomics and is
// reproducible run to run.
#include "rrm_internal.h"

namespace rrm {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

template <int DT>
struct Acc;
template <>
struct Acc<RRM_I8_I32> {
    typedef v4i type;
};
template <>
struct Acc<RRM_BF16_F32> {
    typedef v4f type;
};

__device__ __forceinline__ v4i mma(const uint4& a, const uint4& b, v4i c) {
    return __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(v4i, a), __builtin_bit_cast(v4i, b), c, 0, 0, 0);
}
__device__ __forceinline__ v4f mma(const uint4& a, const uint4& b, v4f c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0,
                                                   0);
}

template <int DT, int MODE, int WM, int TERMS>
__global__ __launch_bounds__(CONV_THREADS) void conv_tile_kernel(
    const unsigned char* __restrict__ src0, const unsigned char* __restrict__ src1,
    const unsigned long long* __restrict__ bitmap, const unsigned int* __restrict__ tileflag, unsigned int epoch,
    const uint4* __restrict__ wpack, const int* __restrict__ offtab, const void* __restrict__ bias_v,
    void* __restrict__ y_v, ConvGeom g, DevStats* __restrict__ stats) {
    typedef typename Acc<DT>::type acc_t;
    constexpr int ESIZE = DT == RRM_I8_I32 ? 1 : 2;
    extern __shared__ uint4 smem[];
    unsigned char* tile0 = reinterpret_cast<unsigned char*>(smem);
    unsigned char* tile1 = tile0 + g.lds_tile_bytes;
    int* tab = reinterpret_cast<int*>(tile0 + (size_t)TERMS * g.lds_tile_bytes);

    const int tile = blockIdx.x;
    if (MODE == MODE_DELTA) {
        if (tileflag[tile] != epoch) return;  // uniform: nothing in this tile's receptive field changed
        if (blockIdx.y == 0 && threadIdx.x == 0) atomicAdd(&stats->active_tiles, 1ull);
    }
    const int tiles_per_img = g.tiles_y * g.tiles_x;
    const int b = tile / tiles_per_img;
    const int trem = tile - b * tiles_per_img;
    const int ty = trem / g.tiles_x, tx = trem - ty * g.tiles_x;
    const int nbg = (g.ncb + WM - 1) / WM;
    const int grp = blockIdx.y / nbg;
    const int bg = blockIdx.y - grp * nbg;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, kgrp = lane >> 4;
    const int cbw = wave % WM, nset = wave / WM;
    const int cb = bg * WM + cbw;
    const bool has_mma = cb < g.ncb;

    const int iy0 = ty * TILE * g.stride - g.pad, ix0 = tx * TILE * g.stride - g.pad;

    int posbase[WM];
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const int st = nset * WM + i;
        const int py = 4 * (st >> 1) + (j >> 2), px = 4 * (st & 1) + (j & 3);
        posbase[i] = ((py * g.stride) * g.tw_in + px * g.stride) * g.pitch;
    }
    acc_t acc[WM];
#pragma unroll
    for (int i = 0; i < WM; ++i) acc[i] = acc_t{0, 0, 0, 0};

    const int ntab = g.nq * 4;
    const long long img_base = (long long)b * g.h * g.w;

    for (int slab = 0; slab < g.nslab; ++slab) {
        const int sc_eff = min(g.sc, g.chunks - slab * g.sc);
        if (slab) __syncthreads();
        // ---- stage this slab of the input window into LDS --------------------------------------
        const int units = g.th_in * g.tw_in * sc_eff;
        for (int u = tid; u < units; u += CONV_THREADS) {
            const int hp = u / sc_eff, cc = u - hp * sc_eff;
            const int hy = hp / g.tw_in, hx = hp - hy * g.tw_in;
            const int iy = iy0 + hy, ix = ix0 + hx;
            uint4 v0 = make_uint4(0, 0, 0, 0), v1 = make_uint4(0, 0, 0, 0);
            if (iy >= 0 && iy < g.h && ix >= 0 && ix < g.w) {
                const long long ebase = ((img_base + (long long)iy * g.w + ix) * g.c_in) + (long long)grp * g.cg +
                                        (long long)(slab * g.sc + cc) * g.per_vec;
                if (g.fast_stage) {
                    const long long vi = ebase / g.per_vec;
                    bool fetch = true;
                    if (MODE == MODE_DELTA) fetch = (bitmap[vi >> 6] >> (vi & 63)) & 1ull;
                    if (fetch) {
                        v0 = *reinterpret_cast<const uint4*>(src0 + vi * 16);
                        if (TERMS == 2) v1 = *reinterpret_cast<const uint4*>(src1 + vi * 16);
                    }
                } else {
                    unsigned int w0[4] = {0, 0, 0, 0}, w1[4] = {0, 0, 0, 0};
                    const int c0 = (slab * g.sc + cc) * g.per_vec;
                    for (int e = 0; e < g.per_vec; ++e) {
                        if (c0 + e >= g.cg) break;
                        const long long ei = ebase + e;
                        bool fetch = true;
                        if (MODE == MODE_DELTA) {
                            const long long vi = ei / g.per_vec;
                            fetch = (bitmap[vi >> 6] >> (vi & 63)) & 1ull;
                        }
                        if (!fetch) continue;
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
            const uint4* wp = wpack + ((((long long)grp * g.ncb + cb) * g.nslab + slab) * g.nq) * 64 + lane;
            for (int q = 0; q < g.nq; ++q) {
                const uint4 a = wp[(long long)q * 64];
                const int off = tab[4 * q + kgrp];
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
    if (!has_mma) return;

    // ---- epilogue: lane holds 4 consecutive output channels of one position -----------------------
    const int co0 = cb * 16 + 4 * kgrp;  // within the group
    if (co0 >= g.og) return;
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const int st = nset * WM + i;
        const int oy = ty * TILE + 4 * (st >> 1) + (j >> 2), ox = tx * TILE + 4 * (st & 1) + (j & 3);
        if (oy >= g.ho || ox >= g.wo) continue;
        const long long ybase = (((long long)b * g.ho + oy) * g.wo + ox) * g.c_out + (long long)grp * g.og + co0;
        if (DT == RRM_I8_I32) {
            int* y = static_cast<int*>(y_v);
            const int* bias = static_cast<const int*>(bias_v);
            const v4i r = __builtin_bit_cast(v4i, acc[i]);
            if (MODE == MODE_DELTA) {
                if ((r.x | r.y | r.z | r.w) == 0) continue;
                if (g.vec_store && co0 + 3 < g.og) {
                    int4* p = reinterpret_cast<int4*>(y + ybase);
                    int4 o = *p;
                    o.x += r.x; o.y += r.y; o.z += r.z; o.w += r.w;
                    *p = o;
                } else {
                    const int rr[4] = {r.x, r.y, r.z, r.w};
                    for (int k = 0; k < 4 && co0 + k < g.og; ++k) y[ybase + k] += rr[k];
                }
            } else {
                const int rr[4] = {r.x, r.y, r.z, r.w};
                if (g.vec_store && co0 + 3 < g.og) {
                    int4 o;
                    const int bo = grp * g.og + co0;
                    o.x = rr[0] + (bias ? bias[bo] : 0);
                    o.y = rr[1] + (bias ? bias[bo + 1] : 0);
                    o.z = rr[2] + (bias ? bias[bo + 2] : 0);
                    o.w = rr[3] + (bias ? bias[bo + 3] : 0);
                    *reinterpret_cast<int4*>(y + ybase) = o;
                } else {
                    for (int k = 0; k < 4 && co0 + k < g.og; ++k)
                        y[ybase + k] = rr[k] + (bias ? bias[grp * g.og + co0 + k] : 0);
                }
            }
        } else {
            float* y = static_cast<float*>(y_v);
            const float* bias = static_cast<const float*>(bias_v);
            const v4f r = __builtin_bit_cast(v4f, acc[i]);
            if (MODE == MODE_DELTA) {
                if (r.x == 0.f && r.y == 0.f && r.z == 0.f && r.w == 0.f) continue;
                if (g.vec_store && co0 + 3 < g.og) {
                    float4* p = reinterpret_cast<float4*>(y + ybase);
                    float4 o = *p;
                    o.x += r.x; o.y += r.y; o.z += r.z; o.w += r.w;
                    *p = o;
                } else {
                    const float rr[4] = {r.x, r.y, r.z, r.w};
                    for (int k = 0; k < 4 && co0 + k < g.og; ++k) y[ybase + k] += rr[k];
                }
            } else {
                const float rr[4] = {r.x, r.y, r.z, r.w};
                if (g.vec_store && co0 + 3 < g.og) {
                    float4 o;
                    const int bo = grp * g.og + co0;
                    o.x = rr[0] + (bias ? bias[bo] : 0.f);
                    o.y = rr[1] + (bias ? bias[bo + 1] : 0.f);
                    o.z = rr[2] + (bias ? bias[bo + 2] : 0.f);
                    o.w = rr[3] + (bias ? bias[bo + 3] : 0.f);
                    *reinterpret_cast<float4*>(y + ybase) = o;
                } else {
                    for (int k = 0; k < 4 && co0 + k < g.og; ++k)
                        y[ybase + k] = rr[k] + (bias ? bias[grp * g.og + co0 + k] : 0.f);
                }
            }
        }
    }
}

template <int DT, int MODE, int WM, int TERMS>
hipError_t launch_one(const void* src0, const void* src1, const unsigned long long* bitmap,
                      const unsigned int* tileflag, unsigned int epoch, const void* wpack, const int* offtab,
                      const void* bias, void* y, const ConvGeom& g, DevStats* stats, hipStream_t s) {
    const int nbg = (g.ncb + WM - 1) / WM;
    dim3 grid((unsigned int)(g.n * g.tiles_y * g.tiles_x), (unsigned int)(g.groups * nbg));
    const size_t lds = (size_t)TERMS * g.lds_tile_bytes + (size_t)g.nq * 4 * sizeof(int);
    hipLaunchKernelGGL((conv_tile_kernel<DT, MODE, WM, TERMS>), grid, dim3(CONV_THREADS), lds, s,
                       static_cast<const unsigned char*>(src0), static_cast<const unsigned char*>(src1), bitmap,
                       tileflag, epoch, static_cast<const uint4*>(wpack), offtab, bias, y, g, stats);
    return hipGetLastError();
}

template <int DT, int MODE, int TERMS>
hipError_t launch_wm(int wm, const void* src0, const void* src1, const unsigned long long* bitmap,
                     const unsigned int* tileflag, unsigned int epoch, const void* wpack, const int* offtab,
                     const void* bias, void* y, const ConvGeom& g, DevStats* stats, hipStream_t s) {
    switch (wm) {
        case 1: return launch_one<DT, MODE, 1, TERMS>(src0, src1, bitmap, tileflag, epoch, wpack, offtab, bias, y, g, stats, s);
        case 2: return launch_one<DT, MODE, 2, TERMS>(src0, src1, bitmap, tileflag, epoch, wpack, offtab, bias, y, g, stats, s);
        default: return launch_one<DT, MODE, 4, TERMS>(src0, src1, bitmap, tileflag, epoch, wpack, offtab, bias, y, g, stats, s);
    }
}

}  // namespace

hipError_t launch_conv(int dtype, int mode, int wm, int terms, const void* src0, const void* src1,
                       const unsigned long long* bitmap, const unsigned int* tileflag, unsigned int epoch,
                       const void* wpack, const int* offtab, const void* bias, void* y, const ConvGeom& g,
                       DevStats* stats, hipStream_t s) {
    if (dtype == RRM_I8_I32) {
        if (mode == MODE_DELTA)
            return launch_wm<RRM_I8_I32, MODE_DELTA, 1>(wm, src0, src1, bitmap, tileflag, epoch, wpack, offtab, bias, y, g, stats, s);
        return launch_wm<RRM_I8_I32, MODE_DENSE, 1>(wm, src0, src1, bitmap, tileflag, epoch, wpack, offtab, bias, y, g, stats, s);
    }
    if (mode == MODE_DENSE)
        return launch_wm<RRM_BF16_F32, MODE_DENSE, 1>(wm, src0, src1, bitmap, tileflag, epoch, wpack, offtab, bias, y, g, stats, s);
    if (terms == 2)
        return launch_wm<RRM_BF16_F32, MODE_DELTA, 2>(wm, src0, src1, bitmap, tileflag, epoch, wpack, offtab, bias, y, g, stats, s);
    return launch_wm<RRM_BF16_F32, MODE_DELTA, 1>(wm, src0, src1, bitmap, tileflag, epoch, wpack, offtab, bias, y, g, stats, s);
}

}  // namespace rrm
