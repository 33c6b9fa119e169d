// Binary (XNOR / popcount) convolution for +1/-1 weights and activations bit-packed along channels.
//
// Sec. 4.3 (XNOR-Net paragraph): after the difference of two +1/-1 frames the surviving entries are
// all +2 or -2, so the delta convolution keeps the binary form up to a constant factor.  With
// m = x_t XOR x_{t-1} (the flip mask) and bit 1 = +1, a flipped input contributes w * 2*x_t, i.e.
//      dP = 2 * ( popc(m) - 2 * popc( m & (w XOR x_t) ) )          summed over the window's words.
// The dense layer (Eq. 3) is the same expression with m = "tap inside the image" and factor 1:
//      P  = b + popc(m) - 2 * popc( m & (w XOR x) ).
// Per lane and 32 inputs this is one v_bfi_b32 ((w & B) | (~w & A) with A = m & x, B = m & ~x, which
// equals m & (w XOR x)) and one v_bcnt_u32_b32 with accumulate: plain vector ALU work, no matrix core.
//
// Mapping: one workgroup = one 8x8 output tile (lane = output position) x 4*CW output channels
// (wavefront w owns CW of them); the filter words of an output channel are wave-uniform and come
// through scalar loads.  A/B words of the tile's input window are staged in LDS once; (slab, tap)
// pairs in which no lane of the wavefront has a flipped bit are skipped.
#include "rrm_internal.h"

namespace rrm {

namespace {

template <int MODE, int CW>
__global__ __launch_bounds__(256) void bin_conv_kernel(const unsigned int* __restrict__ xsrc,
                                                       const unsigned int* __restrict__ flip,
                                                       unsigned int* tileflag,
                                                       const uint4* __restrict__ wpack, const int* __restrict__ bias,
                                                       int* y, BinGeom g, DevStats* __restrict__ stats) {
    extern __shared__ uint4 smem[];
    unsigned int* A = reinterpret_cast<unsigned int*>(smem);
    const int npos = g.th_in * g.tw_in;
    unsigned int* B = A + npos * g.pitch;
    __shared__ unsigned int s_flag;

    const int tile = blockIdx.x;
    if (MODE == MODE_DELTA) {
        // the stamp counts the workgroups that still have to consume this tile (see scan.hip)
        if (threadIdx.x == 0) {
            const unsigned int f = tileflag[tile];
            if (f) {
                atomicSub(&tileflag[tile], 1u);
                if (blockIdx.y == 0) atomicAdd(&stats[tile & (STAT_SLOTS - 1)].active_tiles, 1ull);
            }
            s_flag = f;
        }
        __syncthreads();
        if (s_flag == 0) return;
    }
    const int tiles_per_img = g.tiles_y * g.tiles_x;
    const int b = tile / tiles_per_img;
    const int trem = tile - b * tiles_per_img;
    const int ty = trem / g.tiles_x, tx = trem - ty * g.tiles_x;
    const int nblk = (g.og + 4 * CW - 1) / (4 * CW);
    const int grp = blockIdx.y / nblk;
    const int blk = blockIdx.y - grp * nblk;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int iy0 = ty * TILE * g.stride - g.pad, ix0 = tx * TILE * g.stride - g.pad;
    const int wg4 = g.nslab * 4;

    // ---- stage A = m & x and B = m & ~x of the input window -------------------------------------
    const int units = npos * wg4;
    for (int u = tid; u < units; u += 256) {
        const int hp = (int)(g.magic_wg4 ? __umulhi((unsigned int)u, g.magic_wg4) : (unsigned int)u), wd = u - hp * wg4;
        const int hy = (int)(g.magic_tw ? __umulhi((unsigned int)hp, g.magic_tw) : (unsigned int)hp), hx = hp - hy * g.tw_in;
        const int iy = iy0 + hy, ix = ix0 + hx;
        unsigned int m = 0, xv = 0;
        if (wd < g.wg && iy >= 0 && iy < g.h && ix >= 0 && ix < g.w) {
            const long long wi = (((long long)b * g.h + iy) * g.w + ix) * g.wpp + (long long)grp * g.wg + wd;
            m = MODE == MODE_DELTA ? flip[wi] : 0xFFFFFFFFu;  // the flip buffer is zero where nothing changed
            if (m) xv = xsrc[wi];
        }
        A[hp * g.pitch + wd] = m & xv;
        B[hp * g.pitch + wd] = m & ~xv;
    }
    __syncthreads();

    const int py = lane >> 3, px = lane & 7;
    const int lbase = ((py * g.stride) * g.tw_in + px * g.stride) * g.pitch;
    const int co_w = blk * 4 * CW + wave * CW;  // first output channel of this wavefront in the group
    if (co_w >= g.og) return;
    const int ntaps = g.kh * g.kw;
    int tot[CW];
#pragma unroll
    for (int o = 0; o < CW; ++o) tot[o] = 0;
    int popm = 0;
    // filter words: [group][co/8][slab][tap][co%8] uint4, co padded to a multiple of 16 per group
    const long long ob8 = (long long)grp * g.nob8 + co_w / 8;
    for (int slab = 0; slab < g.nslab; ++slab) {
        for (int tap = 0; tap < ntaps; ++tap) {
            const int ky = tap / g.kw, kx = tap - ky * g.kw;
            const int off = lbase + (ky * g.tw_in + kx) * g.pitch + slab * 4;
            const uint4 a = *reinterpret_cast<const uint4*>(A + off);
            const uint4 bb = *reinterpret_cast<const uint4*>(B + off);
            const unsigned int any = a.x | a.y | a.z | a.w | bb.x | bb.y | bb.z | bb.w;
            if (__ballot(any != 0u) == 0ull) continue;  // wave-uniform: nothing flipped under this tap
            popm += __popc(a.x | bb.x) + __popc(a.y | bb.y) + __popc(a.z | bb.z) + __popc(a.w | bb.w);
#pragma unroll
            for (int o8 = 0; o8 < CW / 8; ++o8) {
                const uint4* wp = wpack + (((ob8 + o8) * g.nslab + slab) * ntaps + tap) * 8;
#pragma unroll
                for (int o = 0; o < 8; ++o) {
                    const uint4 w = wp[o];
                    int t = tot[o8 * 8 + o];
                    t += __popc((w.x & bb.x) | (~w.x & a.x));
                    t += __popc((w.y & bb.y) | (~w.y & a.y));
                    t += __popc((w.z & bb.z) | (~w.z & a.z));
                    t += __popc((w.w & bb.w) | (~w.w & a.w));
                    tot[o8 * 8 + o] = t;
                }
            }
        }
    }
    // ---- epilogue ---------------------------------------------------------------------------------
    const int oy = ty * TILE + py, ox = tx * TILE + px;
    if (oy >= g.ho || ox >= g.wo) return;
    if (MODE == MODE_DELTA && popm == 0) return;
    const long long ybase = (((long long)b * g.ho + oy) * g.wo + ox) * g.c_out + (long long)grp * g.og + co_w;
    const bool vec = (g.c_out & 3) == 0 && (g.og & 3) == 0;
#pragma unroll
    for (int o4 = 0; o4 < CW / 4; ++o4) {
        int r[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int v = popm - 2 * tot[o4 * 4 + k];
            r[k] = MODE == MODE_DELTA ? 2 * v : v;
        }
        const int co = co_w + o4 * 4;
        if (co >= g.og) break;
        if (vec && co + 3 < g.og) {
            int4* p = reinterpret_cast<int4*>(y + ybase + o4 * 4);
            int4 o;
            if (MODE == MODE_DELTA) {
                o = *p;
                o.x += r[0]; o.y += r[1]; o.z += r[2]; o.w += r[3];
            } else {
                const int bo = grp * g.og + co;
                o.x = r[0] + (bias ? bias[bo] : 0);
                o.y = r[1] + (bias ? bias[bo + 1] : 0);
                o.z = r[2] + (bias ? bias[bo + 2] : 0);
                o.w = r[3] + (bias ? bias[bo + 3] : 0);
            }
            *p = o;
        } else {
            for (int k = 0; k < 4 && co + k < g.og; ++k) {
                if (MODE == MODE_DELTA)
                    y[ybase + o4 * 4 + k] += r[k];
                else
                    y[ybase + o4 * 4 + k] = r[k] + (bias ? bias[grp * g.og + co + k] : 0);
            }
        }
    }
}

template <int MODE, int CW>
hipError_t launch_one(const void* xsrc, const void* flip, unsigned int* tileflag, const void* wpack,
                      const void* bias, void* y, const BinGeom& g, DevStats* stats, hipStream_t s) {
    const int nblk = (g.og + 4 * CW - 1) / (4 * CW);
    dim3 grid((unsigned int)(g.n * g.tiles_y * g.tiles_x), (unsigned int)(g.groups * nblk));
    const size_t lds = (size_t)2 * g.th_in * g.tw_in * g.pitch * sizeof(unsigned int);
    hipLaunchKernelGGL((bin_conv_kernel<MODE, CW>), grid, dim3(256), lds, s, static_cast<const unsigned int*>(xsrc),
                       static_cast<const unsigned int*>(flip), tileflag,
                       static_cast<const uint4*>(wpack), static_cast<const int*>(bias), static_cast<int*>(y), g,
                       stats);
    return hipGetLastError();
}

}  // namespace

int bin_consumers(int cw, const BinGeom& g) { return g.groups * ((g.og + 4 * cw - 1) / (4 * cw)); }

hipError_t launch_bin_conv(int mode, int cw, const void* xsrc, const void* flip, unsigned int* tileflag,
                           const void* wpack, const void* bias, void* y, const BinGeom& g, DevStats* stats,
                           hipStream_t s) {
    if (mode == MODE_DELTA) {
        if (cw == 16) return launch_one<MODE_DELTA, 16>(xsrc, flip, tileflag, wpack, bias, y, g, stats, s);
        return launch_one<MODE_DELTA, 8>(xsrc, flip, tileflag, wpack, bias, y, g, stats, s);
    }
    if (cw == 16) return launch_one<MODE_DENSE, 16>(xsrc, flip, tileflag, wpack, bias, y, g, stats, s);
    return launch_one<MODE_DENSE, 8>(xsrc, flip, tileflag, wpack, bias, y, g, stats, s);
}

}  // namespace rrm
