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
// Mapping of the tile kernel (the dense layer, and the delta step of layers whose band does not fit LDS): one
// workgroup = one 8x8 output tile (lane = output position) x 4*CW output channels (wavefront w owns CW of
// them); the filter words of an output channel are wave-uniform and come through scalar loads.  A/B words of
// the tile's input window are staged in LDS once; (slab, tap) pairs in which no lane of the wavefront has a
// flipped bit are skipped.
//
// Mapping of the band kernel (the delta step): one workgroup = a band of output rows of one stream x 4*CW
// output channels.  It stages the band's input window as above, notes which input positions hold a flip, lists
// the output positions whose window sees one (ballot compaction into LDS) and deals that list to the lanes 64
// at a time: a wavefront's lanes are all output positions with work to do, wherever in the band they lie, so
// the work follows the changed positions instead of the 8x8 tiles they fall into.
#include <algorithm>
#include <mutex>

#include "rrm_internal.h"

namespace rrm {

namespace {

constexpr int BAND_THREADS = 512;  // the band kernel's workgroup: eight wavefronts

// t + popcount(v) in one instruction (v_bcnt_u32_b32 adds its second operand; the compiler otherwise counts
// into a fresh register and adds pairs of counts with a third instruction)
__device__ __forceinline__ int popc_acc(unsigned int v, int t) {
    int r;
    asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(r) : "v"(v), "v"(t));
    return r;
}

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
                    t = popc_acc((w.x & bb.x) | (~w.x & a.x), t);
                    t = popc_acc((w.y & bb.y) | (~w.y & a.y), t);
                    t = popc_acc((w.z & bb.z) | (~w.z & a.z), t);
                    t = popc_acc((w.w & bb.w) | (~w.w & a.w), t);
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

// the band kernel's inner part: NP x 64 listed output positions (lane l takes entries first + l, first + 128 + l)
// against the CW output channels of this wavefront; the filter words of a (slab, tap) are loaded once for all NP
template <int CW, int NP, bool WL>
__device__ __forceinline__ void band_items(const unsigned int* A, const unsigned int* B, const unsigned short* list,
                                           int first, int cnt, const uint4* __restrict__ wpack, const uint4* wl, int* y,
                                           const BinGeom& g, int b, int oy0, int grp, int co_w, int lane, int wave) {
    const int ntaps = g.kh * g.kw;
    const long long ob8 = (long long)grp * g.nob8 + co_w / 8;
    const bool vec = (g.c_out & 3) == 0 && (g.og & 3) == 0;
    bool valid[NP];
    int oyl[NP], ox[NP], lbase[NP], popm[NP];
    int tot[NP][CW];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int e = first + p * 128 + lane;
        valid[p] = e < cnt;
        const int q = list[valid[p] ? e : 0];
        oyl[p] = q / g.wo;
        ox[p] = q - oyl[p] * g.wo;
        lbase[p] = ((oyl[p] * g.stride) * g.btw_in + ox[p] * g.stride) * g.pitch;
        popm[p] = 0;
#pragma unroll
        for (int o = 0; o < CW; ++o) tot[p][o] = 0;
    }
    for (int slab = 0; slab < g.nslab; ++slab) {
        for (int tap = 0; tap < ntaps; ++tap) {
            const int ky = tap / g.kw, kx = tap - ky * g.kw;
            const int toff = (ky * g.btw_in + kx) * g.pitch + slab * 4;
            uint4 a[NP], bb[NP];
            unsigned int any = 0;
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                a[p] = *reinterpret_cast<const uint4*>(A + lbase[p] + toff);
                bb[p] = *reinterpret_cast<const uint4*>(B + lbase[p] + toff);
                any |= a[p].x | a[p].y | a[p].z | a[p].w | bb[p].x | bb[p].y | bb[p].z | bb[p].w;
            }
            if (__ballot(any != 0u) == 0ull) continue;  // wave-uniform: nothing flipped under this tap
#pragma unroll
            for (int p = 0; p < NP; ++p)
                popm[p] = popc_acc(a[p].w | bb[p].w, popc_acc(a[p].z | bb[p].z, popc_acc(a[p].y | bb[p].y, popc_acc(a[p].x | bb[p].x, popm[p]))));
#pragma unroll
            for (int o8 = 0; o8 < CW / 8; ++o8) {
                // filter words of eight output channels: from the workgroup's copy in LDS (every lane reads the same
                // address: a broadcast, and plain LDS reads pipeline where scalar loads make the wavefront wait), or
                // through scalar loads
                const uint4* wp = WL ? wl + ((slab * ntaps + tap) * 4 + wave) * CW + o8 * 8
                                     : wpack + (((ob8 + o8) * g.nslab + slab) * ntaps + tap) * 8;
                uint4 wq[8];  // all eight reads in flight before the first is used
#pragma unroll
                for (int o = 0; o < 8; ++o) wq[o] = wp[o];
#pragma unroll
                for (int o = 0; o < 8; ++o) {
                    const uint4 w = wq[o];
#pragma unroll
                    for (int p = 0; p < NP; ++p) {
                        int t = tot[p][o8 * 8 + o];
                        t = popc_acc((w.x & bb[p].x) | (~w.x & a[p].x), t);
                        t = popc_acc((w.y & bb[p].y) | (~w.y & a[p].y), t);
                        t = popc_acc((w.z & bb[p].z) | (~w.z & a[p].z), t);
                        t = popc_acc((w.w & bb[p].w) | (~w.w & a[p].w), t);
                        tot[p][o8 * 8 + o] = t;
                    }
                }
            }
        }
    }
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        if (!valid[p] || popm[p] == 0) continue;
        const long long ybase = (((long long)b * g.ho + oy0 + oyl[p]) * g.wo + ox[p]) * g.c_out + (long long)grp * g.og + co_w;
#pragma unroll
        for (int o4 = 0; o4 < CW / 4; ++o4) {
            const int co = co_w + o4 * 4;
            if (co >= g.og) break;
            int r[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) r[k] = 2 * (popm[p] - 2 * tot[p][o4 * 4 + k]);
            if (vec && co + 3 < g.og) {
                int4* yp = reinterpret_cast<int4*>(y + ybase + o4 * 4);
                int4 o = *yp;
                o.x += r[0]; o.y += r[1]; o.z += r[2]; o.w += r[3];
                *yp = o;
            } else {
                for (int k = 0; k < 4 && co + k < g.og; ++k) y[ybase + o4 * 4 + k] += r[k];
            }
        }
    }
}

// FUSED: the whole step in this one launch.  `xsrc` is the new frame x_t and `flip` the stored input: the flip
// mask is their XOR, formed while the window is staged (no difference kernel, no flip buffer); the change counts
// are taken over the input rows a band owns; and the workgroup of a stream that finishes staging last (arrival
// counter) copies the frame into the stored input, when nobody reads the old one any more, and rearms the counter.
template <int CW, bool FUSED, bool WL>
__global__ __launch_bounds__(BAND_THREADS) void bin_band_kernel(const unsigned int* __restrict__ xsrc,
                                                       const unsigned int* flip, unsigned int* snap,
                                                       unsigned int* arrive,
                                                       const uint4* __restrict__ wpack, int* y, BinGeom g,
                                                       DevStats* __restrict__ stats) {
    extern __shared__ uint4 smem[];
    const int npos = g.bth_in * g.btw_in;
    unsigned int* A = reinterpret_cast<unsigned int*>(smem);
    unsigned int* B = A + npos * g.pitch;
    unsigned char* posany = reinterpret_cast<unsigned char*>(B + npos * g.pitch);     // input position holds a flip
    unsigned short* list = reinterpret_cast<unsigned short*>(posany + ((npos + 15) & ~15));  // active output positions
    // (WL) the workgroup's filter words, [slab][tap][4 * CW channels], behind the list (16-byte aligned)
    uint4* wl = reinterpret_cast<uint4*>(reinterpret_cast<unsigned char*>(list) + (((size_t)g.band_rows * g.wo * 2 + 15) & ~(size_t)15));
    __shared__ unsigned int s_wc[BAND_THREADS / 64], s_prev;

    // grid: x = list split (fastest, so the workgroups that share a band start together), y = channel block,
    // z = stream x band
    const int sb = (int)blockIdx.z, zsplit = (int)blockIdx.x, nsplit = (int)gridDim.x;
    const int b = sb / g.nbands, band = sb - b * g.nbands;
    const int nblk = (g.og + 4 * CW - 1) / (4 * CW);
    const int grp = blockIdx.y / nblk;
    const int blk = blockIdx.y - grp * nblk;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // eight wavefronts: four channel sub-blocks (cwave) times two halves of the list (phalf)
    const int cwave = wave & 3, phalf = wave >> 2;
    const int oy0 = band * g.band_rows;
    const int rows = min(g.band_rows, g.ho - oy0);
    const int iy0 = oy0 * g.stride - g.pad, ix0 = -g.pad;
    const int wg4 = g.nslab * 4;

    for (int i = tid; i < npos; i += BAND_THREADS) posany[i] = 0;
    if (WL) {
        const int nit = g.nslab * g.kh * g.kw;
        for (int i = tid; i < nit * 4 * CW; i += BAND_THREADS) {
            const int it = i / (4 * CW), c = i - it * (4 * CW);
            const int co = blk * 4 * CW + c;  // channel within the group
            uint4 w = make_uint4(0, 0, 0, 0);
            if (co < g.nob8 * 8) w = wpack[(((long long)grp * g.nob8 + co / 8) * nit + it) * 8 + (co & 7)];
            wl[i] = w;
        }
    }
    __syncthreads();
    // (FUSED) input rows whose changes this band counts, by the workgroup of the band's first channel block
    const int own_lo = oy0 * g.stride, own_hi = band == g.nbands - 1 ? g.h : (oy0 + g.band_rows) * g.stride;
    const bool count_here = FUSED && blk == 0 && zsplit == 0;
    unsigned int nbits = 0, nunits = 0;
    // ---- stage A = m & x and B = m & ~x of the band's input window ------------------------------
    if (g.vec4) {
        // four words at a time, both loads issued whatever the mask holds (independent loads, several in flight)
        const int units = npos * g.nslab;
#pragma unroll 4
        for (int u = tid; u < units; u += BAND_THREADS) {
            const int hp = (int)(g.magic_nslab ? __umulhi((unsigned int)u, g.magic_nslab) : (unsigned int)u), sl = u - hp * g.nslab;
            const int hy = (int)(g.magic_btw ? __umulhi((unsigned int)hp, g.magic_btw) : (unsigned int)hp), hx = hp - hy * g.btw_in;
            const int iy = iy0 + hy, ix = ix0 + hx;
            uint4 m = make_uint4(0, 0, 0, 0), xv = make_uint4(0, 0, 0, 0);
            if (iy >= 0 && iy < g.h && ix >= 0 && ix < g.w) {
                const long long wi = (((long long)b * g.h + iy) * g.w + ix) * g.wpp + (long long)grp * g.wg + sl * 4;
                m = *reinterpret_cast<const uint4*>(flip + wi);  // the flip buffer is zero where nothing changed
                xv = *reinterpret_cast<const uint4*>(xsrc + wi);
                if (FUSED) {
                    m = make_uint4(m.x ^ xv.x, m.y ^ xv.y, m.z ^ xv.z, m.w ^ xv.w);
                    if (count_here && iy >= own_lo && iy < own_hi && (m.x | m.y | m.z | m.w)) {
                        nbits += __popc(m.x) + __popc(m.y) + __popc(m.z) + __popc(m.w);
                        ++nunits;
                    }
                }
            }
            if (m.x | m.y | m.z | m.w) posany[hp] = 1;
            *reinterpret_cast<uint4*>(A + hp * g.pitch + sl * 4) = make_uint4(m.x & xv.x, m.y & xv.y, m.z & xv.z, m.w & xv.w);
            *reinterpret_cast<uint4*>(B + hp * g.pitch + sl * 4) = make_uint4(m.x & ~xv.x, m.y & ~xv.y, m.z & ~xv.z, m.w & ~xv.w);
        }
    } else {
        const int units = npos * wg4;
        for (int u = tid; u < units; u += BAND_THREADS) {
            const int hp = (int)(g.magic_wg4 ? __umulhi((unsigned int)u, g.magic_wg4) : (unsigned int)u), wd = u - hp * wg4;
            const int hy = (int)(g.magic_btw ? __umulhi((unsigned int)hp, g.magic_btw) : (unsigned int)hp), hx = hp - hy * g.btw_in;
            const int iy = iy0 + hy, ix = ix0 + hx;
            unsigned int m = 0, xv = 0;
            if (wd < g.wg && iy >= 0 && iy < g.h && ix >= 0 && ix < g.w) {
                const long long wi = (((long long)b * g.h + iy) * g.w + ix) * g.wpp + (long long)grp * g.wg + wd;
                m = flip[wi];  // the flip buffer is zero where nothing changed
                if (m) {
                    xv = xsrc[wi];
                    posany[hp] = 1;
                }
            }
            A[hp * g.pitch + wd] = m & xv;
            B[hp * g.pitch + wd] = m & ~xv;
        }
    }
    __syncthreads();
    if (FUSED) {
        // this workgroup has read the stored input for the last time
        if (tid == 0) s_prev = atomicAdd(&arrive[b], 1u);
        if (count_here) {
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                nbits += __shfl_xor(nbits, o);
                nunits += __shfl_xor(nunits, o);
            }
            if (lane == 0 && nunits) {
                atomicAdd(&stats[sb & (STAT_SLOTS - 1)].changed_elems, (unsigned long long)nbits);
                atomicAdd(&stats[sb & (STAT_SLOTS - 1)].changed_units, (unsigned long long)nunits);
            }
        }
        if (sb == 0 && blockIdx.y == 0 && zsplit == 0 && tid == 0) {  // one launch = one delta step
            atomicAdd(&stats[0].delta_steps, 1ull);
            atomicAdd(&stats[0].total_tiles, (unsigned long long)g.n * g.ho * g.wo);
        }
    }
    // ---- list the output positions of the band whose window holds a flip ------------------------
    const int nout = rows * g.wo;
    int cnt = 0;
    for (int base = 0; base < nout; base += BAND_THREADS) {
        const int q = base + tid;
        bool act = false;
        if (q < nout) {
            const int oyl = q / g.wo, ox = q - oyl * g.wo;
            const unsigned char* pa = posany + (oyl * g.stride) * g.btw_in + ox * g.stride;
            for (int ky = 0; ky < g.kh; ++ky)
                for (int kx = 0; kx < g.kw; ++kx) act |= pa[ky * g.btw_in + kx] != 0;
        }
        // (the same order in every workgroup of the band: the workgroups of a list split deal its chunks among them)
        const unsigned long long mask = __ballot(act);
        if (lane == 0) s_wc[wave] = (unsigned int)__popcll(mask);
        __syncthreads();
        unsigned int wbase = (unsigned int)cnt, all = 0;
#pragma unroll
        for (int w = 0; w < BAND_THREADS / 64; ++w) {
            const unsigned int c = s_wc[w];
            if (w < wave) wbase += c;
            all += c;
        }
        if (act) list[wbase + __popcll(mask & ((1ull << lane) - 1ull))] = (unsigned short)q;
        cnt += (int)all;
        __syncthreads();  // (the counts are overwritten in the next round; after the last one: the list is complete)
    }
    if (cnt > 0 && blockIdx.y == 0 && zsplit == 0 && tid == 0)
        atomicAdd(&stats[sb & (STAT_SLOTS - 1)].active_tiles, (unsigned long long)cnt);

    // The list is dealt in 64-entry chunks: of every four consecutive chunks the first half of the wavefronts takes
    // the even ones and the second half the odd ones (so a list of up to 128 entries is one chunk each, not two
    // for one half), two chunks per pass where a half has two (they share the filter words).
    const int co_w = blk * 4 * CW + cwave * CW;  // first output channel of this wavefront in the group
    if (co_w < g.og) {
        for (int first = zsplit * 256 + phalf * 64; first < cnt; first += nsplit * 256) {
            if (first + 128 < cnt)
                band_items<CW, 2, WL>(A, B, list, first, cnt, wpack, wl, y, g, b, oy0, grp, co_w, lane, cwave);
            else
                band_items<CW, 1, WL>(A, B, list, first, cnt, wpack, wl, y, g, b, oy0, grp, co_w, lane, cwave);
        }
    }
    if (FUSED) {
        // commit: the stream's last workgroup to finish staging (s_prev was published by the list's barriers)
        if (s_prev == (unsigned int)g.nbands * gridDim.y * (unsigned int)nsplit - 1u) {
            const long long words = (long long)g.h * g.w * g.wpp;  // (a multiple of four: whole 16-byte vectors)
            const uint4* src = reinterpret_cast<const uint4*>(xsrc + (long long)b * words);
            uint4* dst = reinterpret_cast<uint4*>(snap + (long long)b * words);
            for (long long i = tid; i < words / 4; i += BAND_THREADS) dst[i] = src[i];
            if (tid == 0) arrive[b] = 0u;
        }
    }
}

template <int MODE, int CW>
hipError_t launch_one(const void* xsrc, const void* flip, unsigned int* tileflag, const void* wpack,
                      const void* bias, void* y, const BinGeom& g, DevStats* stats, hipStream_t s) {
    const int nblk = (g.og + 4 * CW - 1) / (4 * CW);
    dim3 grid((unsigned int)(g.n * g.tiles_y * g.tiles_x), (unsigned int)(g.groups * nblk));
    const size_t lds = (size_t)2 * g.th_in * g.tw_in * g.pitch * sizeof(unsigned int);
    auto kern = bin_conv_kernel<MODE, CW>;
    if (lds > 64 * 1024) {  // (large strided windows; at most BIN_TILE_MAX_LDS, checked at create)
        static std::mutex mu;
        static size_t granted = 0;
        std::lock_guard<std::mutex> lock(mu);
        if (lds > granted) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            granted = lds;
        }
    }
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, static_cast<const unsigned int*>(xsrc),
                       static_cast<const unsigned int*>(flip), tileflag,
                       static_cast<const uint4*>(wpack), static_cast<const int*>(bias), static_cast<int*>(y), g,
                       stats);
    return hipGetLastError();
}

}  // namespace

int bin_consumers(int cw, const BinGeom& g) { return g.groups * ((g.og + 4 * cw - 1) / (4 * cw)); }

template <int CW, bool FUSED, bool WL>
hipError_t launch_band_k(const void* xsrc, const void* flip, void* snap, unsigned int* arrive, const void* wpack, void* y,
                         const BinGeom& g, DevStats* stats, hipStream_t s) {
    const int nblk = (g.og + 4 * CW - 1) / (4 * CW);
    // few streams: deal the band's list over several workgroups (each stages the window again: it is small)
    const long long wgs = (long long)g.n * g.nbands * g.groups * nblk;
    const int chunks = (g.band_rows * g.wo + 255) / 256;  // (a workgroup takes the list 256 entries at a time)
    int z = (int)((2 * NUM_CU + wgs - 1) / wgs);
    z = z < 1 ? 1 : (z > chunks ? chunks : z);
    dim3 grid((unsigned int)z, (unsigned int)(g.groups * nblk), (unsigned int)(g.n * g.nbands));
    const size_t lds = bin_band_lds_bytes(g, g.band_rows);
    auto kern = bin_band_kernel<CW, FUSED, WL>;
    if (lds > 64 * 1024) {
        static std::mutex mu;
        static size_t granted = 0;
        std::lock_guard<std::mutex> lock(mu);
        if (lds > granted) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            granted = lds;
        }
    }
    hipLaunchKernelGGL(kern, grid, dim3(BAND_THREADS), lds, s, static_cast<const unsigned int*>(xsrc),
                       static_cast<const unsigned int*>(flip), static_cast<unsigned int*>(snap), arrive,
                       static_cast<const uint4*>(wpack), static_cast<int*>(y), g, stats);
    return hipGetLastError();
}

template <int CW, bool FUSED>
hipError_t launch_band(const void* xsrc, const void* flip, void* snap, unsigned int* arrive, const void* wpack, void* y,
                       const BinGeom& g, DevStats* stats, hipStream_t s) {
    if (g.wlds) return launch_band_k<CW, FUSED, true>(xsrc, flip, snap, arrive, wpack, y, g, stats, s);
    return launch_band_k<CW, FUSED, false>(xsrc, flip, snap, arrive, wpack, y, g, stats, s);
}

// two launches: xsrc = the stored input after the difference kernel, flip = its flip buffer
hipError_t launch_bin_band(int cw, const void* xsrc, const void* flip, const void* wpack, void* y, const BinGeom& g,
                           DevStats* stats, hipStream_t s) {
    if (g.band_rows < 1 || g.band_rows * g.wo > 65535) return hipErrorInvalidValue;  // (list entries are 16 bits)
    if (cw == 16) return launch_band<16, false>(xsrc, flip, nullptr, nullptr, wpack, y, g, stats, s);
    return launch_band<8, false>(xsrc, flip, nullptr, nullptr, wpack, y, g, stats, s);
}

// one launch: the whole step (needs g.fused_ok: every input position lies in the window of the band that owns it,
// and a group's words per position are whole 16-byte vectors)
hipError_t launch_bin_band_fused(int cw, const void* x_t, void* x_snap, unsigned int* arrive, const void* wpack, void* y,
                                 const BinGeom& g, DevStats* stats, hipStream_t s) {
    if (g.band_rows < 1 || g.band_rows * g.wo > 65535 || !g.fused_ok || !arrive) return hipErrorInvalidValue;
    if (cw == 16) return launch_band<16, true>(x_t, x_snap, x_snap, arrive, wpack, y, g, stats, s);
    return launch_band<8, true>(x_t, x_snap, x_snap, arrive, wpack, y, g, stats, s);
}

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
