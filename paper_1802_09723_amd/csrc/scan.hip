// Fused delta + change-map kernel for convolution layers (int8, bf16, binary).
//
// Algorithm 1, first statement of the inner loop: the difference of this frame's input with the
// stored input.  The GPU form of "skip the zero elements" (Sec. 3.1, Sec. 3.5: the engine scans
// the activation vector for its non-zero entries) is a change map: x is scanned once as a flat
// array of 16-byte units; each wavefront turns its 64 compare results into one 64-bit mask
// (ballot), which is the bitmap word of those units; changed units write their difference, are
// committed to the snapshot, and mark the output blocks whose receptive field contains them: one byte
// flag per 4x4 output sub-tile for the MFMA path (the gather kernel ranks these flags into its work
// list), one stamp per 8x8 output tile for the binary path.
//
// The difference buffer keeps the invariant "zero wherever the bitmap bit is clear": a unit that
// changed in the previous step but not in this one is written back to zero, so the tile kernel can
// stage its input window with plain loads.  A stamped 8x8 tile holds the number of workgroups that
// will consume it; each consumer takes one off, so the stamps are all zero again after the binary
// kernel; the sub-tile flags are cleared by the gather kernel's last workgroup.  Nothing on the host
// has to change between steps (graph replay safe).
//
// HBM traffic per step: 2|x| read, plus (difference + snapshot) written only where x changed.
#include "rrm_internal.h"

namespace rrm {

namespace {

__device__ __forceinline__ float bf16_to_f32(unsigned int h) { return __uint_as_float(h << 16); }

// round-to-nearest-even float -> bf16 pattern (finite inputs)
__device__ __forceinline__ unsigned int f32_to_bf16(float f) {
    unsigned int u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// floor(u / d) for u < 2^31 through the reciprocal rd = 1.0 / d: (u + 0.5) / d is at least 0.5 / d away
// from an integer, far more than the rounding error of the product, so the truncation is exact.
__device__ __forceinline__ unsigned int udiv_big(unsigned int u, double rd) {
    return (unsigned int)(((double)u + 0.5) * rd);
}
// floor(u / d) for u * d < 2^32 through magic = floor(2^32 / d) + 1 (0 encodes d == 1)
__device__ __forceinline__ int udiv_small(int u, unsigned int magic) {
    return magic ? (int)__umulhi((unsigned int)u, magic) : u;
}

__device__ __forceinline__ uint4 load_x_guarded(const unsigned char* x, long long off, long long total_bytes) {
    if (off + 16 <= total_bytes) return *reinterpret_cast<const uint4*>(x + off);
    unsigned int w[4] = {0u, 0u, 0u, 0u};
    for (int i = 0; i < 16; ++i)
        if (off + i < total_bytes) w[i >> 2] |= (unsigned int)x[off + i] << (8 * (i & 3));
    return make_uint4(w[0], w[1], w[2], w[3]);
}

__device__ __forceinline__ void mark_tiles(const ScanGeom& g, int pos, unsigned int* tileflag,
                                           unsigned int stamp) {
    const int hw = g.h * g.w;
    const int b = (int)udiv_big((unsigned int)pos, g.r_hw);
    const int r = pos - b * hw;
    const int iy = (int)udiv_big((unsigned int)r, g.r_w), ix = r - iy * g.w;
    const int ty0 = iy + g.pad - (g.kh - 1), tx0 = ix + g.pad - (g.kw - 1);
    const int oy_lo = ty0 <= 0 ? 0 : udiv_small(ty0 + g.stride - 1, g.magic_stride);
    const int ox_lo = tx0 <= 0 ? 0 : udiv_small(tx0 + g.stride - 1, g.magic_stride);
    int oy_hi = udiv_small(iy + g.pad, g.magic_stride), ox_hi = udiv_small(ix + g.pad, g.magic_stride);
    if (oy_hi > g.ho - 1) oy_hi = g.ho - 1;
    if (ox_hi > g.wo - 1) ox_hi = g.wo - 1;
    if (oy_lo > oy_hi || ox_lo > ox_hi) return;
    for (int ty = oy_lo / TILE; ty <= oy_hi / TILE; ++ty)
        for (int tx = ox_lo / TILE; tx <= ox_hi / TILE; ++tx)
            tileflag[(b * g.tiles_y + ty) * g.tiles_x + tx] = stamp;
}

// Mark the 4x4 output sub-tiles that see input position `pos`: one byte flag each, plain stores
// (every writer stores the same value, so no atomics and no same-address serialisation).
__device__ __forceinline__ void mark_subtiles(const ScanGeom& g, unsigned int pos, unsigned char* flags) {
    const unsigned int hw = (unsigned int)(g.h * g.w);
    const int b = (int)udiv_big(pos, g.r_hw);
    const int r = (int)(pos - (unsigned int)b * hw);
    const int iy = (int)udiv_big((unsigned int)r, g.r_w), ix = r - iy * g.w;
    const int ty0 = iy + g.pad - (g.kh - 1), tx0 = ix + g.pad - (g.kw - 1);
    const int oy_lo = ty0 <= 0 ? 0 : udiv_small(ty0 + g.stride - 1, g.magic_stride);
    const int ox_lo = tx0 <= 0 ? 0 : udiv_small(tx0 + g.stride - 1, g.magic_stride);
    int oy_hi = udiv_small(iy + g.pad, g.magic_stride), ox_hi = udiv_small(ix + g.pad, g.magic_stride);
    if (oy_hi > g.ho - 1) oy_hi = g.ho - 1;
    if (ox_hi > g.wo - 1) ox_hi = g.wo - 1;
    if (oy_lo > oy_hi || ox_lo > ox_hi) return;
    for (int sy = oy_lo >> 2; sy <= (oy_hi >> 2); ++sy)
        for (int sx = ox_lo >> 2; sx <= (ox_hi >> 2); ++sx) flags[(b * g.sty + sy) * g.stx + sx] = 1;
}

// Element index of x element e in the padded / folded difference layout (see ScanGeom).
// (tensors are below 2^30 elements, so 32-bit arithmetic is exact)
__device__ __forceinline__ unsigned int scatter_index(const ScanGeom& g, unsigned int e) {
    const unsigned int p = e / (unsigned int)g.c;
    const unsigned int c = e - p * (unsigned int)g.c;
    const unsigned int r = p / (unsigned int)g.w;
    const unsigned int ix = p - r * (unsigned int)g.w;
    const unsigned int grp = c / (unsigned int)g.cg;
    return ((r * g.wp + ix) * g.groups + grp) * g.cp + (c - grp * g.cg);
}

// Write the 16 bytes of unit v (already computed difference words) element by element into the
// padded / folded layout.  The (row, column, channel) of the first element is divided out once and
// then stepped.
template <int DT>
__device__ __forceinline__ void scatter_unit(const ScanGeom& g, long long v, uint4 w0, uint4 w1, uint4* d0, uint4* d1) {
    constexpr int PV = DT == RRM_I8_I32 ? 16 : 8;
    const unsigned int e0 = (unsigned int)v * PV;
    const unsigned int total = (unsigned int)g.total_elems;
    const unsigned int p = udiv_big(e0, g.r_c);
    int c = (int)(e0 - p * (unsigned int)g.c);
    const unsigned int r0 = udiv_big(p, g.r_w);
    int ix = (int)(p - r0 * (unsigned int)g.w);
    unsigned int rowbase = r0 * (unsigned int)g.wp;
    if (DT == RRM_I8_I32 && g.groups == 1 && g.cp == 4) {
        // Few int8 channels padded to one 32-bit word per position (e.g. RGB -> RGBX): a position that lies
        // wholly inside the unit is one word store (its pad byte is zero anyway); the cut positions at the
        // unit's ends go byte by byte.
        const unsigned long long lo = (unsigned long long)w0.x | (unsigned long long)w0.y << 32;
        const unsigned long long hi = (unsigned long long)w0.z | (unsigned long long)w0.w << 32;
        const unsigned int keep = g.c >= 4 ? 0xFFFFFFFFu : (1u << (8 * g.c)) - 1u;
        unsigned int* dw = reinterpret_cast<unsigned int*>(d0);
        unsigned char* db = reinterpret_cast<unsigned char*>(d0);
        int k = 0;
        while (k < 16 && e0 + (unsigned int)k < total) {
            // the four bytes of the unit starting at byte k (zeros beyond its end)
            const unsigned int four = k < 8 ? (unsigned int)(lo >> (8 * k)) | (k ? (unsigned int)(hi << (64 - 8 * k)) : 0u)
                                            : (unsigned int)(hi >> (8 * (k - 8)));
            if (c == 0 && k + g.c <= 16 && e0 + (unsigned int)(k + g.c) <= total) {
                dw[rowbase + ix] = four & keep;
                k += g.c;
                c = g.c;
            } else {
                db[(rowbase + ix) * 4u + (unsigned int)c] = (unsigned char)four;
                ++k;
                ++c;
            }
            if (c == g.c) {
                c = 0;
                if (++ix == g.w) {
                    ix = 0;
                    rowbase += (unsigned int)g.wp;
                }
            }
        }
        return;
    }
#pragma unroll
    for (int k = 0; k < PV; ++k) {
        if (e0 + k >= total) break;
        const int grp = g.groups == 1 ? 0 : c / g.cg;
        const unsigned int dst = ((rowbase + ix) * g.groups + grp) * g.cp + (c - grp * g.cg);
        if (DT == RRM_I8_I32) {
            const unsigned int word = k < 4 ? w0.x : (k < 8 ? w0.y : (k < 12 ? w0.z : w0.w));
            reinterpret_cast<unsigned char*>(d0)[dst] = (unsigned char)(word >> (8 * (k & 3)));
        } else if (DT == RRM_BF16_F32) {
            const unsigned int a = k < 2 ? w0.x : (k < 4 ? w0.y : (k < 6 ? w0.z : w0.w));
            const unsigned int b = k < 2 ? w1.x : (k < 4 ? w1.y : (k < 6 ? w1.z : w1.w));
            reinterpret_cast<unsigned short*>(d0)[dst] = (unsigned short)(a >> (16 * (k & 1)));
            reinterpret_cast<unsigned short*>(d1)[dst] = (unsigned short)(b >> (16 * (k & 1)));
        }
        if (++c == g.c) {
            c = 0;
            if (++ix == g.w) {
                ix = 0;
                rowbase += (unsigned int)g.wp;
            }
        }
    }
}

template <int ESIZE>
__global__ void repack_kernel(const unsigned char* __restrict__ x, unsigned char* __restrict__ dst, ScanGeom g) {
    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= g.total_elems) return;
    const unsigned int d = scatter_index(g, (unsigned int)e);
    if (ESIZE == 1)
        dst[d] = x[e];
    else
        reinterpret_cast<unsigned short*>(dst)[d] = reinterpret_cast<const unsigned short*>(x)[e];
}

// The same re-layout for few int8 channels padded to one 32-bit word per position (e.g. RGB -> RGBX): one
// thread per position, one word store.
__global__ void repack_word_kernel(const unsigned char* __restrict__ x, unsigned int* __restrict__ dst, ScanGeom g,
                                   unsigned int n_pos) {
    const unsigned int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n_pos) return;
    const unsigned int r = udiv_big(p, g.r_w), ix = p - r * (unsigned int)g.w;
    const unsigned char* src = x + (size_t)p * (unsigned int)g.c;
    unsigned int word = 0;
    for (int c = 0; c < g.c; ++c) word |= (unsigned int)src[c] << (8 * c);
    dst[r * (unsigned int)g.wp + ix] = word;
}

// FUSED: the unit's input is computed from the producer's projection (see FusedSrc); a unit none of whose
// source blocks was written by the producer's last step cannot have changed and is not even loaded.
template <int DT, bool SCATTER, bool FUSED, bool POOL>
__device__ __forceinline__ void scan_body(const unsigned char* __restrict__ x_t, uint4* __restrict__ x_snap,
                                          uint4* __restrict__ d0, uint4* __restrict__ d1,
                                          unsigned long long* __restrict__ bitmap, unsigned int* __restrict__ tileflag,
                                          unsigned int stamp, const ScanGeom& g, long long nvec, long long total_bytes,
                                          DevStats* __restrict__ stats_base, const FusedSrc& fs) {
    // FUSED: neighbouring workgroups read overlapping rows of the producer's projection (pooling windows), and
    // consecutive workgroup ids go to different XCDs, each with an L2 of its own: the grid is a multiple of 8
    // and workgroup id i works on block (i % 8) * (grid / 8) + i / 8, so that an XCD gets a contiguous range.
    const unsigned int blk = FUSED ? (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3) : blockIdx.x;
    const long long v = (long long)blk * blockDim.x + threadIdx.x;
    DevStats* __restrict__ stats = stats_base + (blockIdx.x & (STAT_SLOTS - 1));
    const unsigned long long prev_mask = v < nvec ? bitmap[v >> 6] : 0ull;  // wave-uniform word
    bool changed = false;
    int p0 = 0, p1 = -1;  // input positions of this unit, when it changed
    unsigned int nelem = 0, ntrunc = 0;
    float tsq = 0.f;  // truncated entries of this unit: count and sum of squares (bf16 with a threshold)
    uint4 a = make_uint4(0, 0, 0, 0);
    bool compare = v < nvec;
    uint4 b_early = make_uint4(0, 0, 0, 0);
    if (FUSED && compare) {
        // (c_in is a multiple of 16: the unit is 16 channels of one position)
        const unsigned int e0 = (unsigned int)v * 16u;
        const unsigned int p = udiv_big(e0, g.r_c), c0 = e0 - p * (unsigned int)g.c;
        const unsigned int bb = udiv_big(p, g.r_hw), r = p - bb * (unsigned int)(g.h * g.w);
        const int iy = (int)udiv_big(r, g.r_w), ix = (int)r - iy * g.w;
        // (POOL is a template parameter: the unpooled form keeps no window in registers and runs at twice the
        // occupancy)
        constexpr int span = POOL ? 2 : 0;
        const int y0 = POOL ? 2 * iy : iy, x0 = POOL ? 2 * ix : ix;
        const unsigned char* t = fs.touched + (size_t)bb * fs.sty * fs.stx;
        const int sy0 = y0 >> fs.tshift, sy1 = (y0 + span) >> fs.tshift, sx0 = x0 >> fs.tshift, sx1 = (x0 + span) >> fs.tshift;
        unsigned int any = 0;
        for (int sy = sy0; sy <= sy1; ++sy)
            for (int sx = sx0; sx <= sx1; ++sx) any |= t[sy * fs.stx + sx];
        compare = fs.fresh[0] != 0u || fs.touched_all[0] != 0u || any != 0u;
        if (compare) {
            b_early = x_snap[v];  // in flight together with the window's loads
            int best[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) best[k] = 0;
            const int4* yb = reinterpret_cast<const int4*>(fs.y + (((size_t)bb * fs.hy + y0) * fs.wy + x0) * g.c + c0);
            const size_t c4 = (size_t)g.c / 4;
            // a row of the window at a time: its (up to) 12 loads are in flight together
#pragma unroll
            for (int dy = 0; dy < 3; ++dy) {
                if (dy > span) break;
                int4 w[3][4];
#pragma unroll
                for (int dx = 0; dx < 3; ++dx)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        w[dx][q] = dx <= span ? yb[(size_t)(dy * fs.wy + dx) * c4 + q] : make_int4(0, 0, 0, 0);
#pragma unroll
                for (int dx = 0; dx < 3; ++dx)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        best[4 * q + 0] = max(best[4 * q + 0], w[dx][q].x);
                        best[4 * q + 1] = max(best[4 * q + 1], w[dx][q].y);
                        best[4 * q + 2] = max(best[4 * q + 2], w[dx][q].z);
                        best[4 * q + 3] = max(best[4 * q + 3], w[dx][q].w);
                    }
            }
            // max commutes with the monotone map v -> min(127, max(0, v) >> shift)
            unsigned int wds[4];
#pragma unroll
            for (int q = 0; q < 4; ++q)
                wds[q] = (unsigned int)min(127, best[4 * q] >> fs.shift) | (unsigned int)min(127, best[4 * q + 1] >> fs.shift) << 8 |
                         (unsigned int)min(127, best[4 * q + 2] >> fs.shift) << 16 |
                         (unsigned int)min(127, best[4 * q + 3] >> fs.shift) << 24;
            a = make_uint4(wds[0], wds[1], wds[2], wds[3]);
        }
    }
    if (v < nvec) {
      if (compare) {
        if (!FUSED) a = load_x_guarded(x_t, v * 16, total_bytes);
        const uint4 b = FUSED ? b_early : x_snap[v];
        const unsigned int za = a.x ^ b.x, zb = a.y ^ b.y, zc = a.z ^ b.z, zd = a.w ^ b.w;
        changed = (za | zb | zc | zd) != 0u;
        if (changed) {
            const unsigned int aw[4] = {a.x, a.y, a.z, a.w};
            const unsigned int bw[4] = {b.x, b.y, b.z, b.w};
            unsigned int dw[4], lw[4] = {0u, 0u, 0u, 0u};
            unsigned int sw[4] = {a.x, a.y, a.z, a.w};  // the unit's new snapshot (bf16: entry by entry)
            if (DT == RRM_I8_I32) {
                const unsigned int H = 0x80808080u;
                unsigned int ovf = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    // byte-wise wrapping subtraction and its signed-overflow mask
                    const unsigned int d = ((aw[i] | H) - (bw[i] & ~H)) ^ ((aw[i] ^ ~bw[i]) & H);
                    ovf |= (aw[i] ^ bw[i]) & (aw[i] ^ d) & H;
                    dw[i] = d;
                    const unsigned int z = aw[i] ^ bw[i];
                    nelem += __popc((((z & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | z) & H);
                }
                if (ovf) atomicOr(&stats->range_error, 1u);
            } else if (DT == RRM_BF16_F32) {
                // Truncation threshold (Sec. 3.4, "Improving sparsity"): an entry whose difference is below
                // g.eps in magnitude is not applied and not committed (its snapshot entry keeps the old
                // value), so the stored projection stays the projection of the stored input.  eps = 0: exact.
                bool any_pass = false;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    unsigned int hi2 = 0, lo2 = 0, sn2 = 0;
#pragma unroll
                    for (int k = 0; k < 2; ++k) {
                        const unsigned int xa = (aw[i] >> (16 * k)) & 0xFFFFu, xb = (bw[i] >> (16 * k)) & 0xFFFFu;
                        // difference in fp32 (exact unless the operands are > 2^15 apart in magnitude),
                        // then split into a bf16 head and a bf16 tail; equal inputs give 0 and 0 (no
                        // branch: the lanes of a wavefront would diverge on it)
                        const float d = bf16_to_f32(xa) - bf16_to_f32(xb);
                        const bool differ = xa != xb;
                        const bool trunc = differ && fabsf(d) < g.eps;
                        const bool pass = differ && !trunc;
                        any_pass |= pass;
                        nelem += pass ? 1u : 0u;
                        ntrunc += trunc ? 1u : 0u;
                        tsq += trunc ? d * d : 0.f;
                        const unsigned int hi = pass ? f32_to_bf16(d) : 0u;
                        const unsigned int lo = pass ? f32_to_bf16(d - bf16_to_f32(hi)) : 0u;
                        hi2 |= hi << (16 * k);
                        lo2 |= lo << (16 * k);
                        sn2 |= (pass ? xa : xb) << (16 * k);
                    }
                    dw[i] = hi2;
                    lw[i] = lo2;
                    sw[i] = sn2;
                }
                changed = any_pass;
            } else {  // binary: the flip mask
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    dw[i] = aw[i] ^ bw[i];
                    nelem += __popc(dw[i]);
                }
            }
            if (changed) {  // (bf16: every differing entry of the unit may have been truncated)
                if (!SCATTER) {
                    d0[v] = make_uint4(dw[0], dw[1], dw[2], dw[3]);
                    if (DT == RRM_BF16_F32) d1[v] = make_uint4(lw[0], lw[1], lw[2], lw[3]);
                } else {
                    scatter_unit<DT>(g, v, make_uint4(dw[0], dw[1], dw[2], dw[3]), make_uint4(lw[0], lw[1], lw[2], lw[3]), d0, d1);
                }
                x_snap[v] = make_uint4(sw[0], sw[1], sw[2], sw[3]);  // snapshot of the input, only where it changed
                // input positions covered by this unit
                const unsigned int e0 = (unsigned int)v * g.per_vec;
                unsigned int e1 = e0 + g.per_vec - 1;
                if (e1 > (unsigned int)g.total_elems - 1) e1 = (unsigned int)g.total_elems - 1;
                p0 = (int)udiv_big(e0, g.r_c);
                p1 = (int)udiv_big(e1, g.r_c);
            }
        }
      }  // compare
        if (!changed && ((prev_mask >> (threadIdx.x & 63)) & 1ull)) {
            // changed last step, unchanged now: restore the zero of the difference buffer
            if (!SCATTER) {
                d0[v] = make_uint4(0, 0, 0, 0);
                if (DT == RRM_BF16_F32) d1[v] = make_uint4(0, 0, 0, 0);
            } else {
                scatter_unit<DT>(g, v, make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0), d0, d1);
            }
        }
    }
    // mark the output blocks that see the changed positions
    if (DT == RRM_BIN_I32) {
        if (stamp)  // (stamp 0: the layer's delta kernel reads the flip words itself)
            for (int p = p0; p <= p1; ++p) mark_tiles(g, p, tileflag, stamp);
    } else if (g.sty > 0) {  // (layers on the position-gather kernel read the bitmap instead: no flags)
        for (int p = p0; p <= p1; ++p) mark_subtiles(g, (unsigned int)p, reinterpret_cast<unsigned char*>(tileflag));
    }
    const unsigned long long mask = __ballot(changed);
    if ((threadIdx.x & 63) == 0 && v < nvec) bitmap[v >> 6] = mask;
    // change counts: summed over the wavefront, then over the workgroup, one pair of atomics per workgroup
    // (atomics on one address serialise: a pair per wavefront was the slowest part of a busy scan)
    __shared__ unsigned int s_ne[4], s_nu[4], s_nt[4];
    __shared__ float s_tq[4];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) nelem += __shfl_xor(nelem, o);
    if (DT == RRM_BF16_F32) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            ntrunc += __shfl_xor(ntrunc, o);
            tsq += __shfl_xor(tsq, o);
        }
    }
    if ((threadIdx.x & 63) == 0) {
        s_ne[threadIdx.x >> 6] = nelem;
        s_nu[threadIdx.x >> 6] = (unsigned int)__popcll(mask);
        s_nt[threadIdx.x >> 6] = ntrunc;
        s_tq[threadIdx.x >> 6] = tsq;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int ne = s_ne[0] + s_ne[1] + s_ne[2] + s_ne[3], nu = s_nu[0] + s_nu[1] + s_nu[2] + s_nu[3];
        if (nu) {
            atomicAdd(&stats->changed_elems, (unsigned long long)ne);
            atomicAdd(&stats->changed_units, (unsigned long long)nu);
        }
        const unsigned int nt = s_nt[0] + s_nt[1] + s_nt[2] + s_nt[3];
        if (DT == RRM_BF16_F32 && nt) {
            atomicAdd(&stats->truncated_elems, (unsigned long long)nt);
            atomicAdd(&stats->truncated_sumsq, (double)s_tq[0] + (double)s_tq[1] + (double)s_tq[2] + (double)s_tq[3]);
        }
        if (blockIdx.x == 0) {  // one scan launch = one delta step
            atomicAdd(&stats_base->delta_steps, 1ull);
            atomicAdd(&stats_base->total_tiles, g.tiles_per_step);
        }
    }
}

// The entry points.  The pooled fused form keeps a row of its 3x3 window in flight (12 loads of 16 bytes) and is
// fastest with about 100 registers at four wavefronts per SIMD (measured on the 27 x 27 and 13 x 13 consumers: 47 us
// against 53 us at 64 registers); every other form needs 32 to 52 registers and runs at the occupancy that allows.
template <int DT, bool SCATTER, bool FUSED>
__global__ __launch_bounds__(256) void scan_kernel(const unsigned char* __restrict__ x_t, uint4* __restrict__ x_snap,
                                                   uint4* __restrict__ d0, uint4* __restrict__ d1,
                                                   unsigned long long* __restrict__ bitmap,
                                                   unsigned int* __restrict__ tileflag, unsigned int stamp,
                                                   ScanGeom g, long long nvec, long long total_bytes,
                                                   DevStats* __restrict__ stats_base, FusedSrc fs) {
    scan_body<DT, SCATTER, FUSED, false>(x_t, x_snap, d0, d1, bitmap, tileflag, stamp, g, nvec, total_bytes, stats_base, fs);
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void scan_pooled_kernel(
    uint4* __restrict__ x_snap, uint4* __restrict__ d0, unsigned long long* __restrict__ bitmap,
    unsigned int* __restrict__ tileflag, ScanGeom g, long long nvec, long long total_bytes,
    DevStats* __restrict__ stats_base, FusedSrc fs) {
    scan_body<RRM_I8_I32, false, true, true>(nullptr, x_snap, d0, nullptr, bitmap, tileflag, 0u, g, nvec, total_bytes,
                                             stats_base, fs);
}

}  // namespace

hipError_t launch_repack(int esize, const void* x, void* dst, const ScanGeom& g, hipStream_t s) {
    const long long blocks = (g.total_elems + 255) / 256;
    if (blocks <= 0) return hipSuccess;
    if (esize == 1 && g.groups == 1 && g.cp == 4 && g.c <= 4) {
        const long long n_pos = g.total_elems / g.c;
        hipLaunchKernelGGL(repack_word_kernel, dim3((unsigned int)((n_pos + 255) / 256)), dim3(256), 0, s,
                           (const unsigned char*)x, (unsigned int*)dst, g, (unsigned int)n_pos);
        return hipGetLastError();
    }
    if (esize == 1)
        hipLaunchKernelGGL(repack_kernel<1>, dim3((unsigned int)blocks), dim3(256), 0, s, (const unsigned char*)x,
                           (unsigned char*)dst, g);
    else
        hipLaunchKernelGGL(repack_kernel<2>, dim3((unsigned int)blocks), dim3(256), 0, s, (const unsigned char*)x,
                           (unsigned char*)dst, g);
    return hipGetLastError();
}

hipError_t launch_scan(int dtype, const void* x_t, void* x_snap, void* d0, void* d1, unsigned long long* bitmap,
                       unsigned int* tileflag, unsigned int stamp, const ScanGeom& g, DevStats* stats,
                       hipStream_t s) {
    const int esize = dtype == RRM_I8_I32 ? 1 : (dtype == RRM_BF16_F32 ? 2 : 4);
    const long long total_bytes = g.total_elems * esize;
    const long long nvec = (total_bytes + 15) / 16;
    const long long blocks = (nvec + 255) / 256;
    if (blocks <= 0) return hipSuccess;
    dim3 grid((unsigned int)blocks), block(256);
    const unsigned char* xt = static_cast<const unsigned char*>(x_t);
    const FusedSrc none{};
#define RRM_SCAN(DTV, SC)                                                                                               \
    hipLaunchKernelGGL((scan_kernel<DTV, SC, false>), grid, block, 0, s, xt, (uint4*)x_snap, (uint4*)d0, (uint4*)d1, bitmap, \
                       tileflag, stamp, g, nvec, total_bytes, stats, none)
    if (dtype == RRM_I8_I32) {
        if (g.scatter) RRM_SCAN(RRM_I8_I32, true); else RRM_SCAN(RRM_I8_I32, false);
    } else if (dtype == RRM_BF16_F32) {
        if (g.scatter) RRM_SCAN(RRM_BF16_F32, true); else RRM_SCAN(RRM_BF16_F32, false);
    } else {
        RRM_SCAN(RRM_BIN_I32, false);
    }
#undef RRM_SCAN
    return hipGetLastError();
}

hipError_t launch_scan_fused(const FusedSrc& src, void* x_snap, void* d0, unsigned long long* bitmap, unsigned int* marks,
                             const ScanGeom& g, DevStats* stats, hipStream_t s) {
    if (g.scatter || g.c % 16 != 0) return hipErrorInvalidValue;
    const long long total_bytes = g.total_elems;
    const long long nvec = total_bytes / 16;
    const long long blocks = ((nvec + 255) / 256 + 7) / 8 * 8;  // a multiple of the 8 XCDs (see the kernel)
    if (blocks <= 0) return hipSuccess;
    if (src.pool)
        hipLaunchKernelGGL(scan_pooled_kernel, dim3((unsigned int)blocks), dim3(256), 0, s, (uint4*)x_snap, (uint4*)d0, bitmap,
                           marks, g, nvec, total_bytes, stats, src);
    else
        hipLaunchKernelGGL((scan_kernel<RRM_I8_I32, false, true>), dim3((unsigned int)blocks), dim3(256), 0, s,
                           (const unsigned char*)nullptr, (uint4*)x_snap, (uint4*)d0, (uint4*)nullptr, bitmap, marks, 0u, g, nvec,
                           total_bytes, stats, src);
    return hipGetLastError();
}

}  // namespace rrm
