// Gather-tile implicit-GEMM convolution on the gfx950 matrix cores (int8 -> int32, bf16 -> fp32).
//
// Delta mode computes the second term of Eq. 5, F * (I_t - I_{t-1}), only where it is non-zero, and
// adds it in place into the stored projection (Algorithm 1: P_t = P_{t-1} + F * dI).  Dense mode
// computes Eq. 3, y = b + F * x, everywhere.
//
// Unit of work: a 4x4 block of output positions (a "sub-tile", 16 positions = one MFMA column
// block).  The scan kernel sets one byte flag per sub-tile whose receptive field contains a changed
// input.  Every workgroup of this kernel reads that flag array (a few KB at most), ranks the set flags
// with a popcount prefix sum, and takes its share of the ranked list: up to NT active sub-tiles from
// anywhere in the batch.  They become the N dimension of one GEMM per workgroup:
//     M = NCB blocks of 16 output channels
//     N = 16 x (gathered sub-tiles)
//     K = (filter tap, 16-byte channel chunk) pairs, four per MFMA
//         (v_mfma_i32_16x16x64_i8 / v_mfma_f32_16x16x32_bf16; lane l supplies row/column l%16 and the
//          16 bytes of pair 4q + l/16).
// Both operands go through LDS, one slab of channel chunks at a time:
//   * weights: the filters are packed at create time in per-lane MFMA order, K pairs ordered chunk by
//     chunk, so a slab is a contiguous run of 1 KiB fragments per channel block; wavefronts copy them
//     with LDS-direct loads (global_load_lds_dwordx4, no registers), double-buffered across slabs;
//   * activations: the gathered sub-tiles' input windows, gathered 16 bytes per lane with the same
//     LDS-direct loads (chunk index rotated by position against bank conflicts; units outside the
//     image read a block of zeros), also double-buffered.  In delta mode the source is the difference
//     buffer, zero where nothing changed.
// The source is always in a 16-byte-chunk layout [stream][row][column][group][chunk]: the caller's x
// when its channel runs are 16-byte multiples, otherwise the padded (or column-folded) copy that the
// scan / repack kernels write (see scan.hip); the kernel itself only sees "source positions" of
// pos_bytes bytes with their own strides and window size.
// Each wavefront owns every fourth gathered sub-tile and all NCB channel blocks (register blocking
// NCB x NT/4), so one weight fragment read feeds NT/4 MFMAs and one window read feeds NCB MFMAs.
// The number of sub-tiles per workgroup adapts on the device: few active sub-tiles are spread one per
// workgroup (latency), many are packed NT per workgroup (operand reuse).
// Every output element has exactly one owner: no atomics on y, results reproducible run to run.
// The last workgroup to arrive clears the flag array and the arrival counter, so nothing on the host
// changes between steps (HIP-graph replay safe).
#include <algorithm>

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

#ifdef RRM_TRACE
// debug build only: cycle stamps of workgroup (0,0), wavefront 0 into the spare stats slots
#define RRM_STAMP(k)                                                                               \
    do {                                                                                           \
        if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0)                                \
            reinterpret_cast<unsigned long long*>(stats + 32)[k] = __builtin_readcyclecounter();   \
    } while (0)
#else
#define RRM_STAMP(k) do {} while (0)
#endif

typedef const void __attribute__((address_space(1))) * gptr_t;
typedef void __attribute__((address_space(3))) * lptr_t;

template <int DT, int MODE, int NCB, int NT, int TERMS>
__global__ __launch_bounds__(CONV_THREADS, 2) void conv_gather_kernel(
    const unsigned char* __restrict__ src0, const unsigned char* __restrict__ src1,
    const unsigned char* __restrict__ zero16, unsigned int* flags, unsigned int* ctrl,
    const uint4* __restrict__ wpack, const int* __restrict__ offtab, const void* __restrict__ bias_v, void* y_v,
    ConvGeom g, DevStats* __restrict__ stats) {
    typedef typename Acc<DT>::type acc_t;
    typedef typename Acc<DT>::vec vec_t;
    typedef typename Acc<DT>::scalar sc_t;
    constexpr int NS = NT / 4;  // gathered sub-tiles per wavefront
    constexpr int MAXU = CONV_MAX_STAGE_UNITS;  // staged 16-byte units per thread and slab (host guarantees)
    static_assert(NT % 4 == 0, "NT must be a multiple of the wavefront count");

    // LDS: [weights x nbuf][windows (TERMS planes) x nbuf][K-pair table]
    extern __shared__ uint4 smem[];
    unsigned char* lds = reinterpret_cast<unsigned char*>(smem);
    const int nbuf = g.nslab > 1 ? 2 : 1;
    const int a_bytes = NCB * g.nq * 1024;
    const int plane_bytes = NT * g.slot_bytes;  // one term's windows
    const int b_bytes = TERMS * plane_bytes;
    unsigned char* bbase = lds + nbuf * a_bytes;
    int2* tab = reinterpret_cast<int2*>(bbase + nbuf * b_bytes);
    __shared__ int s_sub[NT];   // gathered sub-tile ids
    __shared__ int s_pix[NT];   // first input position of the sub-tile's image: b*h*w
    __shared__ int s_iy0[NT];   // window origin in the input map (may be negative: padding)
    __shared__ int s_ix0[NT];
    __shared__ int s_ypos[NT];  // output position index of the sub-tile's corner: (b*ho + 4sy)*wo + 4sx
    __shared__ int s_scan[CONV_THREADS / WAVE];
    __shared__ int s_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int ncbg = (g.ncb + NCB - 1) / NCB;  // channel-block groups per filter group
    const int grp = blockIdx.y / ncbg;
    const int cbg = blockIdx.y - grp * ncbg;
    // packed weights: [group][channel block (padded to ncbg*NCB)][K step][lane]; a slab is K steps
    // slab*nq .. slab*nq + nq - 1 of each of this workgroup's NCB blocks
    const int kall = g.nslab * g.nq;
    const uint4* wbase = wpack + ((size_t)(grp * ncbg + cbg) * NCB) * kall * 64 + lane;
    auto stage_weights = [&](int slab) {
        unsigned char* dst = lds + (slab & (nbuf - 1)) * a_bytes;
#pragma unroll
        for (int c = 0; c < NCB; ++c) {
            const uint4* src = wbase + (size_t)(c * kall + slab * g.nq) * 64;
            for (int q = wave; q < g.nq; q += 4)
                __builtin_amdgcn_global_load_lds((gptr_t)(src + (size_t)q * 64), (lptr_t)(dst + (c * g.nq + q) * 1024), 16,
                                                 0, 0);
        }
    };
    RRM_STAMP(0);
    // Small grids (one stream of a small map): the first weight slab does not depend on the work
    // list, so its copy is started before the flag scan and overlaps it.
    if (g.early_weights) stage_weights(0);

    // ---- which sub-tiles does this workgroup own? ----------------------------------------------------
    // The flag array (one byte per sub-tile, padded with zeros to whole 16-byte vectors) is split into
    // contiguous runs of vectors, one run per thread, loaded in one go and kept in registers.
    constexpr int FW = 8;  // words per thread held in registers (more are re-read: > 8192 sub-tiles)
    constexpr unsigned int LOW = 0x01010101u;
    const int wpt = (g.n_words + CONV_THREADS - 1) / CONV_THREADS;
    const int w_lo = tid * wpt;
    unsigned int fw[FW];
    int count, excl = 0, mine = 0;
    if (MODE == MODE_DELTA) {
#pragma unroll
        for (int i = 0; i < FW; ++i) fw[i] = (i < wpt && w_lo + i < g.n_words) ? flags[w_lo + i] & LOW : 0u;
#pragma unroll
        for (int i = 0; i < FW; ++i) mine += __popc(fw[i]);
        for (int i = FW; i < wpt; ++i)
            if (w_lo + i < g.n_words) mine += __popc(flags[w_lo + i] & LOW);
        // popcount prefix sum (every workgroup does the same small scan)
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
    RRM_STAMP(16);
    // The grid holds at most as many workgroups as the chip runs at once.  The active sub-tiles are cut
    // into work units of `per` sub-tiles: few sub-tiles are spread thinly (a unit's latency grows with its
    // size), many are packed NT per unit (operand reuse), and a workgroup takes units blockIdx.x,
    // blockIdx.x + gridDim.x, ... until the list is exhausted (the same bound for every workgroup).
    int per = (count + (int)gridDim.x - 1) / (int)gridDim.x;
    if (per < 1) per = 1;
    if (per > NT) per = NT;
    const int nunits = (count + per - 1) / per;

    unsigned int arrived_before = 0;  // thread 0: workgroups that signalled before this one
    // Arrival signal, sent once this workgroup has read the flags for the last time.  Every thread has
    // consumed its flag loads before a barrier by then and the signalling thread's stores do not matter to
    // the flags, so no memory fence is needed (a device-scope fence would write back the whole L2).  The
    // answer is needed only at the end; the signal is sent where no load of the issuing thread follows
    // closely (returns are in order: a later load would wait for the atomic as well).
    auto arrive = [&]() {
        if (MODE == MODE_DELTA && tid == 0) arrived_before = atomicAdd(&ctrl[0], 1u);
    };
    // The last workgroup to arrive knows that every workgroup has read the flags: it clears them (and
    // the arrival counter) for the next step, at its own end, off everybody's critical path.
    auto retire = [&]() {
        if (MODE != MODE_DELTA) return;
        if (tid == 0) s_last = (arrived_before == gridDim.x * gridDim.y - 1u) ? 1 : 0;
        __syncthreads();
        if (s_last) {
            for (int w = tid; w < g.n_words; w += CONV_THREADS) flags[w] = 0u;
            if (tid == 0) {
                ctrl[0] = 0u;
                if (count) atomicAdd(&stats[0].active_tiles, (unsigned long long)count);
            }
        }
    };
    if ((int)blockIdx.x >= nunits) {
        __builtin_amdgcn_s_waitcnt(0);  // let an early weight copy land before the LDS is released
        arrive();
        retire();
        return;
    }
    for (int e = tid; e < g.nq * 4; e += CONV_THREADS)  // K-pair table, the same for every slab
        tab[e] = reinterpret_cast<const int2*>(offtab)[e];
    // a single slab of weights serves every unit of the workgroup
    const bool w_resident = g.nslab == 1;
    if (w_resident && !g.early_weights) stage_weights(0);

    const int j = lane & 15, kgrp = lane >> 4;
    // lane-constant window position of its output position (tap 0,0)
    const int off_lane = (((j >> 2) * g.str_y) * g.ww + (j & 3) * g.str_x) * g.sc * 16;
    const int rot_lane = g.rot_a * (j >> 2) + g.rot_b * (j & 3);  // this position's share of the chunk rotation
    sc_t* y = static_cast<sc_t*>(y_v);
    const sc_t* bias = static_cast<const sc_t*>(bias_v);
    const bool all_vec = g.vec_store && (cbg * NCB + NCB) * 16 <= g.og;  // every lane's 4 channels exist

    for (int unit = (int)blockIdx.x; unit < nunits; unit += (int)gridDim.x) {
    const bool first_unit = unit == (int)blockIdx.x, last_unit = unit + (int)gridDim.x >= nunits;
    const int first = unit * per;
    int mycount = count - first;
    if (mycount > per) mycount = per;
    if (!first_unit) __syncthreads();  // the previous unit is done with the list and the staged windows
    if (MODE == MODE_DELTA) {
        // the rank of a set flag is the number of set flags before it; keep ranks first .. first+mycount-1
        if (excl + mine > first && excl < first + mycount) {
            int rank = excl - first;
            auto take = [&](unsigned int word, int widx) {
                unsigned int bits = word & LOW;
                while (bits) {
                    const int bpos = __ffs(bits) - 1;
                    bits &= bits - 1;
                    if (rank >= 0 && rank < mycount) s_sub[rank] = widx * 4 + (bpos >> 3);
                    ++rank;
                }
            };
#pragma unroll
            for (int i = 0; i < FW; ++i) take(fw[i], w_lo + i);
            for (int i = FW; i < wpt; ++i)
                if (w_lo + i < g.n_words) take(flags[w_lo + i], w_lo + i);
        }
    } else if (tid < mycount) {
        s_sub[tid] = first + tid;
    }
    __syncthreads();
    RRM_STAMP(17);
    // per-slot geometry, once
    if (tid < mycount) {
        const int id = s_sub[tid];
        const int b = fdiv(id, g.magic_sub);
        const int r = id - b * (g.sty * g.stx);
        const int sy = fdiv(r, g.magic_stx), sx = r - sy * g.stx;
        s_pix[tid] = b * g.src_h * g.src_w;
        s_iy0[tid] = 4 * sy * g.str_y - g.pad_y;
        s_ix0[tid] = 4 * sx * g.str_x - g.pad_x;
        s_ypos[tid] = (b * g.ho + 4 * sy) * g.wo + 4 * sx;
    }
    __syncthreads();
    RRM_STAMP(1);

    // ---- window staging --------------------------------------------------------------------------------
    // A staged unit is 16 bytes of one (sub-tile, window position, chunk-in-slab).  Unit v lives at LDS
    // byte 16*v of its plane, v = (slot*wpos + hp)*sc + cs, where slot cs of a position holds chunk
    // (cs - rotation(position)) mod rot_p, so that the MFMA operand reads of a sub-tile's 16 positions fall into
    // different banks.  Consecutive lanes own consecutive units, which is what the LDS-direct gather
    // (per-lane global address, LDS address = wave base + 16*lane) needs.  The decomposition does not
    // depend on the slab, so each thread works out the source offsets of its units once; a slab only adds
    // its channel offset.  Units outside the image, or whose chunk does not exist in the last slab, read
    // a 16-byte block of zeros instead.
    const int units = mycount * g.wpos * g.sc;
    const int my_units = units > tid ? (units - tid + CONV_THREADS - 1) / CONV_THREADS : 0;  // this thread's share
    unsigned int uoff[MAXU];   // source byte offset at slab 0, 0xFFFFFFFF = zeros
    unsigned int ulast = 0;    // bit i: unit i's chunk does not exist in the last slab
#pragma unroll
    for (int i = 0; i < MAXU; ++i) {
        uoff[i] = 0xFFFFFFFFu;
        if (i < my_units) {
            const int v = tid + i * CONV_THREADS;
            const int r = fdiv(v, g.magic_sc[0]), cs = v - r * g.sc;
            const int slot = fdiv(r, g.magic_wsc[0]), hp = r - slot * g.wpos;
            const int hy = fdiv(hp, g.magic_ww), hx = hp - hy * g.ww;
            int cc = cs;  // the chunk held by slot cs of this position (see rot_p)
            if (cs < g.rot_p)
                cc = (cs - g.rot_a * fdiv(hy, g.magic_sy) - g.rot_b * fdiv(hx, g.magic_sx)) & (g.rot_p - 1);
            const int iy = s_iy0[slot] + hy, ix = s_ix0[slot] + hx;
            if (cc >= g.last_sc) ulast |= 1u << i;
            if (iy >= 0 && iy < g.src_h && ix >= 0 && ix < g.src_w)
                uoff[i] = (unsigned int)(s_pix[slot] + iy * g.src_w + ix) * (unsigned int)g.pos_bytes +
                          (unsigned int)(grp * g.grp_bytes + cc * 16);
        }
    }
    const unsigned int slab_src_bytes = (unsigned int)(g.sc * 16);  // source bytes between consecutive slabs
    auto stage_windows = [&](int slab) {
        unsigned char* dst = bbase + (slab & (nbuf - 1)) * b_bytes;
        const bool last = slab == g.nslab - 1;
#pragma unroll
        for (int i = 0; i < MAXU; ++i) {
            if (i >= my_units) break;
            const bool real = uoff[i] != 0xFFFFFFFFu && !(last && ((ulast >> i) & 1u));
            const unsigned int o = uoff[i] + (unsigned int)slab * slab_src_bytes;
            unsigned char* d = dst + (i * CONV_THREADS + wave * 64) * 16;  // wave-uniform; lane adds 16*lane
            const unsigned char* p0 = real ? src0 + o : zero16;
            __builtin_amdgcn_global_load_lds((gptr_t)p0, (lptr_t)d, 16, 0, 0);
            if (TERMS == 2) {
                const unsigned char* p1 = real ? src1 + o : zero16;
                __builtin_amdgcn_global_load_lds((gptr_t)p1, (lptr_t)(d + plane_bytes), 16, 0, 0);
            }
        }
    };

    // this wavefront's sub-tile slots are wave, wave + 4, ...: how many of them are in use
    const int nact = mycount > wave ? (mycount - wave + 3) / 4 : 0;

    // ---- output addresses: lane holds 4 consecutive output channels of one position ----------------------
    unsigned int ybase[NS];
    bool pos_ok[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int slot = wave + 4 * s;
        pos_ok[s] = false;
        ybase[s] = 0;
        if (slot < mycount) {
            const int yp = s_ypos[slot];               // (b*ho + 4sy)*wo + 4sx
            const int py = j >> 2, px = j & 3;
            const int row = fdiv(yp, g.magic_wo);      // b*ho + 4sy
            const int col = yp - row * g.wo + px;      // 4sx + px
            const int rin = row - fdiv(row, g.magic_ho) * g.ho + py;  // 4sy + py
            pos_ok[s] = col < g.wo && rin < g.ho;
            ybase[s] = (unsigned int)(yp + py * g.wo + px) * (unsigned int)g.c_out + (unsigned int)(grp * g.og);
        }
    }
    // The accumulators start from what the result is added to -- the stored projection (delta: Algorithm 1,
    // P_t = P_{t-1} + F * dI) or the bias (dense: Eq. 3) -- so these loads overlap the staging of the first
    // slab and the epilogue is a plain store.  (Ragged channel counts start from zero and add at the end.)
    acc_t acc[NCB][NS];
#pragma unroll
    for (int c = 0; c < NCB; ++c) {
        vec_t bv = vec_t{0, 0, 0, 0};
        if (MODE == MODE_DENSE && all_vec && bias)
            bv = *reinterpret_cast<const vec_t*>(bias + grp * g.og + (cbg * NCB + c) * 16 + 4 * kgrp);
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            vec_t v = bv;
            if (MODE == MODE_DELTA && all_vec && pos_ok[s])
                v = *reinterpret_cast<const vec_t*>(y + (ybase[s] + (unsigned int)((cbg * NCB + c) * 16 + 4 * kgrp)));
            acc[c][s] = acc_t{v.x, v.y, v.z, v.w};
        }
    }

    // ---- K loop of one slab, compiled per number of sub-tiles in use by the wavefront (no per-sub-tile
    //      branches; unused slots read stale LDS and their results are dropped) --------------------------
    auto k_loop = [&]<int NSA>(const unsigned char* aw, const unsigned char* bw) {
        const unsigned char* ap = aw + lane * 16;
        const unsigned char* bp = bw + wave * g.slot_bytes;
        const int sstride = 4 * g.slot_bytes;
        const int2* tp = tab + kgrp;
        uint4 a[NCB], b0[NSA], b1[TERMS == 2 ? NSA : 1];
        auto fetch = [&](int q, uint4(&a_)[NCB], uint4(&b0_)[NSA], uint4(&b1_)[TERMS == 2 ? NSA : 1]) {
            const int2 t = tp[4 * q];  // tap's byte offset; rotated chunk | mask << 8
            const int off = off_lane + t.x + ((((t.y & 0xFF) + rot_lane) & (t.y >> 8)) << 4);
#pragma unroll
            for (int c = 0; c < NCB; ++c) a_[c] = *reinterpret_cast<const uint4*>(ap + (c * g.nq + q) * 1024);
#pragma unroll
            for (int s = 0; s < NSA; ++s) {
                b0_[s] = *reinterpret_cast<const uint4*>(bp + off + s * sstride);
                if (TERMS == 2) b1_[s] = *reinterpret_cast<const uint4*>(bp + plane_bytes + off + s * sstride);
            }
        };
        // software pipeline: the operands of K step q+1 are read from LDS while step q multiplies
        fetch(0, a, b0, b1);
        for (int q = 0; q < g.nq; ++q) {
            uint4 an[NCB], b0n[NSA], b1n[TERMS == 2 ? NSA : 1];
            fetch(min(q + 1, g.nq - 1), an, b0n, b1n);
            __builtin_amdgcn_sched_barrier(0);  // keep the reads ahead of the multiplies (the scheduler would sink them)
#pragma unroll
            for (int c = 0; c < NCB; ++c)
#pragma unroll
                for (int s = 0; s < NSA; ++s) {
                    acc[c][s] = mma(a[c], b0[s], acc[c][s]);
                    if (TERMS == 2) acc[c][s] = mma(a[c], b1[s], acc[c][s]);
                }
#pragma unroll
            for (int c = 0; c < NCB; ++c) a[c] = an[c];
#pragma unroll
            for (int s = 0; s < NSA; ++s) {
                b0[s] = b0n[s];
                if (TERMS == 2) b1[s] = b1n[s];
            }
        }
    };

    RRM_STAMP(2);
    if (last_unit) arrive();
    if (!w_resident && !(g.early_weights && first_unit)) stage_weights(0);
    stage_windows(0);
    RRM_STAMP(3);
    for (int slab = 0; slab < g.nslab; ++slab) {
        if (slab < 2) RRM_STAMP(4 + 5 * slab);
        __builtin_amdgcn_s_waitcnt(0);  // this wavefront's copies for this slab have landed in LDS
        if (slab < 2) RRM_STAMP(5 + 5 * slab);
        __syncthreads();  // ... and everyone else's; everyone is also done with the other buffer
        if (slab < 2) RRM_STAMP(6 + 5 * slab);
        if (slab + 1 < g.nslab) {  // next slab in flight during this slab's K loop (nslab > 1: weights are not resident)
            stage_weights(slab + 1);
            stage_windows(slab + 1);
        }
        if (slab < 2) RRM_STAMP(7 + 5 * slab);
        const unsigned char* aw = lds + (slab & (nbuf - 1)) * a_bytes;
        const unsigned char* bw = bbase + (slab & (nbuf - 1)) * b_bytes;
        if (nact > 2) {
            if constexpr (NS >= 4) k_loop.template operator()<4>(aw, bw);
        } else if (nact > 1) {
            if constexpr (NS >= 2) k_loop.template operator()<2>(aw, bw);
        } else if (nact > 0) {
            k_loop.template operator()<1>(aw, bw);
        }
        if (slab < 2) RRM_STAMP(8 + 5 * slab);
    }
    RRM_STAMP(14);

    // ---- epilogue ----------------------------------------------------------------------------------------
    if (all_vec) {
#pragma unroll
        for (int c = 0; c < NCB; ++c)
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                if (!pos_ok[s]) continue;
                const acc_t r = acc[c][s];
                vec_t o;
                o.x = r[0]; o.y = r[1]; o.z = r[2]; o.w = r[3];
                *reinterpret_cast<vec_t*>(y + (ybase[s] + (unsigned int)((cbg * NCB + c) * 16 + 4 * kgrp))) = o;
            }
    } else {
        // ragged channel counts: element by element
#pragma unroll
        for (int c = 0; c < NCB; ++c) {
            const int co0 = (cbg * NCB + c) * 16 + 4 * kgrp;  // within the filter group
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                if (!pos_ok[s] || co0 >= g.og) continue;
                sc_t* yp4 = y + (ybase[s] + (unsigned int)co0);
                const acc_t r = acc[c][s];
                for (int k = 0; k < 4 && co0 + k < g.og; ++k) {
                    if (MODE == MODE_DELTA) {
                        if (r[k] != (sc_t)0) yp4[k] += r[k];
                    } else {
                        yp4[k] = r[k] + (bias ? bias[grp * g.og + co0 + k] : (sc_t)0);
                    }
                }
            }
        }
    }
    }  // units
    retire();
    RRM_STAMP(15);
}

template <int DT, int MODE, int NCB, int NT, int TERMS>
hipError_t launch_one(const void* src0, const void* src1, const void* zero16, unsigned int* flags,
                      unsigned int* ctrl, const void* wpack, const int* offtab, const void* bias, void* y,
                      const ConvGeom& g, DevStats* stats, hipStream_t s) {
    const int ncbg = (g.ncb + NCB - 1) / NCB;
    const size_t lds = conv_lds_bytes(g, NCB, NT, TERMS);
    // no more workgroups than are resident at once (the kernel loops over its work units)
    const int gy = g.groups * ncbg;
    const int resident = NUM_CU * (lds * 2 <= 160 * 1024 ? 2 : 1);
    const int gx = std::min((g.n_sub + NT - 1) / NT, std::max(1, resident / gy));
    dim3 grid((unsigned int)gx, (unsigned int)gy);
    auto kern = conv_gather_kernel<DT, MODE, NCB, NT, TERMS>;
    if (lds > 64 * 1024) {
        static size_t granted = 0;  // one per instantiation; creation and launches of a process share it
        if (lds > granted) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            granted = lds;
        }
    }
    hipLaunchKernelGGL(kern, grid, dim3(CONV_THREADS), lds, s, static_cast<const unsigned char*>(src0),
                       static_cast<const unsigned char*>(src1), static_cast<const unsigned char*>(zero16), flags, ctrl,
                       static_cast<const uint4*>(wpack), offtab, bias, y, g, stats);
    return hipGetLastError();
}

template <int DT, int MODE, int TERMS>
hipError_t launch_shape(int ncb, int nt, const void* src0, const void* src1, const void* zero16,
                        unsigned int* flags, unsigned int* ctrl, const void* wpack, const int* offtab, const void* bias, void* y,
                        const ConvGeom& g, DevStats* stats, hipStream_t s) {
#define RRM_CASE(CBV, NTV)                                                                                          \
    if (ncb == CBV && nt == NTV)                                                                                     \
        return launch_one<DT, MODE, CBV, NTV, TERMS>(src0, src1, zero16, flags, ctrl, wpack, offtab, bias, y, g, stats, s);
    RRM_CASE(4, 4) RRM_CASE(4, 8) RRM_CASE(4, 16) RRM_CASE(1, 4) RRM_CASE(1, 8) RRM_CASE(1, 16)
#undef RRM_CASE
    return hipErrorInvalidValue;
}

}  // namespace

size_t conv_lds_bytes(const ConvGeom& g, int ncb, int nt, int terms) {
    return (size_t)(g.nslab > 1 ? 2 : 1) * ((size_t)ncb * g.nq * 1024 + (size_t)terms * nt * g.slot_bytes) +
           (size_t)g.nq * 4 * sizeof(int2);
}

hipError_t launch_conv(int dtype, int mode, int ncb, int nt, int terms, const void* src0, const void* src1,
                       const void* zero16, unsigned int* flags, unsigned int* ctrl, const void* wpack, const int* offtab,
                       const void* bias, void* y, const ConvGeom& g, DevStats* stats, hipStream_t s) {
    if (dtype == RRM_I8_I32) {
        if (mode == MODE_DELTA)
            return launch_shape<RRM_I8_I32, MODE_DELTA, 1>(ncb, nt, src0, src1, zero16, flags, ctrl, wpack, offtab, bias, y, g, stats, s);
        return launch_shape<RRM_I8_I32, MODE_DENSE, 1>(ncb, nt, src0, src1, zero16, flags, ctrl, wpack, offtab, bias, y, g, stats, s);
    }
    if (mode == MODE_DENSE)
        return launch_shape<RRM_BF16_F32, MODE_DENSE, 1>(ncb, nt, src0, src1, zero16, flags, ctrl, wpack, offtab, bias, y, g, stats, s);
    if (terms == 2)
        return launch_shape<RRM_BF16_F32, MODE_DELTA, 2>(ncb, nt, src0, src1, zero16, flags, ctrl, wpack, offtab, bias, y, g, stats, s);
    return launch_shape<RRM_BF16_F32, MODE_DELTA, 1>(ncb, nt, src0, src1, zero16, flags, ctrl, wpack, offtab, bias, y, g, stats, s);
}

}  // namespace rrm
