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
//     M = NCB blocks of 32 output channels
//     N = 16 x (gathered sub-tiles), two sub-tiles per MFMA
//     K = (filter tap, 16-byte channel chunk) pairs, two per MFMA
//         (v_mfma_i32_32x32x32_i8 / v_mfma_f32_32x32x16_bf16; lane l supplies row/column l%32 and the
//          16 bytes of pair 2k + l/32).  The 32x32 shapes are used because one wavefront per SIMD issues
//         them back to back at the full rate, which the 16x16 shapes only reach with two wavefronts.
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
// Each wavefront owns every fourth pair of gathered sub-tiles and all NCB channel blocks (register
// blocking NCB x NT/8), so one weight fragment read feeds NT/8 MFMAs and one window read feeds NCB MFMAs.
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
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

template <int DT>
struct Acc;
template <>
struct Acc<RRM_I8_I32> {
    typedef v16i type;
    typedef int4 vec;
    typedef int scalar;
};
template <>
struct Acc<RRM_BF16_F32> {
    typedef v16f type;
    typedef float4 vec;
    typedef float scalar;
};

// D (32x32) += A (32 x K) * B (K x 32); lane l holds row / column l%32 of A / B and 16 bytes of K
// (half l/32), and of D the column l%32 with rows 8*(r/4) + 4*(l/32) + r%4 in register r.
__device__ __forceinline__ v16i mma(const uint4& a, const uint4& b, v16i c) {
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(v4i, a), __builtin_bit_cast(v4i, b), c, 0, 0, 0);
}
__device__ __forceinline__ v16f mma(const uint4& a, const uint4& b, v16f c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0,
                                                   0);
}

// Issue order of a K step for the instruction scheduler: N_MFMA matrix instructions with N_READ LDS reads
// spread evenly between them.
template <int I, int N_MFMA, int N_READ>
__device__ __forceinline__ void sched_interleave() {
    if constexpr (I < N_MFMA) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
        constexpr int R = (N_READ * (I + 1)) / N_MFMA - (N_READ * I) / N_MFMA;
        if constexpr (R > 0) __builtin_amdgcn_sched_group_barrier(0x100, R, 0);  // R LDS reads
        sched_interleave<I + 1, N_MFMA, N_READ>();
    }
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
__global__ __launch_bounds__(CONV_THREADS, (NCB * NT >= 32 ? 1 : 2)) void conv_gather_kernel(
    const unsigned char* __restrict__ src0, const unsigned char* __restrict__ src1,
    const unsigned char* __restrict__ zero16, unsigned int* flags, unsigned int* ctrl,
    const uint4* __restrict__ wpack, const int* __restrict__ offtab, const void* __restrict__ bias_v, void* y_v,
    ConvGeom g, DevStats* __restrict__ stats) {
    typedef typename Acc<DT>::type acc_t;
    typedef typename Acc<DT>::vec vec_t;
    typedef typename Acc<DT>::scalar sc_t;
    constexpr int NP = NT / 8;  // pairs of gathered sub-tiles per wavefront
    constexpr int MAXU = CONV_MAX_STAGE_UNITS;  // staged 16-byte units per thread and slab (host guarantees)
    static_assert(NT % 8 == 0, "NT must be a multiple of two sub-tiles per wavefront");

    // LDS: [weights x nbuf][windows (TERMS planes) x nbuf][K-pair table]
    extern __shared__ uint4 smem[];
    unsigned char* lds = reinterpret_cast<unsigned char*>(smem);
    const int nbuf = g.nslab > 1 ? 2 : 1;
    const int nq2 = 2 * g.nq;  // MFMA steps (two K pairs each) per slab; a K step is two of them
    const int a_bytes = NCB * nq2 * 1024;
    const int plane_bytes = NT * g.slot_bytes;  // one term's windows
    const int b_bytes = TERMS * plane_bytes;
    unsigned char* bbase = lds + nbuf * a_bytes;
    int2* tab = reinterpret_cast<int2*>(bbase + nbuf * b_bytes);
    __shared__ int s_sub[NT];   // gathered sub-tile ids
    __shared__ unsigned int s_base[NT];  // source byte offset of the window origin (wraps when the origin is in the padding)
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
    // packed weights: [group][32-channel block (padded to ncbg*NCB)][MFMA step][lane]; a slab is MFMA steps
    // slab*nq2 .. slab*nq2 + nq2 - 1 of each of this workgroup's NCB blocks
    const int kall = g.nslab * nq2;
    const uint4* wbase = wpack + ((size_t)(grp * ncbg + cbg) * NCB) * kall * 64 + lane;
    auto stage_weights = [&](int slab) {
        unsigned char* dst = lds + (slab & (nbuf - 1)) * a_bytes;
#pragma unroll
        for (int c = 0; c < NCB; ++c) {
            const uint4* src = wbase + (size_t)(c * kall + slab * nq2) * 64;
            for (int q = wave; q < nq2; q += 4)
                __builtin_amdgcn_global_load_lds((gptr_t)(src + (size_t)q * 64), (lptr_t)(dst + (c * nq2 + q) * 1024), 16,
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
    const int2* utab = reinterpret_cast<const int2*>(offtab) + g.nq * 4;
    for (int e = tid; e < g.nq * 4; e += CONV_THREADS)  // K-pair table, the same for every slab
        tab[e] = reinterpret_cast<const int2*>(offtab)[e];
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
    // a single slab of weights serves every unit of the workgroup
    const bool w_resident = g.nslab == 1;
    if (w_resident && !g.early_weights) stage_weights(0);

    // lane roles: position j of sub-tile `half` of a pair (MFMA column l%32), K pair `khalf` of an MFMA step;
    // of the result it holds channels 8*g + 4*khalf + (0..3), g = 0..3, of each 32-channel block
    const int j = lane & 15, half = (lane >> 4) & 1, khalf = lane >> 5;
    // lane-constant window position of its output position (tap 0,0)
    const int off_lane = (((j >> 2) * g.str_y) * g.ww + (j & 3) * g.str_x) * g.sc * 16;
    const int rot_lane = g.rot_a * (j >> 2) + g.rot_b * (j & 3);  // this position's share of the chunk rotation
    sc_t* y = static_cast<sc_t*>(y_v);
    const sc_t* bias = static_cast<const sc_t*>(bias_v);

    for (int unit = (int)blockIdx.x; unit < nunits; unit += (int)gridDim.x) {
    const bool first_unit = unit == (int)blockIdx.x, last_unit = unit + (int)gridDim.x >= nunits;
    const int first = unit * per;
    int mycount = count - first;
    if (mycount > per) mycount = per;
    if (!first_unit) __syncthreads();  // the previous unit is done with the list and the staged windows
    // this thread's rows of the staging table, and the first weight slab: neither depends on the list
    int2 ut[MAXU];
#pragma unroll
    for (int i = 0; i < MAXU; ++i) {
        const int v = tid + i * CONV_THREADS;
        ut[i] = v < NT * g.wpos * g.sc ? utab[v] : int2{0, 0};
    }
    if (!w_resident && !(g.early_weights && first_unit)) stage_weights(0);
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
        const int iy0 = 4 * sy * g.str_y - g.pad_y, ix0 = 4 * sx * g.str_x - g.pad_x;
        s_iy0[tid] = iy0;
        s_ix0[tid] = ix0;
        s_base[tid] = (unsigned int)((b * g.src_h + iy0) * g.src_w + ix0) * (unsigned int)g.pos_bytes +
                      (unsigned int)(grp * g.grp_bytes);
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
    // depend on the slab or on the sub-tiles, so it comes from a table made at create time; a thread adds
    // the window origins of its units' sub-tiles once per work unit, and a slab only adds its channel offset.  Units outside the image, or whose chunk does not exist in the last slab, read
    // a 16-byte block of zeros instead.
    const int units = mycount * g.wpos * g.sc;
    const int my_units = units > tid ? (units - tid + CONV_THREADS - 1) / CONV_THREADS : 0;  // this thread's share
    unsigned int uoff[MAXU];   // source byte offset at slab 0, 0xFFFFFFFF = zeros
    unsigned int ulast = 0;    // bit i: unit i's chunk does not exist in the last slab
#pragma unroll
    for (int i = 0; i < MAXU; ++i) {
        uoff[i] = 0xFFFFFFFFu;
        if (i < my_units) {
            const int2 u = ut[i];
            const int slot = u.x & 31, hy = (u.x >> 5) & 255, hx = (u.x >> 13) & 255;
            const int iy = s_iy0[slot] + hy, ix = s_ix0[slot] + hx;
            ulast |= (unsigned int)((u.x >> 21) & 1) << i;
            if (iy >= 0 && iy < g.src_h && ix >= 0 && ix < g.src_w) uoff[i] = s_base[slot] + (unsigned int)u.y;
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

    // this wavefront's pairs are slots (2*(wave + 4p), 2*(wave + 4p) + 1): how many pairs are in use
    const int nact = mycount > 2 * wave ? (mycount - 2 * wave + 7) / 8 : 0;

    // ---- output addresses: per pair, this lane's position of its sub-tile --------------------------------
    unsigned int ybase[NP];
    bool pos_ok[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int slot = 2 * (wave + 4 * p) + half;
        pos_ok[p] = false;
        ybase[p] = 0;
        if (slot < mycount) {
            const int yp = s_ypos[slot];               // (b*ho + 4sy)*wo + 4sx
            const int py = j >> 2, px = j & 3;
            const int row = fdiv(yp, g.magic_wo);      // b*ho + 4sy
            const int col = yp - row * g.wo + px;      // 4sx + px
            const int rin = row - fdiv(row, g.magic_ho) * g.ho + py;  // 4sy + py
            pos_ok[p] = col < g.wo && rin < g.ho;
            ybase[p] = (unsigned int)(yp + py * g.wo + px) * (unsigned int)g.c_out + (unsigned int)(grp * g.og);
        }
    }
    // channel (within the filter group) of register 4*gq of block c; the 4 registers are 4 consecutive channels
    auto chan = [&](int c, int gq) { return (cbg * NCB + c) * 32 + 8 * gq + 4 * khalf; };
    // The accumulators start from what the result is added to -- the stored projection (delta: Algorithm 1,
    // P_t = P_{t-1} + F * dI) or the bias (dense: Eq. 3) -- so these loads overlap the staging of the first
    // slab and the epilogue is a plain store.  (Channel counts that are not multiples of 4 start from zero
    // and add element by element at the end.)
    acc_t acc[NCB][NP];
#pragma unroll
    for (int c = 0; c < NCB; ++c)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const int co = chan(c, gq);
            const bool ch_ok = g.vec_store && co < g.og;
            vec_t bv = vec_t{0, 0, 0, 0};
            if (MODE == MODE_DENSE && ch_ok && bias) bv = *reinterpret_cast<const vec_t*>(bias + grp * g.og + co);
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                vec_t v = bv;
                if (MODE == MODE_DELTA && ch_ok && pos_ok[p]) v = *reinterpret_cast<const vec_t*>(y + (ybase[p] + (unsigned int)co));
                acc[c][p][4 * gq + 0] = v.x;
                acc[c][p][4 * gq + 1] = v.y;
                acc[c][p][4 * gq + 2] = v.z;
                acc[c][p][4 * gq + 3] = v.w;
            }
        }

    // ---- K loop of one slab, compiled per number of sub-tile pairs in use by the wavefront (no per-pair
    //      branches; unused slots read stale LDS and their results are dropped).  A K step is four K pairs,
    //      i.e. two MFMA steps.  Software pipeline: while K step q multiplies, the operands of step q+1 are
    //      read from LDS into a second register set (the sets swap roles every step, nothing is copied) and
    //      the table entries of step q+2 are fetched, so that no address waits for a table read.  The reads
    //      are issued one by one between the MFMAs: a wavefront that issues them in a batch leaves the
    //      matrix pipeline idle meanwhile. ----------------------------------------------------------------
    auto k_loop = [&]<int NPA>(const unsigned char* aw, const unsigned char* bw) {
        const unsigned char* ap = aw + lane * 16;
        const unsigned char* bp = bw + (2 * wave + half) * g.slot_bytes;
        const int pstride = 8 * g.slot_bytes;
        const int2* tp = tab + khalf;
        constexpr int NB1 = TERMS == 2 ? NPA : 1;
        struct Ops {
            uint4 a[2][NCB], b0[2][NPA], b1[2][NB1];
        };
        constexpr int N_MFMA = 2 * NCB * NPA * TERMS;
        constexpr int N_READ = 2 * (NCB + NPA * TERMS);
        auto load_tab = [&](int q, int2(&t)[2]) {
            t[0] = tp[4 * q];  // tap's byte offset; rotated chunk | mask << 8
            t[1] = tp[4 * q + 2];
        };
        auto fetch = [&](int q, const int2(&t)[2], Ops& o) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int off = off_lane + t[h].x + ((((t[h].y & 0xFF) + rot_lane) & (t[h].y >> 8)) << 4);
#pragma unroll
                for (int c = 0; c < NCB; ++c) o.a[h][c] = *reinterpret_cast<const uint4*>(ap + (c * nq2 + 2 * q + h) * 1024);
#pragma unroll
                for (int p = 0; p < NPA; ++p) {
                    o.b0[h][p] = *reinterpret_cast<const uint4*>(bp + off + p * pstride);
                    if (TERMS == 2) o.b1[h][p] = *reinterpret_cast<const uint4*>(bp + plane_bytes + off + p * pstride);
                }
            }
        };
        auto multiply = [&](const Ops& o) {
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int c = 0; c < NCB; ++c)
#pragma unroll
                    for (int p = 0; p < NPA; ++p) {
                        acc[c][p] = mma(o.a[h][c], o.b0[h][p], acc[c][p]);
                        if (TERMS == 2) acc[c][p] = mma(o.a[h][c], o.b1[h][p], acc[c][p]);
                    }
        };
        // one K step: multiply `cur`, read step q1 into `nxt`, fetch the table entries of step q2
        auto step = [&](const Ops& cur, Ops& nxt, int2(&t)[2], int q1, int q2) {
            int2 tn[2];
            load_tab(q2, tn);
            fetch(q1, t, nxt);
            multiply(cur);
            t[0] = tn[0];
            t[1] = tn[1];
            // issue order: the table reads, then MFMAs with the operand reads spread between them
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            sched_interleave<0, N_MFMA, N_READ>();
        };
        Ops o0, o1;
        int2 t[2];
        const int qmax = g.nq - 1;
        load_tab(0, t);
        fetch(0, t, o0);
        load_tab(min(1, qmax), t);
        for (int q = 0; q < g.nq; q += 2) {
            step(o0, o1, t, min(q + 1, qmax), min(q + 2, qmax));
            if (q + 1 < g.nq) step(o1, o0, t, min(q + 2, qmax), min(q + 3, qmax));
        }
    };

    RRM_STAMP(2);
    if (last_unit) arrive();
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
        if (nact > 1) {
            if constexpr (NP >= 2) k_loop.template operator()<2>(aw, bw);
        } else if (nact > 0) {
            k_loop.template operator()<1>(aw, bw);
        }
        if (slab < 2) RRM_STAMP(8 + 5 * slab);
    }
    RRM_STAMP(14);

    // ---- epilogue ----------------------------------------------------------------------------------------
    if (g.vec_store) {
#pragma unroll
        for (int c = 0; c < NCB; ++c)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int co = chan(c, gq);
                if (co >= g.og) continue;
#pragma unroll
                for (int p = 0; p < NP; ++p) {
                    if (!pos_ok[p]) continue;
                    vec_t o;
                    o.x = acc[c][p][4 * gq + 0];
                    o.y = acc[c][p][4 * gq + 1];
                    o.z = acc[c][p][4 * gq + 2];
                    o.w = acc[c][p][4 * gq + 3];
                    *reinterpret_cast<vec_t*>(y + (ybase[p] + (unsigned int)co)) = o;
                }
            }
    } else {
        // channel counts that are not multiples of 4: element by element
#pragma unroll
        for (int c = 0; c < NCB; ++c)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int co0 = chan(c, gq);
#pragma unroll
                for (int p = 0; p < NP; ++p) {
                    if (!pos_ok[p] || co0 >= g.og) continue;
                    sc_t* yp4 = y + (ybase[p] + (unsigned int)co0);
                    for (int k = 0; k < 4 && co0 + k < g.og; ++k) {
                        const sc_t r = acc[c][p][4 * gq + k];
                        if (MODE == MODE_DELTA) {
                            if (r != (sc_t)0) yp4[k] += r;
                        } else {
                            yp4[k] = r + (bias ? bias[grp * g.og + co0 + k] : (sc_t)0);
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
    const int resident = NUM_CU * ((lds * 2 <= 160 * 1024 && NCB * NT < 32) ? 2 : 1);  // (the largest shape uses > 256 registers)
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
    RRM_CASE(2, 16) RRM_CASE(2, 8) RRM_CASE(1, 16) RRM_CASE(1, 8)
#undef RRM_CASE
    return hipErrorInvalidValue;
}

}  // namespace

size_t conv_lds_bytes(const ConvGeom& g, int ncb, int nt, int terms) {
    return (size_t)(g.nslab > 1 ? 2 : 1) * ((size_t)ncb * 2 * g.nq * 1024 + (size_t)terms * nt * g.slot_bytes) +
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
