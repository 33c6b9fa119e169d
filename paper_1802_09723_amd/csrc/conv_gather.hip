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
// A workgroup has eight wavefronts with two roles.  Wavefronts 0-3 ("producers") own the work list and
// the copies into LDS; wavefronts 4-7 ("consumers", one per SIMD) only multiply and write results.  Each
// consumer owns every fourth pair of gathered sub-tiles and all NCB channel blocks (register blocking
// NCB x NT/8), so one weight fragment read feeds NT/8 MFMAs and one window read feeds NCB MFMAs.  While
// the consumers multiply slab k, the producers stage slab k+1 -- or the first slab of the workgroup's next
// work unit, including its list and address work -- into the other buffer; the two roles meet at one
// barrier per slab.  The producers' address arithmetic and load issue thus run in the shadow of the matrix
// instructions of another wavefront on the same SIMD.
// The number of sub-tiles per workgroup adapts on the device: few active sub-tiles are spread one per
// workgroup (latency), many are packed NT per workgroup (operand reuse).
// Every output element has exactly one owner: no atomics on y, results reproducible run to run.
// The grid holds no more workgroups than the chip runs at once; a workgroup takes work units
// blockIdx.x, blockIdx.x + gridDim.x, ... of the ranked list.
// The last workgroup to arrive clears the flag array and the arrival counter, so nothing on the host
// changes between steps (HIP-graph replay safe).
#include <algorithm>
#include <mutex>

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

// Workgroup barrier that publishes LDS contents only: it waits for this wavefront's LDS operations, not for its
// outstanding global loads (__syncthreads() would also wait for the copies into LDS that were started early).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

typedef const void __attribute__((address_space(1))) * gptr_t;
typedef void __attribute__((address_space(3))) * lptr_t;

constexpr int WG_THREADS = 2 * CONV_THREADS;  // 4 producer + 4 consumer wavefronts
constexpr int LIST_CAP = 1024;                // ranked sub-tile ids held in LDS per ranking round

template <int DT, int MODE, int NCB, int NT, int TERMS>
__global__ __launch_bounds__(WG_THREADS) void conv_gather_kernel(
    const unsigned char* __restrict__ src0, const unsigned char* __restrict__ src1,
    const unsigned char* __restrict__ zero16, unsigned int* flags, unsigned int* ctrl,
    const uint4* __restrict__ wpack, const int* __restrict__ offtab, const void* __restrict__ bias_v, void* y_v,
    ConvGeom g, DevStats* __restrict__ stats) {
    typedef typename Acc<DT>::type acc_t;
    typedef typename Acc<DT>::vec vec_t;
    typedef typename Acc<DT>::scalar sc_t;
    constexpr int NP = NT / 8;  // pairs of gathered sub-tiles per consumer wavefront
    constexpr int MAXU = CONV_MAX_STAGE_UNITS;  // staged 16-byte units per producer thread and slab (host guarantees)
    static_assert(NT % 8 == 0 && NT <= 32, "NT: two sub-tiles per consumer wavefront, slot index in 5 bits");
    static_assert(LIST_CAP >= 2 * NT, "a ranking round holds at least two work units");

    // LDS: [weights x nbuf_a][windows (TERMS planes) x 2][K-pair table]
    extern __shared__ uint4 smem[];
    unsigned char* lds = reinterpret_cast<unsigned char*>(smem);
    const int nbuf_a = g.nslab > 1 ? 2 : 1;  // a single slab of weights is staged once and serves every unit
    const int nq2 = 2 * g.nq;  // MFMA steps (two K pairs each) per slab; a K step is two of them
    const int a_bytes = NCB * nq2 * 1024;
    const int plane_bytes = g.nt * g.slot_bytes;  // one term's windows (g.nt <= NT slots: large windows get fewer)
    const int b_bytes = TERMS * plane_bytes;
    unsigned char* bbase = lds + nbuf_a * a_bytes;
    int2* tab = reinterpret_cast<int2*>(bbase + 2 * b_bytes);
    __shared__ int s_list[LIST_CAP];         // ranked sub-tile ids of this workgroup's units of a round
    __shared__ unsigned int s_base[4][NT];   // per producer wavefront: source byte offset of the window origin
    __shared__ int s_iy0[4][NT];             //   (wraps when the origin is in the padding) and the origin itself
    __shared__ int s_ix0[4][NT];
    __shared__ int s_scan[CONV_THREADS / WAVE];
    __shared__ int s_excl[CONV_THREADS];     // per producer thread: set flags before its share, within its wavefront
    __shared__ int s_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool producer = wave < 4;
    const int cw = wave - 4;  // consumer index
    // Workgroup coordinates: BX of GX unit lanes (a lane takes work units BX, BX + GX, ...), BY of GY channel-block
    // groups.  With g.xcd_gy set the grid is one-dimensional and the coordinates are dealt so that the GY
    // workgroups of a lane, which gather the same input windows, sit on the same XCD (workgroups go to the
    // eight XCDs round-robin by their linear index) and find each other's windows in that XCD's L2.
    int BX, BY, GX, GY;
    if (g.xcd_gy) {
        const int lin = (int)blockIdx.x;
        GY = g.xcd_gy;
        GX = (int)gridDim.x / GY;
        const int dealt = (GX >> 3) * 8 * GY;  // workgroups of the lanes that are dealt XCD by XCD
        if (lin < dealt) {
            const int slot = lin >> 3;
            BY = slot % GY;
            BX = (slot / GY) * 8 + (lin & 7);
        } else {  // (the few lanes beyond a multiple of eight: wherever they fall)
            const int rem = lin - dealt;
            BY = rem % GY;
            BX = (GX >> 3) * 8 + rem / GY;
        }
    } else {
        BX = (int)blockIdx.x;
        BY = (int)blockIdx.y;
        GX = (int)gridDim.x;
        GY = (int)gridDim.y;
    }

    const int ncbg = (g.ncb + NCB - 1) / NCB;  // channel-block groups per filter group
    const int grp = BY / ncbg;
    const int cbg = BY - grp * ncbg;
    // packed weights: [group][32-channel block (padded to ncbg*NCB)][MFMA step][lane]; a slab is MFMA steps
    // slab*nq2 .. slab*nq2 + nq2 - 1 of each of this workgroup's NCB blocks
    const int kall = g.nslab * nq2;
    const uint4* wbase = wpack + ((size_t)(grp * ncbg + cbg) * NCB) * kall * 64 + lane;
    auto stage_weights = [&](int slab, int buf) {  // producers
        unsigned char* dst = lds + buf * a_bytes;
#pragma unroll
        for (int c = 0; c < NCB; ++c) {
            const uint4* src = wbase + (size_t)(c * kall + slab * nq2) * 64;
            for (int q = wave; q < nq2; q += 4)
                __builtin_amdgcn_global_load_lds((gptr_t)(src + (size_t)q * 64), (lptr_t)(dst + (c * nq2 + q) * 1024), 16,
                                                 0, 0);
        }
    };
    // The first weight slab and this thread's rows of the staging table (which serve every unit) do not
    // depend on the work list.  A dense launch starts their loads at once; a delta launch after the loads
    // of the list phase, which would otherwise queue behind them (loads return in order), and not at all in
    // a workgroup that gets no unit.
    const int2* utab = reinterpret_cast<const int2*>(offtab) + g.nq * 4;
    int2 ut[MAXU];
    auto early_loads = [&]() {
        if (!producer) return;
        stage_weights(0, 0);
#pragma unroll
        for (int i = 0; i < MAXU; ++i) {
            const int v = tid + i * CONV_THREADS;
            ut[i] = v < g.nt * g.wpos * g.sc ? utab[v] : int2{0, 0};
        }
    };
    if (MODE == MODE_DENSE) early_loads();
    for (int e = tid; e < g.nq * 4; e += WG_THREADS)  // K-pair table, the same for every slab
        tab[e] = reinterpret_cast<const int2*>(offtab)[e];

    // ---- how many sub-tiles are active? -------------------------------------------------------------
    // The flag array (one byte per sub-tile) is split into contiguous runs of 64-flag groups, one run per
    // producer thread.  A group is loaded as four 16-byte vectors and squeezed into a 64-bit mask; a thread's
    // first group stays in registers, further ones (more than 16384 sub-tiles per launch) are re-read.
    constexpr unsigned int LOW = 0x01010101u;
    const uint4* fvp = reinterpret_cast<const uint4*>(flags);
    const int n_vec = (g.n_words + 3) >> 2;
    const int n_grp = (n_vec + 3) >> 2;
    const int gpt = (n_grp + CONV_THREADS - 1) / CONV_THREADS;
    auto load_group = [&](int gi) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = 4 * gi + u < n_vec ? fvp[4 * gi + u] : uint4{0u, 0u, 0u, 0u};
        unsigned long long m = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            // (byte flags 0/1 of a word -> 4 bits: the product moves byte i's bit to bit 24 + i)
            auto nib = [](unsigned int w) { return ((w & LOW) * 0x01020408u) >> 24; };
            const unsigned int h = nib(v[u].x) | nib(v[u].y) << 4 | nib(v[u].z) << 8 | nib(v[u].w) << 12;
            m |= (unsigned long long)h << (16 * u);
        }
        return m;
    };
    // Small flag arrays are spread over more threads -- 1, 4 or 16 flags each instead of 64 -- because the
    // ranking walks a thread's set bits one by one.  (Then gpt == 1.)
    const int fpt = g.n_sub <= CONV_THREADS ? 1 : g.n_sub <= 4 * CONV_THREADS ? 4 : g.n_sub <= 16 * CONV_THREADS ? 16 : 64;
    auto nib = [](unsigned int w) { return ((w & LOW) * 0x01020408u) >> 24; };  // byte flags of a word -> 4 bits
    // The k-th 64-flag mask of (producer) thread t's share of the flag array, and the sub-tile of its bit 0.
    auto thread_mask = [&](int t, int k, int& id0) -> unsigned long long {
        if (fpt == 1) {
            id0 = t;
            return t < g.n_sub ? (unsigned long long)(reinterpret_cast<const unsigned char*>(flags)[t] & 1u) : 0ull;
        }
        if (fpt == 4) {
            id0 = 4 * t;
            return t < g.n_words ? (unsigned long long)nib(flags[t]) : 0ull;
        }
        if (fpt == 16) {
            id0 = 16 * t;
            if (t >= n_vec) return 0ull;
            const uint4 v = fvp[t];
            return (unsigned long long)(nib(v.x) | nib(v.y) << 4 | nib(v.z) << 8 | nib(v.w) << 12);
        }
        const int gi = t * gpt + k;
        id0 = 64 * gi;
        return gi < n_grp ? load_group(gi) : 0ull;
    };
    const int masks_per_thread = fpt == 64 ? gpt : 1;
    int count, mine = 0;
    // Few sub-tiles in all (one stream of a small map: at most 256, and every group of nt consecutive sub-tiles
    // has a workgroup of its own in the grid): the launch is latency bound, so there is no global list.  A workgroup reads
    // the flags of its own group only, compacts them with one ballot, and is done after one barrier.
    const bool own_group = MODE == MODE_DELTA && g.n_sub <= GX * g.nt && g.n_sub <= CONV_THREADS;
    if (own_group) {
        if (wave == 0) {
            const int id = BX * g.nt + lane;
            const bool f = lane < g.nt && id < g.n_sub && (reinterpret_cast<const unsigned char*>(flags)[id] & 1u);
            const unsigned long long m = __ballot(f);
            if (f) s_list[__popcll(m & ((1ull << lane) - 1ull))] = id;
            if (lane < 4) s_scan[lane] = lane == 0 ? (int)__popcll(m) : 0;
        }
        lds_barrier();
        count = s_scan[0];
    } else if (MODE == MODE_DELTA) {
        if (producer) {
            // (four masks at a time: their loads are in flight together)
            for (int k0 = 0; k0 < masks_per_thread; k0 += 4) {
                unsigned long long m[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    int id0;
                    m[k] = k0 + k < masks_per_thread ? thread_mask(tid, k0 + k, id0) : 0ull;
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) mine += __popcll(m[k]);
            }
            // popcount prefix sum (every workgroup does the same small scan)
            int incl = mine;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_up(incl, o);
                if (lane >= o) incl += t;
            }
            if (lane == 63) s_scan[wave] = incl;
            s_excl[tid] = incl - mine;  // set flags before this thread's, within its wavefront
        }
        lds_barrier();
        count = s_scan[0] + s_scan[1] + s_scan[2] + s_scan[3];
    } else {
        count = g.n_sub;
    }
    // Above a density of active sub-tiles where reading and re-writing the stored projection costs more than
    // recomputing it, a delta launch recomputes everything instead (Eq. 3): all sub-tiles, the committed
    // input x_t (the scan has made the snapshot equal to it) as the source, one term, accumulators from the
    // bias.  The switch is the same in every workgroup (same count).
    const int n_flagged = count;
    const bool full = MODE == MODE_DELTA && !own_group && g.xfull != nullptr &&
                      (long long)count * 100 > (long long)g.n_sub * g.full_pct;
    if (full) count = g.n_sub;
    const bool listed = MODE == MODE_DELTA && !full;  // sub-tile ids come from the ranked list (else: all, in order)
    const bool from_y = listed;                        // accumulators start from the stored projection (else: bias)
    // The active sub-tiles are cut into work units of `per` sub-tiles: few sub-tiles are spread thinly (a
    // unit's latency grows with its size), many are packed NT per unit (operand reuse).
    // (a workgroup with a sub-tile group of its own: one unit, the group's active sub-tiles)
    const int gx = own_group ? 1 : GX;
    const int bx = own_group ? 0 : BX;
    // (several units per workgroup: as many as full-size units would need, but of equal size, so that the
    // last pass over the grid is not a nearly empty one of full-size units)
    const int passes = max(1, (count + gx * g.nt - 1) / (gx * g.nt));
    int per = (count + gx * passes - 1) / (gx * passes);
    if (per < 1) per = 1;
    if (per > g.nt) per = g.nt;
    const int nunits = (count + per - 1) / per;

    unsigned int arrived_before = 0;  // thread 0: workgroups that signalled before this one
    // Arrival signal, sent once this workgroup has read the flags for the last time.  Every thread has
    // consumed its flag loads before a barrier by then and this workgroup's stores do not touch the flags,
    // so no memory fence is needed (a device-scope fence would write back the whole L2).  The answer is
    // needed only at the end.  (Dense launches have no flags and no signal.)
    auto arrive = [&]() {
        if (MODE == MODE_DELTA && tid == 0) arrived_before = atomicAdd(&ctrl[0], 1u);
    };
    // The last workgroup to arrive knows that every workgroup has read the flags: it clears them (and
    // the arrival counter) for the next step, at its own end, off everybody's critical path.
    auto retire = [&]() {
        if (MODE != MODE_DELTA) return;
        if (tid == 0) s_last = (arrived_before == (unsigned int)(GX * GY) - 1u) ? 1 : 0;
        __syncthreads();
        if (s_last) {
            for (int w = tid; w < g.n_words; w += WG_THREADS) {
                if (g.touched) g.touched[w] = full ? LOW : flags[w];  // what this step wrote in y, for an incremental nonlinearity
                flags[w] = 0u;
            }
            if (tid == 0) {
                ctrl[0] = 0u;
                if (g.fresh) g.fresh[0] = 0u;  // the stored input now holds this step's input
                if (g.touched_all) g.touched_all[0] = 0u;  // `touched` describes this step
                if (n_flagged && !own_group) atomicAdd(&stats[0].active_tiles, (unsigned long long)n_flagged);
            }
        }
        // (each workgroup counted only its own group's flags)
        if (own_group && tid == 0 && n_flagged && BY == 0)
            atomicAdd(&stats[(unsigned int)BX & (STAT_SLOTS - 1)].active_tiles, (unsigned long long)n_flagged);
    };
    if (bx >= nunits) {
        __builtin_amdgcn_s_waitcnt(0);  // let the early weight copy land before the LDS is released
        arrive();
        retire();
        return;
    }
    // this workgroup's units: BX + i*gx, i = 0 .. my_nunits-1, ranked in rounds of `ur` units
    const int my_nunits = (nunits - bx + gx - 1) / gx;
    const int ur = LIST_CAP / per;

    // lane roles of a consumer: position j of sub-tile `half` of a pair (MFMA column l%32), K pair `khalf` of
    // an MFMA step; of the result it holds channels 8*gq + 4*khalf + (0..3), gq = 0..3, of each 32-channel block
    const int j = lane & 15, half = (lane >> 4) & 1, khalf = lane >> 5;
    // lane-constant window position of its output position (tap 0,0)
    const int off_lane = (((j >> 2) * g.str_y) * g.ww + (j & 3) * g.str_x) * g.sc * 16;
    const int rot_lane = g.rot_a * (j >> 2) + g.rot_b * (j & 3);  // this position's share of the chunk rotation
    sc_t* y = static_cast<sc_t*>(y_v);
    const sc_t* bias = static_cast<const sc_t*>(bias_v);
    // channel (within the filter group) of register 4*gq of block c; the 4 registers are 4 consecutive channels
    auto chan = [&](int c, int gq) { return (cbg * NCB + c) * 32 + 8 * gq + 4 * khalf; };
    const unsigned int slab_src_bytes = (unsigned int)(g.sc * 16);  // source bytes between consecutive slabs

    int gs = 0;  // stages (slabs) done so far: the window buffer, and the weight buffer if there are two, alternate

    // The two roles run the same loops (ranking rounds, units, slabs) and meet at the same barriers, but
    // each in its own copy of the loops: what one role keeps in registers across iterations is not live
    // in the other's code.
    if (producer) {
    for (int r0 = 0; r0 < my_nunits; r0 += ur) {
    const int r1 = min(r0 + ur, my_nunits);
    // ---- ranking round: the sub-tile ids of units r0 .. r1-1 of this workgroup go to s_list ------------
    if (MODE == MODE_DELTA) {
        if (r0 > 0) __syncthreads();  // the previous round's list is no longer in use
        if (listed && !own_group) {  // (own_group: the list was made with the count)
            // The rank of a set flag is the number of set flags before it; this workgroup owns the ranks
            // unit*per .. unit*per + per - 1 of its units BX + i*gx, i = r0 .. r1-1.  Every producer
            // thread looks its share of those ranks up: which thread's flags hold the rank (binary search in
            // the prefix counts), then which of that thread's set bits it is.  Nobody walks a long run of bits.
            const int n_owned = (r1 - r0) * per;
            for (int jj = tid; jj < n_owned; jj += CONV_THREADS) {
                const int iu = jj / per, kk = jj - iu * per;
                const int t = (bx + (r0 + iu) * gx) * per + kk;  // the rank
                if (t >= count) continue;
                int w = 0, lt = t;  // wavefront holding the rank, rank within it
                while (lt >= s_scan[w]) lt -= s_scan[w++];
                int lo = 0, hi = WAVE - 1;  // last thread of the wavefront with s_excl <= lt
                while (lo < hi) {
                    const int mid = (lo + hi + 1) >> 1;
                    if (s_excl[w * WAVE + mid] <= lt) lo = mid;
                    else hi = mid - 1;
                }
                const int owner = w * WAVE + lo;
                int lr = lt - s_excl[owner];  // rank among the owner's flags
                int id = -1;
                for (int k0 = 0; k0 < masks_per_thread && id < 0; k0 += 4) {
                    unsigned long long m[4];
                    int id0[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        id0[k] = 0;
                        m[k] = k0 + k < masks_per_thread ? thread_mask(owner, k0 + k, id0[k]) : 0ull;
                    }
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const int pc = (int)__popcll(m[k]);
                        if (id < 0 && lr < pc) {
                            unsigned long long mm = m[k];
                            while (lr-- > 0) mm &= mm - 1;  // drop the lr lowest set bits
                            id = id0[k] + __ffsll((long long)mm) - 1;
                        } else if (id < 0) {
                            lr -= pc;
                        }
                    }
                }
                s_list[jj] = id;
            }
        }
        if (r0 == 0) early_loads();
        lds_barrier();  // the list is published
    } else if (r0 == 0) {
        lds_barrier();  // (the K-pair table is published)
    }


    for (int iu = r0; iu < r1; ++iu) {
    const int unit = bx + iu * gx;
    const int first = unit * per;
    int mycount = count - first;
    if (mycount > per) mycount = per;
    {
        // ---- window origins of the unit's sub-tiles (each producer wavefront keeps its own copy: no barrier) --
        if (lane < mycount) {
            const int id = listed ? s_list[(iu - r0) * per + lane] : first + lane;
            const int b = (int)udiv_magic((unsigned int)id, (unsigned int)(g.sty * g.stx), g.magic_sub);
            const int r = id - b * (g.sty * g.stx);
            const int sy = (int)udiv_magic((unsigned int)r, (unsigned int)g.stx, g.magic_stx), sx = r - sy * g.stx;
            const int iy0 = 4 * sy * g.str_y - g.pad_y, ix0 = 4 * sx * g.str_x - g.pad_x;
            s_iy0[wave][lane] = iy0;
            s_ix0[wave][lane] = ix0;
            s_base[wave][lane] = (unsigned int)((b * g.src_h + iy0) * g.src_w + ix0) * (unsigned int)g.pos_bytes +
                                 (unsigned int)(grp * g.grp_bytes);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // LDS operations of one wavefront execute in order
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---- window staging ----------------------------------------------------------------------------
        // A staged unit is 16 bytes of one (sub-tile, window position, chunk-in-slab).  Unit v lives at LDS
        // byte 16*v of its plane, v = (slot*wpos + hp)*sc + cs, where slot cs of a position holds chunk
        // (cs - rotation(position)) mod rot_p, so that the MFMA operand reads of a sub-tile's 16 positions
        // fall into different banks.  Consecutive lanes own consecutive units, which is what the LDS-direct
        // gather (per-lane global address, LDS address = wave base + 16*lane) needs.  The decomposition
        // does not depend on the slab or on the sub-tiles, so it comes from a table made at create time; a
        // thread adds the window origins of its units' sub-tiles once per work unit, and a slab only adds
        // its channel offset.  Units outside the image, or whose chunk does not exist in the last slab,
        // read a 16-byte block of zeros instead.
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
                const int iy = s_iy0[wave][slot] + hy, ix = s_ix0[wave][slot] + hx;
                ulast |= (unsigned int)((u.x >> 21) & 1) << i;
                if (iy >= 0 && iy < g.src_h && ix >= 0 && ix < g.src_w) uoff[i] = s_base[wave][slot] + (unsigned int)u.y;
            }
        }
        // the flags were read for the last time in the last ranking round (the signal is sent where no load
        // of the issuing thread is waited for soon: returns are in order, a wait would include the atomic)
        if (iu == r0 && r1 == my_nunits) arrive();
        auto stage_windows = [&](int slab, int buf) {
            unsigned char* dst = bbase + buf * b_bytes;
            const bool last = slab == g.nslab - 1;
#pragma unroll
            for (int i = 0; i < MAXU; ++i) {
                if (i >= my_units) break;
                const bool real = uoff[i] != 0xFFFFFFFFu && !(last && ((ulast >> i) & 1u));
                const unsigned int o = uoff[i] + (unsigned int)slab * slab_src_bytes;
                unsigned char* d = dst + (i * CONV_THREADS + wave * 64) * 16;  // wave-uniform; lane adds 16*lane
                const unsigned char* p0 = real ? (full ? g.xfull : src0) + o : zero16;
                __builtin_amdgcn_global_load_lds((gptr_t)p0, (lptr_t)d, 16, 0, 0);
                if (TERMS == 2 && !full) {
                    const unsigned char* p1 = real ? src1 + o : zero16;
                    __builtin_amdgcn_global_load_lds((gptr_t)p1, (lptr_t)(d + plane_bytes), 16, 0, 0);
                }
            }
        };
        // Stage by stage: slab k of this unit goes into the buffers of parity gs + k.  Slab 0 is staged
        // while the consumers still multiply the previous unit's last slab (other parity).
        if (nbuf_a == 2 && iu > 0) stage_weights(0, gs & 1);  // (the very first slab was started at kernel entry)
        stage_windows(0, gs & 1);
        for (int k = 0; k < g.nslab; ++k) {
            __builtin_amdgcn_s_waitcnt(0);  // this wavefront's copies for slab k have landed in LDS
            __syncthreads();                // slab k is published; the consumers are done with slab k-1
            ++gs;
            if (k + 1 < g.nslab) {
                stage_weights(k + 1, gs & 1);
                stage_windows(k + 1, gs & 1);
            }
        }
    }
    }  // units of the round
    }  // rounds
    } else {
    // Consumer state of a unit: output addresses (per pair, this lane's position of its sub-tile) and the
    // accumulators.  The accumulators start from what the result is added to -- the stored projection (delta:
    // Algorithm 1, P_t = P_{t-1} + F * dI) or the bias (dense: Eq. 3) -- so the epilogue is a plain store.
    // They are fetched as soon as the previous unit's results are stored (the sub-tile ids come from the
    // ranked list, not from the producers), long before the unit's first slab is staged.  (Channel counts
    // that are not multiples of 4 start from zero and add element by element at the end.)
    unsigned int ybase[NP];
    bool pos_ok[NP];
    acc_t acc[NCB][NP];
    auto begin_unit = [&](int iu2, int r0) {
        const int first2 = (bx + iu2 * gx) * per;
        const int mycount2 = min(per, count - first2);
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int slot = 2 * (cw + 4 * p) + half;
            pos_ok[p] = false;
            ybase[p] = 0;
            if (slot < mycount2) {
                const int id = listed ? s_list[(iu2 - r0) * per + slot] : first2 + slot;
                const int b = (int)udiv_magic((unsigned int)id, (unsigned int)(g.sty * g.stx), g.magic_sub);
                const int r = id - b * (g.sty * g.stx);
                const int sy = (int)udiv_magic((unsigned int)r, (unsigned int)g.stx, g.magic_stx), sx = r - sy * g.stx;
                const int oy = 4 * sy + (j >> 2), ox = 4 * sx + (j & 3);
                pos_ok[p] = ox < g.wo && oy < g.ho;
                ybase[p] = (unsigned int)((b * g.ho + oy) * g.wo + ox) * (unsigned int)g.c_out + (unsigned int)(grp * g.og);
            }
        }
#pragma unroll
        for (int c = 0; c < NCB; ++c)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int co = chan(c, gq);
                const bool ch_ok = g.vec_store && co < g.og;
                vec_t bv = vec_t{0, 0, 0, 0};
                if (!from_y && ch_ok && bias) bv = *reinterpret_cast<const vec_t*>(bias + grp * g.og + co);
#pragma unroll
                for (int p = 0; p < NP; ++p) {
                    vec_t v = bv;
                    if (from_y && ch_ok && pos_ok[p])
                        v = *reinterpret_cast<const vec_t*>(y + (ybase[p] + (unsigned int)co));
                    acc[c][p][4 * gq + 0] = v.x;
                    acc[c][p][4 * gq + 1] = v.y;
                    acc[c][p][4 * gq + 2] = v.z;
                    acc[c][p][4 * gq + 3] = v.w;
                }
            }
    };
    for (int r0 = 0; r0 < my_nunits; r0 += ur) {
    const int r1 = min(r0 + ur, my_nunits);
    // the barriers of the ranking round
    if (MODE == MODE_DELTA) {
        if (r0 > 0) __syncthreads();
        lds_barrier();
    } else if (r0 == 0) {
        lds_barrier();
    }
    begin_unit(r0, r0);
    for (int iu = r0; iu < r1; ++iu) {
    const int unit = bx + iu * gx;
    const int first = unit * per;
    int mycount = count - first;
    if (mycount > per) mycount = per;
    const int nact = mycount > 2 * cw ? (mycount - 2 * cw + 7) / 8 : 0;  // pairs in use (slots 2*(cw+4p), +1)
    {
        // ---- consumers ---------------------------------------------------------------------------------
        // K loop of one slab, compiled per number of sub-tile pairs in use by the wavefront (no per-pair
        // branches; unused slots read stale LDS and their results are dropped).  A K step is four K pairs,
        // i.e. two MFMA steps.  Software pipeline: while K step q multiplies, the operands of step q+1 are
        // read from LDS into a second register set (the sets swap roles every step, nothing is copied) and
        // the table entries of step q+2 are fetched, so that no address waits for a table read.  The reads
        // are issued one by one between the MFMAs: a wavefront that issues them in a batch leaves the
        // matrix pipeline idle meanwhile.
        auto k_loop = [&]<int NPA, int T>(const unsigned char* aw, const unsigned char* bw) {  // T: terms multiplied
            const unsigned char* ap = aw + lane * 16;
            // (slots beyond the allocated ones are never in use; their lanes read slot 0 instead of running
            // off the buffer)
            const unsigned char* bp = bw + (2 * cw + half < g.nt ? 2 * cw + half : 0) * g.slot_bytes;
            const int pstride = NPA > 1 ? 8 * g.slot_bytes : 0;
            const int2* tp = tab + khalf;
            constexpr int NB1 = T == 2 ? NPA : 1;
            struct Ops {
                uint4 a[2][NCB], b0[2][NPA], b1[2][NB1];
            };
            constexpr int N_MFMA = 2 * NCB * NPA * T;
            constexpr int N_READ = 2 * (NCB + NPA * T);
            auto load_tab = [&](int q, int2(&t)[2]) {
                t[0] = tp[4 * q];  // tap's byte offset; rotated chunk | mask << 8
                t[1] = tp[4 * q + 2];
            };
            auto fetch = [&](int q, const int2(&t)[2], Ops& o) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int off = off_lane + t[h].x + ((((t[h].y & 0xFF) + rot_lane) & (t[h].y >> 8)) << 4);
#pragma unroll
                    for (int c = 0; c < NCB; ++c)
                        o.a[h][c] = *reinterpret_cast<const uint4*>(ap + (c * nq2 + 2 * q + h) * 1024);
#pragma unroll
                    for (int p = 0; p < NPA; ++p) {
                        o.b0[h][p] = *reinterpret_cast<const uint4*>(bp + off + p * pstride);
                        if (T == 2) o.b1[h][p] = *reinterpret_cast<const uint4*>(bp + plane_bytes + off + p * pstride);
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
                            if (T == 2) acc[c][p] = mma(o.a[h][c], o.b1[h][p], acc[c][p]);
                        }
            };
            // one K step: multiply `cur`, read step q1 (table entries `t`) into `nxt`, fetch the table entries
            // of step q2 into `tn`; operand sets and table registers swap roles every step, nothing is copied
            auto step = [&](const Ops& cur, Ops& nxt, const int2(&t)[2], int2(&tn)[2], int q1, int q2) {
                load_tab(q2, tn);
                fetch(q1, t, nxt);
                multiply(cur);
                // issue order: the table read, then MFMAs with the operand reads spread between them
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                sched_interleave<0, N_MFMA, N_READ>();
            };
            Ops o0, o1;
            int2 ta[2], tb[2];
            const int qmax = g.nq - 1;
            load_tab(0, tb);
            fetch(0, tb, o0);
            load_tab(min(1, qmax), ta);
            for (int q = 0; q < g.nq; q += 2) {
                step(o0, o1, ta, tb, min(q + 1, qmax), min(q + 2, qmax));
                if (q + 1 < g.nq) step(o1, o0, tb, ta, min(q + 2, qmax), min(q + 3, qmax));
            }
        };

        for (int k = 0; k < g.nslab; ++k) {
            // slab k is staged.  A bare barrier: the producers waited for their copies before they arrived,
            // and this wavefront's own stores and loads of stored projections (previous / this unit) need not
            // have completed -- __syncthreads() would wait for all of them.
            asm volatile("s_barrier" ::: "memory");
            const unsigned char* aw = lds + (nbuf_a == 2 ? (gs & 1) : 0) * a_bytes;
            const unsigned char* bw = bbase + (gs & 1) * b_bytes;
            ++gs;
            if (TERMS == 2 && !full) {
                if (nact > 1) {
                    if constexpr (NP >= 2 && TERMS == 2) k_loop.template operator()<2, 2>(aw, bw);
                } else if (nact > 0) {
                    if constexpr (TERMS == 2) k_loop.template operator()<1, 2>(aw, bw);
                }
            } else if (nact > 1) {
                if constexpr (NP >= 2) k_loop.template operator()<2, 1>(aw, bw);
            } else if (nact > 0) {
                k_loop.template operator()<1, 1>(aw, bw);
            }
        }

        // ---- epilogue ----------------------------------------------------------------------------------
        // (the store addresses are rebuilt from ybase here: kept across the K loops they would cost two
        // registers per store)
#pragma unroll
        for (int p = 0; p < NP; ++p) asm volatile("" : "+v"(ybase[p]));
        // The MFMA layout gives a lane 4 consecutive channels of ONE position, so a store instruction writes
        // 32-byte pieces of 32 different rows of y; measured, read-modify-writing an output tile that way runs at
        // 5.9 TB/s against 8 TB/s when the stores are whole 128-byte rows.  So each result block (32 positions x
        // 32 channels) is turned through LDS first: written in the MFMA layout, read back with 8 lanes along the
        // channels of a position, 8 positions per store.  The scratch is the window area of this wavefront's own
        // first two slots in the buffer of the slab just finished: only this wavefront reads those windows, and
        // the producers are filling the other buffer.
        constexpr int RP = 36;  // words per position row of the scratch (16-byte aligned, spreads the banks)
        if (g.vec_store && g.nt >= 8 && 2 * g.slot_bytes >= 32 * RP * 4) {
            vec_t* scr = reinterpret_cast<vec_t*>(bbase + ((gs - 1) & 1) * b_bytes + (2 * cw) * g.slot_bytes);
            const int posl = lane & 31;
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                // the two sub-tiles of the pair (the same in every lane)
                unsigned int corner[2];
                int ny[2], nx[2];
#pragma unroll
                for (int sl = 0; sl < 2; ++sl) {
                    const int slot = 2 * (cw + 4 * p) + sl;
                    corner[sl] = 0;
                    ny[sl] = nx[sl] = 0;
                    if (slot < mycount) {
                        const int id = listed ? s_list[(iu - r0) * per + slot] : first + slot;
                        const int b = (int)udiv_magic((unsigned int)id, (unsigned int)(g.sty * g.stx), g.magic_sub);
                        const int r = id - b * (g.sty * g.stx);
                        const int sy = (int)udiv_magic((unsigned int)r, (unsigned int)g.stx, g.magic_stx), sx = r - sy * g.stx;
                        ny[sl] = g.ho - 4 * sy;
                        nx[sl] = g.wo - 4 * sx;
                        corner[sl] = (unsigned int)((b * g.ho + 4 * sy) * g.wo + 4 * sx) * (unsigned int)g.c_out +
                                     (unsigned int)(grp * g.og);
                    }
                }
#pragma unroll
                for (int c = 0; c < NCB; ++c) {
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // (the previous block's reads are done)
#pragma unroll
                    for (int gq = 0; gq < 4; ++gq) {
                        vec_t o;
                        o.x = acc[c][p][4 * gq + 0];
                        o.y = acc[c][p][4 * gq + 1];
                        o.z = acc[c][p][4 * gq + 2];
                        o.w = acc[c][p][4 * gq + 3];
                        scr[(posl * RP + 8 * gq + 4 * khalf) >> 2] = o;
                    }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // LDS operations of a wavefront execute in order
                    __builtin_amdgcn_wave_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                    const int ch = (cbg * NCB + c) * 32 + 4 * (lane & 7);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int q = 8 * i + (lane >> 3);  // position of the pair: sub-tile q / 16, position q % 16
                        const vec_t o = scr[(q * RP + 4 * (lane & 7)) >> 2];
                        const int sl = i >> 1, py = 2 * (i & 1) + (lane >> 5), px = (lane >> 3) & 3;
                        if (py < ny[sl] && px < nx[sl] && ch < g.og)
                            *reinterpret_cast<vec_t*>(y + (corner[sl] + (unsigned int)((py * g.wo + px) * g.c_out + ch))) = o;
                    }
                }
            }
        } else if (g.vec_store) {
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
                            if (from_y) {
                                if (r != (sc_t)0) yp4[k] += r;
                            } else {
                                yp4[k] = r + (bias ? bias[grp * g.og + co0 + k] : (sc_t)0);
                            }
                        }
                    }
                }
        }
        if (iu + 1 < r1) begin_unit(iu + 1, r0);  // (a new round's first unit waits for its ranking)
    }
    }  // units of the round
    }  // rounds
    }
    retire();
}

template <int DT, int MODE, int NCB, int NT, int TERMS>
hipError_t launch_one(const void* src0, const void* src1, const void* zero16, unsigned int* flags,
                      unsigned int* ctrl, const void* wpack, const int* offtab, const void* bias, void* y,
                      const ConvGeom& g, DevStats* stats, hipStream_t s) {
    const int ncbg = (g.ncb + NCB - 1) / NCB;
    const size_t lds = conv_lds_bytes(g, NCB, g.nt, TERMS);
    // no more workgroups than are resident at once (the kernel loops over its work units)
    const int gy = g.groups * ncbg;
    const int resident = NUM_CU;  // eight wavefronts with up to 256 registers each fill a compute unit
    int gx = std::min((g.n_sub + g.nt - 1) / g.nt, std::max(1, resident / gy));
    dim3 grid((unsigned int)gx, (unsigned int)gy);
    // A full grid (more units than lanes): one-dimensional, with the channel-block groups of a lane on one XCD
    // (see the kernel).
    ConvGeom gg = g;
    gg.xcd_gy = 0;
    if (gx >= 8 && gx == resident / gy) {
        grid = dim3((unsigned int)(gx * gy), 1u);
        gg.xcd_gy = gy;
    }
    auto kern = conv_gather_kernel<DT, MODE, NCB, NT, TERMS>;
    if (lds > 64 * 1024) {
        // one per instantiation, shared by every handle and thread of the process: guarded, so that
        // distinct handles stay independent
        static std::mutex mu;
        static size_t granted = 0;
        std::lock_guard<std::mutex> lock(mu);
        if (lds > granted) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            granted = lds;
        }
    }
    hipLaunchKernelGGL(kern, grid, dim3(WG_THREADS), lds, s, static_cast<const unsigned char*>(src0),
                       static_cast<const unsigned char*>(src1), static_cast<const unsigned char*>(zero16), flags, ctrl,
                       static_cast<const uint4*>(wpack), offtab, bias, y, gg, stats);
    return hipGetLastError();
}

template <int DT, int MODE, int TERMS>
hipError_t launch_shape(int ncb, int nt, const void* src0, const void* src1, const void* zero16,
                        unsigned int* flags, unsigned int* ctrl, const void* wpack, const int* offtab, const void* bias, void* y,
                        const ConvGeom& g, DevStats* stats, hipStream_t s) {
#define RRM_CASE(CBV, NTV)                                                                                          \
    if (ncb == CBV && nt == NTV)                                                                                     \
        return launch_one<DT, MODE, CBV, NTV, TERMS>(src0, src1, zero16, flags, ctrl, wpack, offtab, bias, y, g, stats, s);
    if (nt < 8) nt = 8;  // fewer slots than the smallest shape: same code, the slot count is in g.nt
    RRM_CASE(2, 16) RRM_CASE(2, 8) RRM_CASE(1, 16) RRM_CASE(1, 8)
#undef RRM_CASE
    return hipErrorInvalidValue;
}

}  // namespace

size_t conv_lds_bytes(const ConvGeom& g, int ncb, int nt, int terms) {
    return (size_t)(g.nslab > 1 ? 2 : 1) * (size_t)ncb * 2 * g.nq * 1024 + 2 * (size_t)terms * nt * g.slot_bytes +
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
