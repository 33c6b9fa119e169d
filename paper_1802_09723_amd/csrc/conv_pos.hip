// Position-gather implicit-GEMM convolution on the gfx950 matrix cores (int8 -> int32, bf16 -> fp32), for
// stride-1 layers whose channel runs are 16-byte multiples.
//
// Delta mode computes the second term of Eq. 5, F * (I_t - I_{t-1}), only at the output positions whose
// receptive field holds a changed input, and adds it in place into the stored projection (Algorithm 1:
// P_t = P_{t-1} + F * dI).  Dense mode computes Eq. 3, y = b + F * x, everywhere.  The cost of a delta step is
// proportional to the number of such output positions (Table 1 / Eq. 6 at the granularity a matrix instruction
// allows: one output position = one column of the product, 16 channels of one input position = one K chunk).
//
// Unit of work: a band of R output rows of G consecutive streams, times one block of 128 output channels.
//   * The band's input rows (R + kh - 1 of them, halo included) of the difference buffer are copied into LDS
//     once per K slab (32 bytes of channels per position) with LDS-direct loads, in the global row order with a
//     row pitch of w + pad positions: the zeros left of row r + 1 double as the zeros right of row r, rows and
//     columns outside the image are copies of a block of zeros.  Nothing is gathered: a tap is a constant offset.
//   * The scan leaves a bitmap of changed 16-byte input units.  The workgroup turns the bitmap bits of its band
//     into one flag per input position, dilates them by the filter window into one flag per output position, and
//     compacts the active output positions with ballots into a column list (LDS).  The flags of the output
//     positions are also written out for the next layer ("touched"); every position is written by exactly one
//     workgroup in every step, so nothing has to be cleared.
//   * The columns are multiplied 32 at a time: v_mfma_i32_32x32x32_i8 / v_mfma_f32_32x32x16_bf16 with M = 32
//     output channels, N = 32 gathered positions, K = 2 chunks of one tap.  A consumer wavefront owns 4 channel
//     blocks x 2 column tiles (one weight fragment feeds 2 products, one window fragment 4), the four consumers of
//     a workgroup 256 columns; longer lists take several passes.  Weights are packed at create time in per-lane
//     fragment order, one contiguous run per (slab, tap group), double-buffered in LDS like the bands.
//   * The accumulators start from the stored projection (delta) or the bias (dense) and are stored back: one owner
//     per output element, no atomics, results reproducible run to run.
// A workgroup has eight wavefronts in two roles (see the kernel): four only copy into LDS, one stage ahead, four
// only multiply; the roles meet at one barrier per stage.  Work units are handed out by an atomic counter (their
// cost varies with the number of active columns); the last workgroup to leave rearms the counters, so a step
// needs no host-side state and can be replayed in a HIP graph.
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

template <int I, int N_MFMA, int N_READ>
__device__ __forceinline__ void sched_interleave() {
    if constexpr (I < N_MFMA) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
        constexpr int R = (N_READ * (I + 1)) / N_MFMA - (N_READ * I) / N_MFMA;
        if constexpr (R > 0) __builtin_amdgcn_sched_group_barrier(0x100, R, 0);  // R LDS reads
        sched_interleave<I + 1, N_MFMA, N_READ>();
    }
}

typedef const void __attribute__((address_space(1))) * gptr_t;
typedef void __attribute__((address_space(3))) * lptr_t;

constexpr int PT = POS_THREADS;
constexpr int PP = POS_PROD;
constexpr int NCB = POS_NCB;

template <int DT, int MODE, int TERMS>
__global__ __launch_bounds__(PT) void conv_pos_kernel(const unsigned char* __restrict__ src0,
                                                      const unsigned char* __restrict__ src1,
                                                      const unsigned char* __restrict__ zero16,
                                                      const unsigned long long* __restrict__ bitmap,
                                                      unsigned int* ctrl, const unsigned char* __restrict__ wpack,
                                                      const void* __restrict__ bias_v, void* y_v, PosGeom g,
                                                      DevStats* __restrict__ stats) {
    typedef typename Acc<DT>::type acc_t;
    typedef typename Acc<DT>::vec vec_t;
    typedef typename Acc<DT>::scalar sc_t;
    constexpr int NP = 2;  // column tiles per consumer wavefront and pass

    // LDS: [weights x 2][bands (TERMS planes) x 2][input-position flags][column list: band position, y position]
    extern __shared__ uint4 smem[];
    unsigned char* lds = reinterpret_cast<unsigned char*>(smem);
    const int a_bytes = g.a_stage_bytes;
    const int plane = g.b_plane_bytes;
    const int b_bytes = TERMS * plane;
    unsigned char* abase = lds;
    unsigned char* bbase = lds + POS_ABUF * a_bytes;
    unsigned char* in_act = bbase + 2 * b_bytes;
    unsigned short* s_colq = reinterpret_cast<unsigned short*>(in_act + g.act_bytes);
    unsigned int* s_coly = reinterpret_cast<unsigned int*>(s_colq + g.col_cap);
    __shared__ int s_cnt[POS_MAXO][PT / 64];
    __shared__ int s_next;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Two roles.  Wavefronts 0-3 ("consumers", one per SIMD) only multiply and write results; wavefronts 4-7
    // ("producers") only copy weights and bands into LDS.  An LDS-direct copy occupies its wavefront's issue slot
    // for a hundred cycles or more; issued by a wavefront of its own it runs in the shadow of the matrix
    // instructions of the consumer on the same SIMD instead of delaying them.
    const bool producer = wave >= 4;
    const int ptid = tid - PP;  // producer thread index
    const int khalf = lane >> 5;
    sc_t* y = static_cast<sc_t*>(y_v);
    const sc_t* bias = static_cast<const sc_t*>(bias_v);

    // Slots of a thread (the same decomposition for every unit, divided out again per unit: a handful of divisions
    // against a unit's thousands of matrix instructions):
    //   staged unit v = ptid + PP*i of a producer thread: 16 bytes (chunk v & 1 of the slab) of band position
    //     q = v >> 1, q = (stream * RB + row) * WP + column (column < pad: the zeros between rows);
    //   output position lo = tid + PT*i of a unit: (stream * R + row) * wo + column.
    const int band_pos = g.G * g.RB * g.WP;
    const int upos = g.pos_bytes >> 4;  // bitmap bits (16-byte units) per input position

    unsigned int nxt_pending = 0;
    int unit = blockIdx.x;
    while (unit < g.total_units) {
        // the next unit's number is asked for now and needed at the end of this one
        if (tid == 0) nxt_pending = atomicAdd(&ctrl[2], 1u);
        int u = unit;
        const int cgrp = u % g.ncg;
        u /= g.ncg;
        const int grp = u % g.groups;
        u /= g.groups;
        const int band = u % g.nbands;
        const int sgi = u / g.nbands;
        const int r0 = band * g.R, b0 = sgi * g.G;
        const int rows_here = min(g.R, g.ho - r0);
        const bool flag_owner = grp == 0 && cgrp == 0;

        // ---- flags of the band's input positions (all threads); source offsets of the producers' units ---------
        if (MODE == MODE_DELTA) {
            for (int q = tid; q < g.npos; q += PT) {
                const int gg = q / (g.RB * g.WP), rem = q - gg * (g.RB * g.WP);
                const int row = rem / g.WP, col = rem - row * g.WP;
                const int b = b0 + gg, iy = r0 - g.pad + row;
                unsigned char f = 0;
                if (q < band_pos && col >= g.pad && b < g.n && iy >= 0 && iy < g.h) {
                    // any changed 16-byte unit among this position's?
                    const unsigned int p = (unsigned int)((b * g.h + iy) * g.w + col - g.pad);
                    const unsigned int lo = p * (unsigned int)upos, hi = lo + (unsigned int)upos;
                    for (unsigned int wd = lo >> 6; wd <= (hi - 1u) >> 6; ++wd) {
                        unsigned long long m = bitmap[wd];
                        if (wd == lo >> 6) m &= ~0ull << (lo & 63u);
                        if (wd == (hi - 1u) >> 6 && (hi & 63u)) m &= ~0ull >> (64u - (hi & 63u));
                        if (m) f = 1;
                    }
                }
                in_act[q] = f;
            }
        }
        unsigned int uoff[POS_MAXU];  // producers: byte offset at slab 0, 0xFFFFFFFF = zeros
        unsigned int odd_chunk = 0;   // bit i: unit i holds the slab's second chunk
        if (producer) {
#pragma unroll
            for (int i = 0; i < POS_MAXU; ++i) {
                const int q0 = (ptid + PP * i) >> 1;
                const int gg = q0 / (g.RB * g.WP), rem = q0 - gg * (g.RB * g.WP);
                const int row = rem / g.WP, col = rem - row * g.WP;
                const int b = b0 + gg, iy = r0 - g.pad + row;
                const bool ok = q0 < band_pos && col >= g.pad && b < g.n && iy >= 0 && iy < g.h;
                const unsigned int p = (unsigned int)((b * g.h + iy) * g.w + col - g.pad);
                // (the two chunks of a position swap places with bits 2 and 3 of the position index: the operand
                // reads of consecutive positions then fall into different LDS banks)
                const unsigned int chunk = (unsigned int)((ptid ^ (q0 >> 2) ^ (q0 >> 3)) & 1);
                uoff[i] = ok ? p * (unsigned int)g.pos_bytes + (unsigned int)(grp * g.grp_bytes) + chunk * 16u : 0xFFFFFFFFu;
                if (chunk) odd_chunk |= 1u << i;
            }
        }
        __syncthreads();

        // ---- active output positions -> column list -----------------------------------------------------------
        bool valid[POS_MAXO], act[POS_MAXO];
        int qbase[POS_MAXO];
        unsigned int ypos[POS_MAXO];
#pragma unroll
        for (int i = 0; i < POS_MAXO; ++i) {
            const int lo = tid + PT * i;
            const int gg = lo / (g.R * g.wo), rem = lo - gg * (g.R * g.wo);
            const int row = rem / g.wo, col = rem - row * g.wo;
            const int b = b0 + gg;
            valid[i] = lo < g.G * g.R * g.wo && b < g.n && row < rows_here;
            qbase[i] = (gg * g.RB + row) * g.WP + col;
            ypos[i] = (unsigned int)((b * g.ho + r0 + row) * g.wo + col);
            bool a = valid[i];
            if (MODE == MODE_DELTA && a) {
                unsigned int any = 0;
                for (int ky = 0; ky < g.kh; ++ky)
                    for (int kx = 0; kx < g.kw; ++kx) any |= in_act[qbase[i] + ky * g.WP + kx];
                a = any != 0;
            }
            act[i] = a;
        }
        // (ordered compaction: ballots, wavefront counts through LDS)
        auto build_list = [&]() -> int {
#pragma unroll
            for (int i = 0; i < POS_MAXO; ++i) {
                const unsigned long long m = __ballot(act[i]);
                if (lane == 0) s_cnt[i][wave] = (int)__popcll(m);
            }
            __syncthreads();
            int before = 0, total = 0;
#pragma unroll
            for (int i = 0; i < POS_MAXO; ++i) {
                const unsigned long long m = __ballot(act[i]);
                int mine = before;
                for (int w = 0; w < PT / 64; ++w) {
                    const int c = s_cnt[i][w];
                    if (w < wave) mine += c;
                    total += c;
                }
                before = total;
                if (act[i]) {
                    const int pos = mine + (int)__popcll(m & ((1ull << lane) - 1ull));
                    s_colq[pos] = (unsigned short)qbase[i];
                    s_coly[pos] = ypos[i];
                }
            }
            __syncthreads();
            return total;
        };
        int ncols = build_list();
        // Above a share of active positions where reading and re-writing the stored projection costs more than
        // recomputing it (and, for bf16, multiplying two terms), the unit recomputes its band instead (Eq. 3):
        // all positions, the committed input (the scan has made the snapshot equal to x_t) as the source, one
        // term, accumulators from the bias.  The decision is the unit's own: every output has one owner.
        bool full = false;
        if (MODE == MODE_DELTA && g.xfull != nullptr) {
            const int unit_pos = min(g.G, g.n - b0) * rows_here * g.wo;
            full = (long long)ncols * 100 > (long long)unit_pos * g.full_pct;
            if (full) {
#pragma unroll
                for (int i = 0; i < POS_MAXO; ++i) act[i] = valid[i];
                ncols = build_list();
            }
        }
        if (MODE == MODE_DELTA && flag_owner) {
            if (g.touched) {
#pragma unroll
                for (int i = 0; i < POS_MAXO; ++i)
                    if (valid[i]) g.touched[ypos[i]] = act[i] ? 1 : 0;
            }
            if (tid == 0 && ncols) atomicAdd(&stats[unit & (STAT_SLOTS - 1)].active_tiles, (unsigned long long)ncols);
        }
        const bool from_y = MODE == MODE_DELTA && !full;
        const unsigned char* s0 = full ? g.xfull : src0;
        const bool two = TERMS == 2 && !full;
        const int nst = g.nslab * g.nstage;
        // Every unit walks the slabs in a rotated order of its own, so that at any moment the workgroups of the chip
        // read different parts of the packed weights.  The rotation is a fixed function of the unit: results repeat
        // from run to run.
        const int rot = (unit * 5 + (unit >> 3)) % g.nslab;
        auto phys = [&](int sl) {
            const int p2 = sl + rot;
            return p2 >= g.nslab ? p2 - g.nslab : p2;
        };

        if (producer) {
            // ================= producers: copies into LDS, one stage ahead of the consumers =======================
            const unsigned char* wsrc = wpack + (size_t)(grp * g.ncg + cgrp) * g.nslab * g.ntaps * (NCB * 1024);
            auto stage_a = [&](int slab, int tg, int buf) {
                const int t0 = tg * g.ts, nt = min(g.ts, g.ntaps - t0);
                const unsigned char* src = wsrc + (size_t)(slab * g.ntaps + t0) * (NCB * 1024) + ptid * 16;
                unsigned char* dst = abase + buf * a_bytes + (wave - 4) * 1024;
                for (int t = 0; t < nt; ++t)  // (NCB * 1024 bytes = one round of the 256 producer threads)
                    __builtin_amdgcn_global_load_lds((gptr_t)(src + t * (NCB * 1024)), (lptr_t)(dst + t * (NCB * 1024)), 16, 0, 0);
            };
            auto stage_b = [&](int slab, int buf) {
                unsigned char* dst = bbase + buf * b_bytes;
#pragma unroll
                for (int i = 0; i < POS_MAXU; ++i) {
                    if ((ptid + PP * i) >> 1 >= g.npos) break;
                    // (a chunk beyond the group's channels is a copy of zeros: odd chunk counts are padded)
                    const bool real = uoff[i] != 0xFFFFFFFFu && 2 * slab + (int)((odd_chunk >> i) & 1u) < g.chunks;
                    const unsigned int o = uoff[i] + (unsigned int)slab * 32u;
                    unsigned char* d = dst + (i * PP + (wave - 4) * 64) * 16;  // wave-uniform; the lane adds 16 * lane
                    __builtin_amdgcn_global_load_lds((gptr_t)(real ? s0 + o : zero16), (lptr_t)d, 16, 0, 0);
                    if (TERMS == 2 && two)
                        __builtin_amdgcn_global_load_lds((gptr_t)(real ? src1 + o : zero16), (lptr_t)(d + plane), 16, 0, 0);
                }
            };
            for (int p0 = 0; p0 < ncols; p0 += POS_COLS) {
                stage_a(phys(0), 0, 0);
                stage_b(phys(0), 0);
                int slab = 0, tg = 0;
                for (int s = 0; s < nst; ++s) {
                    __builtin_amdgcn_s_waitcnt(0);  // this wavefront's copies for stage s have landed
                    __syncthreads();                // stage s is published; the consumers are done with stage s - 1
                    int sl1 = slab, tg1 = tg + 1;
                    if (tg1 == g.nstage) {
                        tg1 = 0;
                        ++sl1;
                    }
                    if (s + 1 < nst) {
                        stage_a(phys(sl1), tg1, (s + 1) & 1);
                        if (tg1 == 0) stage_b(phys(sl1), sl1 & 1);
                    }
                    slab = sl1;
                    tg = tg1;
                }
                __syncthreads();  // the consumers are done with the last stage: its buffers are free
            }
        } else {
            // ================= consumers: the matrix products ==========================================================
            for (int p0 = 0; p0 < ncols; p0 += POS_COLS) {
                // ---- this wavefront's column tiles of the pass: tiles wave and wave + 4 --------------------------
                const int ntile = min(POS_COLS / 32, (ncols - p0 + 31) >> 5);
                const int nact = (ntile > wave ? 1 : 0) + (ntile > wave + 4 ? 1 : 0);
                bool cv[NP];
                unsigned int boff[NP], ybase[NP];
#pragma unroll
                for (int j = 0; j < NP; ++j) {
                    const int cidx = p0 + (wave + 4 * j) * 32 + (lane & 31);
                    cv[j] = j < nact && cidx < ncols;
                    boff[j] = cv[j] ? (unsigned int)s_colq[cidx] : 0u;  // band position of the column (tap 0, 0)
                    ybase[j] = (cv[j] ? s_coly[cidx] : 0u) * (unsigned int)g.c_out + (unsigned int)(grp * g.og);
                }
                // channel (within the filter group) of register 4*gq of block c; the 4 registers are consecutive channels
                auto chan = [&](int c, int gq) { return (cgrp * NCB + c) * 32 + 8 * gq + 4 * khalf; };
                // accumulators start from what the result is added to
                acc_t acc[NCB][NP];
#pragma unroll
                for (int c = 0; c < NCB; ++c)
#pragma unroll
                    for (int gq = 0; gq < 4; ++gq) {
                        const int co = chan(c, gq);
                        const bool ch_ok = co < g.og;
                        vec_t bv = vec_t{0, 0, 0, 0};
                        if (!from_y && ch_ok && bias) bv = *reinterpret_cast<const vec_t*>(bias + grp * g.og + co);
#pragma unroll
                        for (int j = 0; j < NP; ++j) {
                            vec_t v = bv;
                            if (from_y && ch_ok && cv[j]) v = *reinterpret_cast<const vec_t*>(y + (ybase[j] + (unsigned int)co));
                            acc[c][j][4 * gq + 0] = v.x;
                            acc[c][j][4 * gq + 1] = v.y;
                            acc[c][j][4 * gq + 2] = v.z;
                            acc[c][j][4 * gq + 3] = v.w;
                        }
                    }

                // K loop of one stage (the taps t0 .. t0 + NT - 1 of one slab), unrolled over the taps: the operands
                // of tap i + 1 are read from LDS into a second register set while tap i multiplies, the reads issued
                // one by one between the matrix instructions.  NT = 0: any number of taps (nt), one after the other.
                auto k_loop = [&]<int NPA, int T, int NT>(const unsigned char* aw, const unsigned char* bw, int t0, int nt) {
                    constexpr int NB1 = T == 2 ? NPA : 1;
                    struct Ops {
                        uint4 a[NCB], b0[NPA], b1[NB1];
                    };
                    constexpr int N_MFMA = NCB * NPA * T;
                    constexpr int N_READ = NCB + NPA * T;
                    int ky = t0 / g.kw, kx = t0 - ky * g.kw;
                    auto fetch = [&](int i, Ops& o) {  // (taps in order: the window offset steps along)
                        const unsigned int tapq = (unsigned int)(ky * g.WP + kx);
                        if (++kx == g.kw) {
                            kx = 0;
                            ++ky;
                        }
#pragma unroll
                        for (int c = 0; c < NCB; ++c) o.a[c] = *reinterpret_cast<const uint4*>(aw + (i * NCB + c) * 1024);
#pragma unroll
                        for (int j = 0; j < NPA; ++j) {
                            // (the position's two chunks are stored swapped according to bits 2 and 3 of its index)
                            const unsigned int q = boff[j] + tapq;
                            const unsigned int off = q * 32u + (((unsigned int)khalf ^ (q >> 2) ^ (q >> 3)) & 1u) * 16u;
                            o.b0[j] = *reinterpret_cast<const uint4*>(bw + off);
                            if (T == 2) o.b1[j] = *reinterpret_cast<const uint4*>(bw + plane + off);
                        }
                    };
                    auto multiply = [&](const Ops& o) {
#pragma unroll
                        for (int t = 0; t < T; ++t)
#pragma unroll
                            for (int c = 0; c < NCB; ++c)
#pragma unroll
                                for (int j = 0; j < NPA; ++j)
                                    acc[c][j] = mma(o.a[c], t == 0 ? o.b0[j] : o.b1[j < NB1 ? j : 0], acc[c][j]);
                    };
                    if constexpr (NT > 0) {
                        Ops o[2];
                        fetch(0, o[0]);
#pragma unroll
                        for (int i = 0; i < NT; ++i) {
                            if (i + 1 < NT) fetch(i + 1, o[(i + 1) & 1]);
                            multiply(o[i & 1]);
                            if (i + 1 < NT) sched_interleave<0, N_MFMA, N_READ>();
                        }
                    } else {
                        for (int i = 0; i < nt; ++i) {
                            Ops o;
                            fetch(i, o);
                            multiply(o);
                        }
                    }
                };

                // ---- stages: (slab, tap group).  The loop is compiled per (column tiles in use, terms, taps per
                // stage): a variant's accumulators never change registers.
                auto run_stages = [&]<int NPA, int T, int NT>() {
                    int slab = 0, tg = 0;
                    for (int s = 0; s < nst; ++s) {
                        // Stage s is staged.  A bare barrier: the producers waited for their copies before they
                        // arrived, and this wavefront's own loads of stored projections and its stores need not
                        // have completed.
                        asm volatile("s_barrier" ::: "memory");
                        if constexpr (NPA > 0) {
                            const unsigned char* aw = abase + (s & 1) * a_bytes + lane * 16;
                            const unsigned char* bw = bbase + (slab & 1) * b_bytes;
                            const int t0 = tg * g.ts;
                            k_loop.template operator()<(NPA > 0 ? NPA : 1), T, NT>(aw, bw, t0, min(g.ts, g.ntaps - t0));
                        }
                        if (++tg == g.nstage) {
                            tg = 0;
                            ++slab;
                        }
                    }
                    // every LDS read of the last stage has been consumed by a matrix instruction issued above
                    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
                };
                // (stages of exactly ts taps get the unrolled loop: 1, 3, 5 and 9 taps, when ts divides the tap count)
                const int nt_fixed = (g.ntaps % g.ts == 0 && (g.ts == 1 || g.ts == 3 || g.ts == 5 || g.ts == 9)) ? g.ts : 0;
                auto run_tiles = [&]<int T>() {
#define RRM_POS_RUN(NPA)                                                     \
    do {                                                                     \
        if (nt_fixed == 9) run_stages.template operator()<NPA, T, 9>();      \
        else if (nt_fixed == 3) run_stages.template operator()<NPA, T, 3>(); \
        else if (nt_fixed == 5) run_stages.template operator()<NPA, T, 5>(); \
        else if (nt_fixed == 1) run_stages.template operator()<NPA, T, 1>(); \
        else run_stages.template operator()<NPA, T, 0>();                    \
    } while (0)
                    if (nact > 1) RRM_POS_RUN(2);
                    else if (nact > 0) RRM_POS_RUN(1);
                    else run_stages.template operator()<0, T, 0>();  // (no column tile: barriers only)
#undef RRM_POS_RUN
                };
                if (two) {
                    if constexpr (TERMS == 2) run_tiles.template operator()<2>();
                } else {
                    run_tiles.template operator()<1>();
                }

                // ---- results back (while the producers stage the next pass / unit) ----------------------------------
#pragma unroll
                for (int c = 0; c < NCB; ++c)
#pragma unroll
                    for (int gq = 0; gq < 4; ++gq) {
                        const int co = chan(c, gq);
                        if (co >= g.og) continue;
#pragma unroll
                        for (int j = 0; j < NP; ++j) {
                            if (!cv[j]) continue;
                            vec_t o;
                            o.x = acc[c][j][4 * gq + 0];
                            o.y = acc[c][j][4 * gq + 1];
                            o.z = acc[c][j][4 * gq + 2];
                            o.w = acc[c][j][4 * gq + 3];
                            *reinterpret_cast<vec_t*>(y + (ybase[j] + (unsigned int)co)) = o;
                        }
                    }
            }
        }

        if (tid == 0) s_next = (int)gridDim.x + (int)nxt_pending;
        __syncthreads();  // (also: both roles are done with this unit's lists)
        unit = s_next;
        __syncthreads();  // (s_next is rewritten at the end of the next unit; the lists at its start)
    }

    // ---- the last workgroup to leave rearms the counters ---------------------------------------------------------
    if (tid == 0) {
        const unsigned int before = atomicAdd(&ctrl[0], 1u);
        if (before == gridDim.x - 1u) {
            ctrl[0] = 0u;
            ctrl[2] = 0u;
            if (MODE == MODE_DELTA && g.fresh) g.fresh[0] = 0u;  // the stored input now holds this step's input
            if (MODE == MODE_DELTA && g.touched_all) g.touched_all[0] = 0u;  // `touched` describes this step
        }
    }
}

template <int DT, int MODE, int TERMS>
hipError_t launch_one(const void* src0, const void* src1, const void* zero16, const unsigned long long* bitmap,
                      unsigned int* ctrl, const void* wpack, const void* bias, void* y, const PosGeom& g, DevStats* stats,
                      hipStream_t s) {
    const size_t lds = conv_pos_lds_bytes(g, TERMS);
    const int gx = std::min(g.total_units, NUM_CU);  // (one workgroup per compute unit; it loops over units)
    auto kern = conv_pos_kernel<DT, MODE, TERMS>;
    if (lds > 64 * 1024) {
        static std::mutex mu;  // one per instantiation, shared by every handle and thread of the process
        static size_t granted = 0;
        std::lock_guard<std::mutex> lock(mu);
        if (lds > granted) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            granted = lds;
        }
    }
    hipLaunchKernelGGL(kern, dim3((unsigned int)gx), dim3(PT), lds, s, static_cast<const unsigned char*>(src0),
                       static_cast<const unsigned char*>(src1), static_cast<const unsigned char*>(zero16), bitmap, ctrl,
                       static_cast<const unsigned char*>(wpack), bias, y, g, stats);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_conv_pos(int dtype, int mode, int terms, const void* src0, const void* src1, const void* zero16,
                           const unsigned long long* bitmap, unsigned int* ctrl, const void* wpack, const void* bias, void* y,
                           const PosGeom& g, DevStats* stats, hipStream_t s) {
    if (dtype == RRM_I8_I32) {
        if (mode == MODE_DELTA)
            return launch_one<RRM_I8_I32, MODE_DELTA, 1>(src0, src1, zero16, bitmap, ctrl, wpack, bias, y, g, stats, s);
        return launch_one<RRM_I8_I32, MODE_DENSE, 1>(src0, src1, zero16, bitmap, ctrl, wpack, bias, y, g, stats, s);
    }
    if (mode == MODE_DENSE)
        return launch_one<RRM_BF16_F32, MODE_DENSE, 1>(src0, src1, zero16, bitmap, ctrl, wpack, bias, y, g, stats, s);
    if (terms == 2)
        return launch_one<RRM_BF16_F32, MODE_DELTA, 2>(src0, src1, zero16, bitmap, ctrl, wpack, bias, y, g, stats, s);
    return launch_one<RRM_BF16_F32, MODE_DELTA, 1>(src0, src1, zero16, bitmap, ctrl, wpack, bias, y, g, stats, s);
}

}  // namespace rrm
