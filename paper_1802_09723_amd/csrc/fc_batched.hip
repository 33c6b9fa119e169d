// Fully-connected layers with many streams: the layer is a skinny matrix product, W [c_out x c_in] times the
// streams' vectors [c_in x n], and it runs on the matrix cores with W read once for all streams.
//
// Dense layer (Eq. 3, FC form):      Y = b + W X^T
// Delta step (Algorithm 1, FC branch), int8: Y += W D^T with D = X_t - X_{t-1} for all streams, in two launches:
//   fc_diff_kernel     writes D (the byte differences), commits the stored input and counts the changes;
//   fc_bt_kernel       multiplies.  With tens of streams the union of the changed columns is most of the matrix
//                      (64 streams at 1 % each already touch half of the columns), so the product runs over all of
//                      W: its cost is one pass over W whatever the density, a tenth of what n separate column walks
//                      cost at 64 streams.
// bf16: the fp32 difference of two bf16 values needs two bf16 terms (hi and lo), so the delta product would be two
// passes of matrix instructions for the same pass over W that the layer itself takes; the step therefore commits,
// counts and recomputes Y = b + W X_t^T (which is also free of the step-to-step rounding of an accumulated sum).
// Shapes: v_mfma_i32_16x16x64_i8 / v_mfma_f32_16x16x32_bf16.  Lane l of a wavefront supplies 16 bytes of A (row
// l % 16 of a 16-row block of W, k-group l / 16: contiguous in W's own row-major layout) and 16 bytes of B (stream
// l % 16 of a 16-stream tile, same k-group: contiguous in a stream's vector), and receives rows 4 (l / 16) .. + 3
// of column l % 16: four consecutive output channels of one stream, one 16-byte store.
// The k range is split over workgroups (fc_bt_kernel, partial sums per split) and a second launch adds the splits
// in a fixed order (fc_bt_reduce_kernel: bit-reproducible fp32).  (Adding them in the product kernel, by the last
// split to arrive, needs device-scope fences around the arrival count; with those the kernel measured 28 us
// slower on the 9216 x 4096 layer -- the second launch costs 4.)
#include <algorithm>
#include <type_traits>

#include "rrm_internal.h"

namespace rrm {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));


// D = x_t - x_snap for every stream, x_snap <- x_t, change counts.  One thread per 16-byte unit.  !WRITE_D: the commit
// and the counts only (the step recomputes the layer from x_t).
template <int DT, bool WRITE_D>
__global__ __launch_bounds__(256) void fc_diff_kernel(const uint4* __restrict__ x_t, uint4* __restrict__ x_snap,
                                                      uint4* __restrict__ d0, uint4* __restrict__ d1, long long nvec,
                                                      unsigned long long n_cin, DevStats* __restrict__ stats) {
    const long long v = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    unsigned int nchanged = 0;
    if (v < nvec) {
        const uint4 a = x_t[v], s = x_snap[v];
        uint4 hi = make_uint4(0, 0, 0, 0), lo = hi;
        if ((a.x ^ s.x) | (a.y ^ s.y) | (a.z ^ s.z) | (a.w ^ s.w)) {
            const unsigned int aw[4] = {a.x, a.y, a.z, a.w}, sw[4] = {s.x, s.y, s.z, s.w};
            unsigned int hw[4], lw[4] = {0u, 0u, 0u, 0u};
            if (DT == RRM_I8_I32) {
                const unsigned int H = 0x80808080u;
                unsigned int ovf = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    // byte-wise wrapping subtraction and its signed-overflow mask
                    const unsigned int d = ((aw[i] | H) - (sw[i] & ~H)) ^ ((aw[i] ^ ~sw[i]) & H);
                    ovf |= (aw[i] ^ sw[i]) & (aw[i] ^ d) & H;
                    hw[i] = d;
                    const unsigned int z = aw[i] ^ sw[i];
                    nchanged += __popc((((z & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | z) & H);
                }
                if (ovf) atomicOr(&stats->range_error, 1u);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    unsigned int h2 = 0, l2 = 0;
#pragma unroll
                    for (int k = 0; k < 2; ++k) {
                        const unsigned int xa = (aw[i] >> (16 * k)) & 0xFFFFu, xb = (sw[i] >> (16 * k)) & 0xFFFFu;
                        if (xa == xb) continue;
                        ++nchanged;
                        if (!WRITE_D) continue;
                        const float d = __uint_as_float(xa << 16) - __uint_as_float(xb << 16);
                        // round-to-nearest-even bf16 of d, and of what is left
                        auto to_bf16 = [](float f) {
                            const unsigned int u = __float_as_uint(f);
                            return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
                        };
                        const unsigned int h = to_bf16(d);
                        const unsigned int l = to_bf16(d - __uint_as_float(h << 16));
                        h2 |= (h & 0xFFFFu) << (16 * k);
                        l2 |= (l & 0xFFFFu) << (16 * k);
                    }
                    hw[i] = h2;
                    lw[i] = l2;
                }
            }
            hi = make_uint4(hw[0], hw[1], hw[2], hw[3]);
            lo = make_uint4(lw[0], lw[1], lw[2], lw[3]);
            x_snap[v] = a;
        }
        if (WRITE_D) {
            d0[v] = hi;
            if (DT == RRM_BF16_F32) d1[v] = lo;
        }
    }
    // counts: wavefront, then workgroup, then one set of atomics
    __shared__ unsigned int s_n[4];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) nchanged += __shfl_xor(nchanged, o);
    if ((threadIdx.x & 63) == 0) s_n[threadIdx.x >> 6] = nchanged;
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int tot = s_n[0] + s_n[1] + s_n[2] + s_n[3];
        if (tot) {
            DevStats* slot = stats + (blockIdx.x & (STAT_SLOTS - 1));
            atomicAdd(&slot->changed_elems, (unsigned long long)tot);
            atomicAdd(&slot->changed_units, (unsigned long long)tot);
            atomicAdd(&slot->active_tiles, (unsigned long long)tot);
        }
        if (blockIdx.x == 0) {  // one launch = one delta step
            atomicAdd(&stats->delta_steps, 1ull);
            atomicAdd(&stats->total_tiles, n_cin);
        }
    }
}

// Partial products P[split] = W[:, k range of the split] B[:, k range]^T.  w: [c_out][c_in] row-major; b: [n][c_in]
// (the streams' vectors, or their differences); part: [splits][n][c_out] 4-byte sums.
// Workgroup (blockIdx.x, blockIdx.y) = (64-row group of W, split of the k range); wavefront v of its four takes the
// 16-row block v of the group.  The k range is walked in chunks of CK steps (a step = 64 bytes of a row and of every
// stream's vector).  Per chunk the workgroup copies the streams' bytes into LDS once -- all four wavefronts multiply
// the same streams, and read from memory they would cost four times the bytes of W -- while every lane reads its own
// 16 bytes of W per step straight into registers.  Loads run four chunks ahead of the matrix instructions, LDS is
// double-buffered, one barrier per chunk.
// LDS layout: (step of the chunk, stream) -> 80 bytes (64 used): the 16 streams that a group of 16 lanes reads for
// one k-group start 20 banks apart and fall on 16 different 4-bank groups.
template <int DT, int TMAX, int CK>
__global__ __launch_bounds__(256) void fc_bt_kernel(const unsigned char* __restrict__ w, const unsigned char* __restrict__ b,
                                                    void* __restrict__ part_v, FcGeom g, int cps) {
    constexpr int ESIZE = DT == RRM_I8_I32 ? 1 : 2;
    constexpr int KSTEP = 64 / ESIZE;  // elements per step: 64 int8 / 32 bf16
    constexpr int NS = 16 * TMAX;      // stream slots of the LDS layout
    constexpr int UPT = (NS * CK * 4 + 255) / 256;  // 16-byte units of the streams' chunk per thread
    constexpr int SPP = 256 / (CK * 4);             // streams covered by one pass of the 256 threads
    static_assert(256 % (CK * 4) == 0, "a pass of the threads covers whole streams");
    typedef typename std::conditional<DT == RRM_I8_I32, int, float>::type val_t;
    typedef typename std::conditional<DT == RRM_I8_I32, v4i, v4f>::type acc_t;
    __shared__ uint4 xs[2][CK * NS * 5];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kg = lane >> 4;  // k-group: bytes 16 kg .. 16 kg + 15 of a step
    const long long row_bytes = (long long)g.c_in * ESIZE;
    const int nsteps = g.c_in / KSTEP;
    const int kbeg = (int)blockIdx.y * cps * CK;
    const int kend = min(kbeg + cps * CK, nsteps);
    const int nch = (kend - kbeg + CK - 1) / CK;  // (>= 1: the host launches no empty split)
    // W: row of this lane (blocks beyond c_out read the last row; their sums are not stored)
    const int o0 = (int)blockIdx.x * 64 + wave * 16;
    const int row = min(o0 + (lane & 15), g.c_out - 1);
    // (byte offsets in 32 bits from the uniform bases: W and the streams' vectors are below 4 GB, checked at create)
    const unsigned int aoff = (unsigned int)row * (unsigned int)row_bytes + kg * 16;
    // streams' chunk: unit tid + 256 i = (stream tid / (4 CK) + SPP i, step (tid / 4) % CK, k-group tid % 4)
    const int xc = (tid >> 2) % CK;
    unsigned int xp[UPT], xm[UPT];
    int xoff[UPT];
#pragma unroll
    for (int i = 0; i < UPT; ++i) {
        const int s = tid / (CK * 4) + i * SPP;
        xm[i] = (unsigned int)-(int)(s < g.n);  // (a stream beyond n reads offset 0: never stored)
        xp[i] = (unsigned int)min(s, g.n - 1) * (unsigned int)row_bytes + (tid & 3) * 16;  // (streams beyond n: the last one's bytes, unused)
        xoff[i] = (xc * NS + s) * 5 + (tid & 3);
    }
    acc_t acc[TMAX];
#pragma unroll
    for (int t = 0; t < TMAX; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[t][i] = 0;
    auto mma = [&](const uint4& a, const uint4& bb, acc_t c) {
        if constexpr (DT == RRM_I8_I32)
            return __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(v4i, a), __builtin_bit_cast(v4i, bb), c, 0, 0, 0);
        else
            return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, bb), c, 0, 0, 0);
    };
    struct Set {
        uint4 a[CK], x[UPT];
    };
    // Loads and LDS stores are unconditional and free of branches, so that the counted waits stay exact (a wait
    // placed after a branch would be for all outstanding loads, the newest included, and the prefetch would be
    // worth nothing): a chunk beyond the split, or a stream slot beyond the tiles in use, reads offset 0 -- one
    // cached line for the whole wavefront -- and the bytes it stores to LDS are never multiplied.  A step beyond
    // the range re-reads the last step: loaded, never multiplied.
    auto issue = [&](int chunk, Set& s) __attribute__((always_inline)) {
        const int k0 = kbeg + chunk * CK;
        const unsigned int lm = (unsigned int)-(int)(chunk < nch);
#pragma unroll
        for (int c = 0; c < CK; ++c)
            s.a[c] = *reinterpret_cast<const uint4*>(w + (size_t)((aoff + (unsigned int)min(k0 + c, nsteps - 1) * 64u) & lm));
#pragma unroll
        for (int i = 0; i < UPT; ++i)
            s.x[i] = *reinterpret_cast<const uint4*>(b + (size_t)((xp[i] + (unsigned int)min(k0 + xc, nsteps - 1) * 64u) & lm & xm[i]));
    };
    auto stage = [&](const Set& s, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < UPT; ++i) xs[buf][xoff[i]] = s.x[i];
    };
    const int boff = (lane & 15) * 5 + kg;
    // (TMAX is the number of 16-stream tiles in use or the next instantiated count: a tile beyond the streams
    // multiplies the bytes that the masked loads brought -- its sums are not stored -- so the products of a chunk
    // are one straight line of LDS reads and matrix instructions)
    auto compute = [&](const uint4(&a)[CK], int buf, int chunk) __attribute__((always_inline)) {
        const int k0 = kbeg + chunk * CK;
        if (k0 + CK <= kend) {
#pragma unroll
            for (int c = 0; c < CK; ++c)
#pragma unroll
                for (int t = 0; t < TMAX; ++t) acc[t] = mma(a[c], xs[buf][(c * NS + 16 * t) * 5 + boff], acc[t]);
            // issue order: the LDS reads of a step ahead of the matrix instructions of the step before it (one
            // wavefront per SIMD: nothing else hides the LDS latency)
            __builtin_amdgcn_sched_group_barrier(0x100, TMAX, 0);
#pragma unroll
            for (int c = 0; c + 1 < CK; ++c) {
                __builtin_amdgcn_sched_group_barrier(0x100, TMAX, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, TMAX, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, TMAX, 0);
        } else {  // the ragged last chunk of the range
#pragma unroll
            for (int c = 0; c < CK; ++c) {
                if (k0 + c >= kend) break;
#pragma unroll
                for (int t = 0; t < TMAX; ++t) acc[t] = mma(a[c], xs[buf][(c * NS + 16 * t) * 5 + boff], acc[t]);
            }
        }
    };
    // Four register sets in a ring: while chunk j is multiplied, chunks j + 1 .. j + 4 are in flight (one workgroup
    // per compute unit: the depth in registers is what keeps enough bytes in flight).  Per chunk: multiply; the next
    // chunk's streams go to the other LDS buffer (every wavefront finished reading it before the last barrier) and
    // its rows of W to `acur`; the freed set is refilled with the chunk four further on; one barrier.
    Set s0, s1, s2, s3;
    uint4 acur[CK];
    auto take = [&](const Set& s) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < CK; ++c) acur[c] = s.a[c];
    };
    auto phase = [&](int j, int buf, Set& nxt) __attribute__((always_inline)) {
        if (j < nch) compute(acur, buf, j);
        stage(nxt, buf ^ 1);
        take(nxt);
        issue(j + 5, nxt);
        __syncthreads();
    };
    issue(0, s0);
    issue(1, s1);
    issue(2, s2);
    issue(3, s3);
    stage(s0, 0);
    take(s0);
    issue(4, s0);
    __syncthreads();
    for (int j = 0; j < nch; j += 4) {
        phase(j, 0, s1);
        phase(j + 1, 1, s2);
        phase(j + 2, 0, s3);
        phase(j + 3, 1, s0);
    }
    // this split's sums: rows 4 (lane / 16) .. + 3 of the block for stream lane % 16 of every tile
    if (o0 < g.c_out) {
        val_t* part = static_cast<val_t*>(part_v) + (long long)blockIdx.y * g.n * g.c_out;
        const int oc = o0 + 4 * kg;
#pragma unroll
        for (int t = 0; t < TMAX; ++t) {
            const int s = 16 * t + (lane & 15);
            if (s < g.n) *reinterpret_cast<acc_t*>(part + (long long)s * g.c_out + oc) = acc[t];
        }
    }
}

// y = base + the splits' sums, added in the order of the splits (bit-reproducible fp32); base: y itself (delta step)
// or the bias.  One thread per four consecutive output channels of one stream.
template <int DT, bool DELTA>
__global__ __launch_bounds__(256) void fc_bt_reduce_kernel(const void* __restrict__ part_v, const void* __restrict__ bias_v,
                                                           void* y_v, long long nvec, int c_out4, int splits) {
    typedef typename std::conditional<DT == RRM_I8_I32, v4i, v4f>::type acc_t;
    const long long v = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= nvec) return;
    const acc_t* part = static_cast<const acc_t*>(part_v);
    acc_t sum = part[v];
    for (int sp = 1; sp < splits; ++sp) {
        const acc_t o = part[(long long)sp * nvec + v];
#pragma unroll
        for (int i = 0; i < 4; ++i) sum[i] += o[i];
    }
    acc_t* y = static_cast<acc_t*>(y_v);
    acc_t base;
    if (DELTA) {
        base = y[v];
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) base[i] = 0;
        if (bias_v) base = static_cast<const acc_t*>(bias_v)[v % c_out4];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) base[i] += sum[i];
    y[v] = base;
}

int bt_chunk(int ntiles) { return ntiles <= 4 ? 4 : 2; }

// streams per launch of the product kernel: more than 128 go in equal groups (a launch for 256 streams would walk the
// k range in single steps with a barrier each and far fewer splits: two launches of 128 take half its time, W is read
// twice)
constexpr int BT_MAX_STREAMS = 128;
int bt_group(int n) {
    const int ngroups = (n + BT_MAX_STREAMS - 1) / BT_MAX_STREAMS;
    return std::min(n, ((n + ngroups - 1) / ngroups + 15) / 16 * 16);
}

template <int DT, bool DELTA>
void launch_batched(const void* w_rm, const void* b0, void* part, const void* bias, void* y, const FcGeom& g, hipStream_t s) {
    const int esize = DT == RRM_I8_I32 ? 1 : 2;
    const int nsteps = g.c_in * esize / 64;
    const int per = bt_group(g.n);
    const unsigned char* w = static_cast<const unsigned char*>(w_rm);
    for (int s0 = 0; s0 < g.n; s0 += per) {
        FcGeom gg = g;
        gg.n = std::min(per, g.n - s0);
        const int ntiles = (gg.n + 15) / 16;
        const int ck = bt_chunk(ntiles);
        const int chunks = (nsteps + ck - 1) / ck;
        const int want = fc_batched_splits(DT, gg);
        const int cps = (chunks + want - 1) / want;
        const int splits = (chunks + cps - 1) / cps;  // (no empty split)
        dim3 grid((unsigned int)((g.c_out + 63) / 64), (unsigned int)splits);
        const unsigned char* p0 = static_cast<const unsigned char*>(b0) + (size_t)s0 * g.c_in * esize;
        unsigned char* yg = static_cast<unsigned char*>(y) + (size_t)s0 * g.c_out * 4;
#define RRM_BT(T, C)                                                                                                  \
    if (ntiles <= T) {                                                                                                \
        hipLaunchKernelGGL((fc_bt_kernel<DT, T, C>), grid, dim3(256), 0, s, w, p0, part, gg, cps);                    \
    } else
        RRM_BT(1, 4) RRM_BT(2, 4) RRM_BT(3, 4) RRM_BT(4, 4) RRM_BT(6, 2) RRM_BT(8, 2) {}
#undef RRM_BT
        const long long nvec = (long long)gg.n * g.c_out / 4;
        hipLaunchKernelGGL((fc_bt_reduce_kernel<DT, DELTA>), dim3((unsigned int)((nvec + 255) / 256)), dim3(256), 0, s, part, bias,
                           yg, nvec, g.c_out / 4, splits);
    }
}

}  // namespace

// Splits of the k range: about one workgroup per compute unit, at least three chunks per split, and partial sums
// (written and read once per split) of at most half the bytes of W.
int fc_batched_splits(int dtype, const FcGeom& g) {
    const int esize = dtype == RRM_I8_I32 ? 1 : 2;
    const int n = bt_group(g.n);  // (streams of one launch)
    const int ck = bt_chunk((n + 15) / 16);
    const int chunks = (g.c_in * esize / 64 + ck - 1) / ck;
    const int groups = (g.c_out + 63) / 64;
    int s = (NUM_CU + groups - 1) / groups;
    s = std::min(s, chunks / 3);
    s = std::min(s, g.c_in * esize / (16 * n));
    return std::max(s, 1);
}

bool fc_batched_ok(int dtype, const FcGeom& g) {
    const int esize = dtype == RRM_I8_I32 ? 1 : 2;
    // (whole 16-row blocks and 64-byte steps; byte offsets into W in 32 bits)
    return g.n >= FC_BATCH_MIN_STREAMS && g.n <= FC_BATCH_MAX_STREAMS && g.c_out % 16 == 0 && (g.c_in * esize) % 64 == 0 &&
           (long long)g.c_in * esize * g.c_out <= 0xFFFFFFFFll;
}

hipError_t launch_fc_batched_dense(int dtype, const void* w_rm, const void* x, void* part, const void* bias, void* y,
                                   const FcGeom& g, hipStream_t s) {
    if (!fc_batched_ok(dtype, g)) return hipErrorInvalidValue;
    if (dtype == RRM_I8_I32)
        launch_batched<RRM_I8_I32, false>(w_rm, x, part, bias, y, g, s);
    else
        launch_batched<RRM_BF16_F32, false>(w_rm, x, part, bias, y, g, s);
    return hipGetLastError();
}

hipError_t launch_fc_batched_delta(int dtype, const void* w_rm, const void* x_t, void* x_snap, void* d0, void* part,
                                   const void* bias, void* y, const FcGeom& g, DevStats* stats, hipStream_t s) {
    if (!fc_batched_ok(dtype, g) || g.eps != 0.0f) return hipErrorInvalidValue;
    const int esize = dtype == RRM_I8_I32 ? 1 : 2;
    const long long nvec = (long long)g.n * g.c_in * esize / 16;
    const unsigned long long n_cin = (unsigned long long)g.n * (unsigned long long)g.c_in;
    dim3 dgrid((unsigned int)((nvec + 255) / 256)), dblock(256);
    if (dtype == RRM_I8_I32) {
        hipLaunchKernelGGL((fc_diff_kernel<RRM_I8_I32, true>), dgrid, dblock, 0, s, (const uint4*)x_t, (uint4*)x_snap, (uint4*)d0,
                           (uint4*)nullptr, nvec, n_cin, stats);
        launch_batched<RRM_I8_I32, true>(w_rm, d0, part, nullptr, y, g, s);
    } else {
        // bf16: the difference needs two bf16 terms, i.e. two products over all of W, while the layer itself (Eq. 3)
        // is one -- and it does not accumulate rounding from step to step.  The step commits, counts and recomputes.
        hipLaunchKernelGGL((fc_diff_kernel<RRM_BF16_F32, false>), dgrid, dblock, 0, s, (const uint4*)x_t, (uint4*)x_snap,
                           (uint4*)nullptr, (uint4*)nullptr, nvec, n_cin, stats);
        launch_batched<RRM_BF16_F32, false>(w_rm, x_t, part, bias, y, g, s);
    }
    return hipGetLastError();
}

}  // namespace rrm
