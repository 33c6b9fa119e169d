// Fully-connected layers: the sparse-delta step P_t = P_{t-1} + W (I_t - I_{t-1}) (Algorithm 1, FC branch) and the
// dense layer P = b + W I (Eq. 3, FC form).
//
// The engine the paper relies on (Sec. 3.5) scans the activation vector for non-zero entries, broadcasts
// (a_j, j) and multiplies the weight column W_j, summing into row accumulators.  Here the weights are stored
// input-major (W^T [c_in][c_out], every column of W contiguous) and a step is ONE launch (fc_delta_kernel): compare,
// compaction of the changed entries, the walk over their columns and the sum into the stored projection.  The
// layer is memory bound: bytes moved are (changed columns) x c_out x element size.
// The dense layer streams all of W^T, split over rows and output-channel slices (fc_dense_kernel), and adds the
// splits' partial sums in a fixed order (fc_reduce_kernel): no atomics, bit-reproducible for fp32.
#include <algorithm>
#include <mutex>
#include <type_traits>

#include "rrm_internal.h"

namespace rrm {

namespace {

constexpr int FCD_THREADS = 512;   // 8 wavefronts (up to 256 registers each: nothing spills)
constexpr int FCD_CH = 8192;        // inputs of one compare round = capacity of the changed-column list in LDS
constexpr int FCD_UN = 8;           // columns in flight per lane
constexpr int FCD_SEG = 64;         // bytes of a weight column one workgroup owns (4 lanes of 16 bytes)

__device__ __forceinline__ float bf16_to_f32(unsigned int h) { return __uint_as_float(h << 16); }

// One launch per step (Algorithm 1, FC branch; the column walk of Sec. 3.5): workgroup (r, b) owns FCD_SEG bytes
// worth of output channels of stream b.  Every workgroup compares x_t with the stored input itself (the vector is
// a few KB: redoing the compare costs less than a second launch), compacts the changed entries (index, difference)
// in index order into LDS, streams its 64-byte piece of every listed column of W (rows of W^T), and adds the
// column sum into its own channels of the stored projection: one owner per output, no partial sums in memory, no
// atomics on y, the same summation order in every run.  The stored input is committed by whichever workgroup of
// the stream finishes its compare last (an arrival counter tells it that nobody reads the old values any more);
// it also rearms the counter, so a step leaves no host-visible state behind (graph replay safe).
//
// CSC = true (pruned weights, Sec. 4.3: the compressed model keeps its non-zero weights only): the columns of W
// are stored as (row, value) lists.  Workgroup (r, b) takes every gridDim.x-th block of eight listed columns, one
// column per wavefront with the lanes over its non-zeros, and adds the products into a private copy of the
// projection's update in LDS (all c_out rows); at the end it adds the rows it touched into the stored projection
// with atomic adds (exact for integers; fp32 sums then depend on the order within the layer's tolerance).
template <int DT, bool CSC>
__global__ __launch_bounds__(FCD_THREADS) void fc_delta_kernel(const unsigned char* __restrict__ x_t,
                                                               unsigned char* x_snap,
                                                               const unsigned char* __restrict__ wT, void* y_v,
                                                               unsigned int* arrive, FcGeom g,
                                                               DevStats* __restrict__ stats) {
    constexpr int PV = DT == RRM_I8_I32 ? 16 : 8;
    constexpr int ESIZE = DT == RRM_I8_I32 ? 1 : 2;
    constexpr int NCG = FCD_THREADS / 4;  // column groups: 4 lanes (64 bytes) per column
    typedef typename std::conditional<DT == RRM_I8_I32, int, float>::type val_t;
    __shared__ unsigned short l_idx[FCD_CH];
    __shared__ val_t l_val[FCD_CH];
    __shared__ val_t red[FCD_THREADS / 64][4][PV];
    __shared__ int wave_tot[FCD_THREADS / 64];
    __shared__ unsigned int s_prev;
    extern __shared__ uint4 fc_dyn[];  // CSC: one update accumulator per output row
    val_t* ly = reinterpret_cast<val_t*>(fc_dyn);
    const int r = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (CSC)
        for (int o = tid; o < g.c_out; o += FCD_THREADS) ly[o] = 0;  // (the first round's barriers order this)
    // integer layers split long lists over gridDim.z workgroups, pass by pass (pass p of NCG * FCD_UN columns goes
    // to workgroup p % gridDim.z), and add with integer atomics: exact in any order
    const int ks = blockIdx.z, nks = gridDim.z;
    const int sub = tid & 3, cgid = tid >> 2;
    const long long row = (long long)b * g.c_in;
    const int co0 = r * (FCD_SEG / ESIZE) + sub * PV;  // this lane's first output channel
    const bool live = co0 < g.c_out_p;
    const unsigned char* wcol = wT + (long long)(live ? co0 : 0) * ESIZE;
    const long long pitch = (long long)g.c_out_p * ESIZE;
    val_t acc[PV];
#pragma unroll
    for (int e = 0; e < PV; ++e) acc[e] = 0;
    unsigned int ntrunc = 0, total = 0;
    float tsq = 0.f;

    // the two copies of one 16-byte unit (PV entries from element e0 of the row); rows that are not 16-byte
    // multiples are gathered element by element (zeros beyond the row's end)
    auto load_unit = [&](int e0, uint4& a, uint4& s) {
        if (g.vec_ok) {
            a = *reinterpret_cast<const uint4*>(x_t + (row + e0) * ESIZE);
            s = *reinterpret_cast<const uint4*>(x_snap + (row + e0) * ESIZE);
            return;
        }
        unsigned int aw[4] = {0u, 0u, 0u, 0u}, sw[4] = {0u, 0u, 0u, 0u};
        for (int e = 0; e < PV; ++e) {
            if (e0 + e >= g.c_in) break;
            if (DT == RRM_I8_I32) {
                aw[e >> 2] |= (unsigned int)x_t[row + e0 + e] << (8 * (e & 3));
                sw[e >> 2] |= (unsigned int)x_snap[row + e0 + e] << (8 * (e & 3));
            } else {
                aw[e >> 1] |= (unsigned int)reinterpret_cast<const unsigned short*>(x_t)[row + e0 + e] << (16 * (e & 1));
                sw[e >> 1] |= (unsigned int)reinterpret_cast<const unsigned short*>(x_snap)[row + e0 + e] << (16 * (e & 1));
            }
        }
        a = make_uint4(aw[0], aw[1], aw[2], aw[3]);
        s = make_uint4(sw[0], sw[1], sw[2], sw[3]);
    };
    // difference of a unit: mask of the entries to apply, their values, and the unit's new snapshot
    auto diff_unit = [&](const uint4& a, const uint4& s, val_t (&dv)[PV], unsigned int& mask, uint4& n_out) {
        mask = 0;
        n_out = a;
        if (!((a.x ^ s.x) | (a.y ^ s.y) | (a.z ^ s.z) | (a.w ^ s.w))) return;
        const unsigned int aw[4] = {a.x, a.y, a.z, a.w}, sw[4] = {s.x, s.y, s.z, s.w};
        unsigned int nw[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int e = 0; e < PV; ++e) {
            if (DT == RRM_I8_I32) {
                const int xa = (int)(signed char)(aw[e >> 2] >> (8 * (e & 3)));
                const int xb = (int)(signed char)(sw[e >> 2] >> (8 * (e & 3)));
                dv[e] = (val_t)(xa - xb);
                if (xa != xb) mask |= 1u << e;
            } else {
                // (truncation threshold, Sec. 3.4 "Improving sparsity": a difference below g.eps is neither
                // applied nor committed; eps = 0 is the exact method)
                const unsigned int xa = (aw[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                const unsigned int xb = (sw[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                const float d = bf16_to_f32(xa) - bf16_to_f32(xb);
                dv[e] = (val_t)d;
                if (xa != xb) {
                    if (fabsf(d) < g.eps) {
                        ++ntrunc;
                        tsq += d * d;
                        nw[e >> 1] = (nw[e >> 1] & ~(0xFFFFu << (16 * (e & 1)))) | (xb << (16 * (e & 1)));
                    } else {
                        mask |= 1u << e;
                    }
                }
            }
        }
        n_out = make_uint4(nw[0], nw[1], nw[2], nw[3]);
    };
    auto store_unit = [&](int e0, const uint4& nw) {  // commit a unit's new snapshot
        if (g.vec_ok) {
            *reinterpret_cast<uint4*>(x_snap + (row + e0) * ESIZE) = nw;
            return;
        }
        const unsigned int w[4] = {nw.x, nw.y, nw.z, nw.w};
        for (int e = 0; e < PV; ++e) {
            if (e0 + e >= g.c_in) break;
            if (DT == RRM_I8_I32)
                x_snap[row + e0 + e] = (unsigned char)(w[e >> 2] >> (8 * (e & 3)));
            else
                reinterpret_cast<unsigned short*>(x_snap)[row + e0 + e] = (unsigned short)(w[e >> 1] >> (16 * (e & 1)));
        }
    };
    auto fma16 = [&](const uint4& w, val_t d) {
        const unsigned int ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int e = 0; e < PV; ++e) {
            if (DT == RRM_I8_I32)
                acc[e] += d * (val_t)(int)(signed char)(ww[e >> 2] >> (8 * (e & 3)));
            else
                acc[e] += d * (val_t)__uint_as_float((e & 1) ? (ww[e >> 1] & 0xFFFF0000u) : (ww[e >> 1] << 16));
        }
    };

    // One compare round covers FCD_CH inputs, at most one 16-byte unit per thread: the loads of round c + 1 are
    // issued before round c's columns are streamed, and the first KEEP rounds' new snapshots stay in registers for
    // the commit.
    constexpr int CHU = FCD_THREADS * PV < FCD_CH ? FCD_THREADS * PV : FCD_CH;
    static_assert(CHU / PV <= FCD_THREADS && CHU <= FCD_CH, "one unit per thread and round; the list holds a round");
    constexpr int KEEP = 2;
    const int nchunk = (g.c_in + CHU - 1) / CHU;
    uint4 keep_nw[KEEP];
    unsigned int keep_mask[KEEP];
#pragma unroll
    for (int i = 0; i < KEEP; ++i) keep_mask[i] = 0;
    // this workgroup's channels of the stored projection, fetched now and needed at the end
    const int co_y = r * (FCD_SEG / ESIZE) + tid;
    val_t y_old = 0;
    if (!CSC && nks == 1 && tid < 4 * PV && co_y < g.c_out) y_old = static_cast<const val_t*>(y_v)[(long long)b * g.c_out + co_y];
    uint4 cur_a = make_uint4(0, 0, 0, 0), cur_s = cur_a;
    if (tid * PV < min(CHU, g.c_in)) load_unit(tid * PV, cur_a, cur_s);
    for (int ch = 0; ch < nchunk; ++ch) {
        const int base = ch * CHU;
        const int n_in = min(CHU, g.c_in - base);
        const int nunits = (n_in + PV - 1) / PV;
        // ---- compare + ordered compaction of this round's inputs ------------------------------------------
        int running = 0;
        {
            const int u = tid;
            val_t dv[PV];
            unsigned int mask = 0;
            uint4 nw = cur_a;
            if (u < nunits) diff_unit(cur_a, cur_s, dv, mask, nw);
#pragma unroll
            for (int i = 0; i < KEEP; ++i)
                if (ch == i) {
                    keep_nw[i] = nw;
                    keep_mask[i] = mask;
                }
            // the next round's units are on their way while this round's columns are streamed
            if (ch + 1 < nchunk && tid * PV < CHU && base + CHU + tid * PV < g.c_in)
                load_unit(base + CHU + tid * PV, cur_a, cur_s);
            const int cnt = __popc(mask);
            int incl = cnt;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_up(incl, o);
                if (lane >= o) incl += t;
            }
            if (lane == 63) wave_tot[wave] = incl;
            __syncthreads();
            int wbase = 0, btot = 0;
            for (int w = 0; w < FCD_THREADS / 64; ++w) {
                const int t = wave_tot[w];
                if (w < wave) wbase += t;
                btot += t;
            }
            int pos = wbase + incl - cnt;
            if (mask) {
#pragma unroll
                for (int e = 0; e < PV; ++e)
                    if (mask & (1u << e)) {
                        l_idx[pos] = (unsigned short)(u * PV + e);
                        l_val[pos] = dv[e];
                        ++pos;
                    }
            }
            running = btot;
            __syncthreads();  // the list is published (and wave_tot may be rewritten)
        }
        const int cnt = running;
        total += (unsigned int)cnt;
        // every read of the stored input by this workgroup is done: tell the stream's other workgroups
        if (ch == nchunk - 1 && tid == 0) s_prev = atomicAdd(&arrive[b], 1u);
        if (CSC) {
            // ---- this workgroup's blocks of eight listed columns, one column per wavefront ---------------------
            const unsigned int* cptr = g.csc_ptr;
            constexpr int NW = FCD_THREADS / 64, PRE = 4;  // (PRE columns' offsets in flight per wavefront)
            const int kstep = (int)gridDim.x * NW;
            for (int k0 = (int)blockIdx.x * NW + wave; k0 < cnt; k0 += PRE * kstep) {
                unsigned int p0[PRE], p1[PRE];
                val_t d[PRE];
#pragma unroll
                for (int i = 0; i < PRE; ++i) {
                    const int k = k0 + i * kstep;
                    const bool ok = k < cnt;
                    const int j = ok ? base + l_idx[k] : 0;
                    d[i] = ok ? l_val[k] : (val_t)0;
                    p0[i] = ok ? cptr[j] : 0u;
                    p1[i] = ok ? cptr[j + 1] : 0u;
                }
#pragma unroll
                for (int i = 0; i < PRE; ++i) {
#pragma unroll 8
                    for (unsigned int e = p0[i] + lane; e < p1[i]; e += 64) {
                        const int o = g.csc_row[e];
                        val_t w;
                        if (DT == RRM_I8_I32)
                            w = (val_t)(int)static_cast<const signed char*>(g.csc_val)[e];
                        else
                            w = (val_t)bf16_to_f32(static_cast<const unsigned short*>(g.csc_val)[e]);
                        atomicAdd(&ly[o], d[i] * w);  // (LDS: rows of one column are distinct, wavefronts may share a row)
                    }
                }
            }
        } else if (live) {
            // ---- this workgroup's 64 bytes of every listed column ------------------------------------------------
            for (int k0 = ks * (FCD_UN * NCG); k0 < cnt; k0 += nks * (FCD_UN * NCG)) {
                const int k = k0 + cgid;
                int j[FCD_UN];
                val_t d[FCD_UN];
                uint4 w[FCD_UN];
                if (k0 + FCD_UN * NCG <= cnt) {  // a full pass (the same branch in every thread)
#pragma unroll
                    for (int u = 0; u < FCD_UN; ++u) {
                        j[u] = base + l_idx[k + u * NCG];
                        d[u] = l_val[k + u * NCG];
                    }
#pragma unroll
                    for (int u = 0; u < FCD_UN; ++u) w[u] = *reinterpret_cast<const uint4*>(wcol + j[u] * pitch);
                } else {  // the list's tail: whatever is there, in flight together
#pragma unroll
                    for (int u = 0; u < FCD_UN; ++u) {
                        const bool ok = k + u * NCG < cnt;
                        j[u] = ok ? base + l_idx[k + u * NCG] : 0;
                        d[u] = ok ? l_val[k + u * NCG] : (val_t)0;
                    }
#pragma unroll
                    for (int u = 0; u < FCD_UN; ++u)
                        w[u] = k + u * NCG < cnt ? *reinterpret_cast<const uint4*>(wcol + j[u] * pitch) : uint4{0u, 0u, 0u, 0u};
                }
#pragma unroll
                for (int u = 0; u < FCD_UN; ++u) fma16(w[u], d[u]);
            }
        }
        if (ch + 1 < nchunk) __syncthreads();  // the list is rewritten by the next round
    }

    // ---- column groups -> one sum per channel: butterfly inside the wavefront (lanes with the same `sub`), then
    // the wavefronts in order through LDS.  The order is fixed, so fp32 results repeat from run to run.
    if (CSC) {
        __syncthreads();  // every wavefront's LDS adds are done
        if (total) {
            val_t* yb = static_cast<val_t*>(y_v) + (long long)b * g.c_out;
            for (int o = tid; o < g.c_out; o += FCD_THREADS) {
                const val_t v = ly[o];
                if (v != (val_t)0) atomicAdd(yb + o, v);
            }
        }
    } else if (total) {  // (the same in every thread: the list lengths)
#pragma unroll
        for (int e = 0; e < PV; ++e) {
            val_t v = acc[e];
            v += __shfl_xor(v, 4);
            v += __shfl_xor(v, 8);
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            acc[e] = v;
        }
        if (lane < 4) {
#pragma unroll
            for (int e = 0; e < PV; ++e) red[wave][lane][e] = acc[e];
        }
        __syncthreads();
        if (tid < 4 * PV) {
            val_t sum = 0;
#pragma unroll
            for (int w = 0; w < FCD_THREADS / 64; ++w) sum += red[w][tid / PV][tid % PV];
            if (co_y < g.c_out) {
                val_t* yp = static_cast<val_t*>(y_v) + (long long)b * g.c_out + co_y;
                if constexpr (DT == RRM_I8_I32) {
                    if (nks > 1) {
                        if (sum != 0) atomicAdd(yp, sum);
                    } else {
                        *yp = y_old + sum;
                    }
                } else {
                    *yp = y_old + sum;
                }
            }
        }
    }
    // ---- statistics (one workgroup per stream) ----------------------------------------------------------
    if (r == 0 && ks == 0) {
        if (DT == RRM_BF16_F32) {
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                ntrunc += __shfl_xor(ntrunc, o);
                tsq += __shfl_xor(tsq, o);
            }
            if (lane == 0 && ntrunc) {
                atomicAdd(&stats->truncated_elems, (unsigned long long)ntrunc);
                atomicAdd(&stats->truncated_sumsq, (double)tsq);
            }
        }
        if (tid == 0) {
            if (b == 0) {  // one launch = one delta step
                atomicAdd(&stats->delta_steps, 1ull);
                atomicAdd(&stats->total_tiles, (unsigned long long)g.n * (unsigned long long)g.c_in);
            }
            if (total) {
                atomicAdd(&stats->changed_elems, (unsigned long long)total);
                atomicAdd(&stats->changed_units, (unsigned long long)total);
                atomicAdd(&stats->active_tiles, (unsigned long long)total);
            }
        }
    }
    // ---- commit: the workgroup that finished comparing last snapshots the input (applied entries only) -------
    __syncthreads();  // (s_prev was written by thread 0 after the last round's barrier)
    if (s_prev == gridDim.x * gridDim.z - 1u) {
#pragma unroll
        for (int i = 0; i < KEEP; ++i)
            if (i < nchunk && keep_mask[i]) store_unit(i * CHU + tid * PV, keep_nw[i]);
        for (int ch = KEEP; ch < nchunk; ++ch) {  // (long rows: compare again)
            const int e0 = ch * CHU + tid * PV;
            if (tid * PV >= CHU || e0 >= g.c_in) continue;
            uint4 a, s, nw;
            val_t dv[PV];
            unsigned int mask = 0;
            load_unit(e0, a, s);
            const unsigned int nt0 = ntrunc;
            const float tq0 = tsq;
            diff_unit(a, s, dv, mask, nw);
            ntrunc = nt0;  // (already counted)
            tsq = tq0;
            if (mask) store_unit(e0, nw);
        }
        if (tid == 0) arrive[b] = 0u;
    }
}

constexpr int FC_LANES = 64;      // lanes of a dense workgroup along the output channels (16 bytes each)
constexpr int FC_KG = 8;          // row groups of a dense workgroup (512 threads = 8 wavefronts)
constexpr int FC_MAX_SPLITS = 64;

// Dense layer (Eq. 3, FC form), first of two kernels.  Workgroup (slice, split s, stream): 64 lanes of 16 bytes
// of output channels each, times FC_KG wavefronts; wavefront kg of split s takes rows s*FC_KG + kg,
// + splits*FC_KG, ... of W^T, eight 16-byte loads in flight per lane.  The wavefronts' sums are added through LDS
// in a fixed order, so a split leaves one row of partial sums in the scratch `part` [stream][split][c_out_p].
template <int DT>
__global__ __launch_bounds__(FC_KG * FC_LANES) void fc_dense_kernel(const unsigned char* __restrict__ wT,
                                                                    const unsigned char* __restrict__ x,
                                                                    void* __restrict__ part_v, FcGeom g, int splits) {
    constexpr int PV = DT == RRM_I8_I32 ? 16 : 8;
    constexpr int ESIZE = DT == RRM_I8_I32 ? 1 : 2;
    constexpr int UN = 8;  // rows in flight per lane
    typedef typename std::conditional<DT == RRM_I8_I32, int, float>::type val_t;
    typedef typename std::conditional<DT == RRM_I8_I32, int4, float4>::type vec_t;
    __shared__ vec_t red[FC_KG - 1][PV / 4][FC_LANES];
    const int b = blockIdx.z, s = blockIdx.y;
    const int cnt = g.c_in;
    const int lane = threadIdx.x & (FC_LANES - 1), kg = threadIdx.x / FC_LANES;
    const int co0 = (blockIdx.x * FC_LANES + lane) * PV;
    const bool live = co0 < g.c_out_p;
    const long long row = (long long)b * g.c_in;
    val_t acc[PV];
#pragma unroll
    for (int e = 0; e < PV; ++e) acc[e] = 0;
    const unsigned char* wcol = wT + (long long)(live ? co0 : 0) * ESIZE;
    const long long pitch = (long long)g.c_out_p * ESIZE;

    auto input = [&](int k) -> val_t {
        if (DT == RRM_I8_I32) return (val_t)(int)(signed char)x[row + k];
        return (val_t)bf16_to_f32(reinterpret_cast<const unsigned short*>(x)[row + k]);
    };
    auto fma16 = [&](const uint4& w, val_t d) {
        const unsigned int ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int e = 0; e < PV; ++e) {
            if (DT == RRM_I8_I32)
                acc[e] += d * (val_t)(int)(signed char)(ww[e >> 2] >> (8 * (e & 3)));
            else
                acc[e] += d * (val_t)__uint_as_float((e & 1) ? (ww[e >> 1] & 0xFFFF0000u) : (ww[e >> 1] << 16));
        }
    };

    if (live) {
        const int step = splits * FC_KG;
        int k = s * FC_KG + kg;
        for (; k + (UN - 1) * step < cnt; k += UN * step) {
            val_t d[UN];
            uint4 w[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) w[u] = *reinterpret_cast<const uint4*>(wcol + (k + u * step) * pitch);
#pragma unroll
            for (int u = 0; u < UN; ++u) d[u] = input(k + u * step);
#pragma unroll
            for (int u = 0; u < UN; ++u) fma16(w[u], d[u]);
        }
        {   // the rest of this wavefront's rows (fewer than UN), in flight together
            val_t d[UN];
            uint4 w[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const bool ok = k + u * step < cnt;
                w[u] = ok ? *reinterpret_cast<const uint4*>(wcol + (k + u * step) * pitch) : uint4{0u, 0u, 0u, 0u};
                d[u] = ok ? input(k + u * step) : (val_t)0;
            }
#pragma unroll
            for (int u = 0; u < UN; ++u) fma16(w[u], d[u]);
        }
    }
    // wavefronts 1.. hand their sums to wavefront 0 (added in order: the result does not depend on timing)
    if (kg > 0) {
#pragma unroll
        for (int e = 0; e < PV; e += 4) {
            vec_t o;
            o.x = acc[e]; o.y = acc[e + 1]; o.z = acc[e + 2]; o.w = acc[e + 3];
            red[kg - 1][e >> 2][lane] = o;
        }
    }
    __syncthreads();
    if (kg == 0 && live) {
#pragma unroll
        for (int q = 0; q < FC_KG - 1; ++q)
#pragma unroll
            for (int e = 0; e < PV; e += 4) {
                const vec_t o = red[q][e >> 2][lane];
                acc[e] += o.x; acc[e + 1] += o.y; acc[e + 2] += o.z; acc[e + 3] += o.w;
            }
        val_t* part = static_cast<val_t*>(part_v) + ((long long)b * splits + s) * g.c_out_p + co0;
#pragma unroll
        for (int e = 0; e < PV; e += 4) {
            vec_t o;
            o.x = acc[e]; o.y = acc[e + 1]; o.z = acc[e + 2]; o.w = acc[e + 3];
            *reinterpret_cast<vec_t*>(part + e) = o;
        }
    }
}

// Second kernel of the dense layer.  Workgroup (block of 64 channels, stream): 16 lanes of 4 channels each times
// 64 split groups, one partial row per group (all loads in flight at once); the groups' values meet in LDS and 16
// threads add them in split order and write y = bias + sum.
template <int DT>
__global__ __launch_bounds__(FC_MAX_SPLITS * 16) void fc_reduce_kernel(const void* __restrict__ part_v,
                                                                       const void* __restrict__ bias_v,
                                                                       void* __restrict__ y_v, FcGeom g, int splits) {
    typedef typename std::conditional<DT == RRM_I8_I32, int, float>::type val_t;
    typedef typename std::conditional<DT == RRM_I8_I32, int4, float4>::type vec_t;
    __shared__ vec_t red[FC_MAX_SPLITS][16];
    const int b = blockIdx.y;
    const int lane = threadIdx.x & 15, sg = threadIdx.x >> 4;
    const int co = (blockIdx.x * 16 + lane) * 4;
    const bool live = co < g.c_out_p;  // (c_out_p is a multiple of 4)
    if (sg < splits)
        red[sg][lane] = live ? *reinterpret_cast<const vec_t*>(static_cast<const val_t*>(part_v) +
                                                               ((long long)b * splits + sg) * g.c_out_p + co)
                             : vec_t{0, 0, 0, 0};
    __syncthreads();
    if (sg != 0 || !live) return;
    vec_t sum = red[0][lane];
    for (int q = 1; q < splits; ++q) {
        const vec_t o = red[q][lane];
        sum.x += o.x; sum.y += o.y; sum.z += o.z; sum.w += o.w;
    }
    val_t* y = static_cast<val_t*>(y_v) + (long long)b * g.c_out;
    const val_t* bias = static_cast<const val_t*>(bias_v);
    const val_t r[4] = {sum.x, sum.y, sum.z, sum.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        if (co + k >= g.c_out) break;
        y[co + k] = (bias ? bias[co + k] : (val_t)0) + r[k];
    }
}

}  // namespace

hipError_t launch_fc_delta(int dtype, const void* x_t, void* x_snap, const void* wT, void* y, unsigned int* arrive,
                           const FcGeom& g, DevStats* stats, hipStream_t s) {
    const int esize = dtype == RRM_I8_I32 ? 1 : 2;
    dim3 block(FCD_THREADS);
    if (g.csc_ptr) {
        // pruned weights: up to 64 workgroups per stream share the list (each pays c_out atomic adds at the end)
        const int nw = std::max(1, std::min(64, NUM_CU / g.n));
        const size_t lds = ((size_t)g.c_out * 4 + 15) & ~(size_t)15;
        static std::once_flag once;
        static hipError_t attr = hipSuccess;
        std::call_once(once, [] {
            attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&fc_delta_kernel<RRM_I8_I32, true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, FC_CSC_MAX_LDS);
            if (attr == hipSuccess)
                attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&fc_delta_kernel<RRM_BF16_F32, true>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, FC_CSC_MAX_LDS);
        });
        if (attr != hipSuccess) return attr;
        if (lds > (size_t)FC_CSC_MAX_LDS) return hipErrorInvalidValue;
        dim3 grid((unsigned int)nw, (unsigned int)g.n, 1u);
        if (dtype == RRM_I8_I32)
            hipLaunchKernelGGL((fc_delta_kernel<RRM_I8_I32, true>), grid, block, lds, s, (const unsigned char*)x_t,
                               (unsigned char*)x_snap, (const unsigned char*)wT, y, arrive, g, stats);
        else
            hipLaunchKernelGGL((fc_delta_kernel<RRM_BF16_F32, true>), grid, block, lds, s, (const unsigned char*)x_t,
                               (unsigned char*)x_snap, (const unsigned char*)wT, y, arrive, g, stats);
        return hipGetLastError();
    }
    const int ranges = (g.c_out_p * esize + FCD_SEG - 1) / FCD_SEG;
    // integer layers with long input vectors: up to four list splits while that fills more of the chip's 256
    // compute units (measured: pays off from about a thousand changed columns; short vectors lose to the extra
    // workgroups' compare)
    const int nks = dtype == RRM_I8_I32 && g.c_in >= 8192 ? std::max(1, std::min(4, 256 / (ranges * g.n))) : 1;
    dim3 grid((unsigned int)ranges, (unsigned int)g.n, (unsigned int)nks);
    if (dtype == RRM_I8_I32)
        hipLaunchKernelGGL((fc_delta_kernel<RRM_I8_I32, false>), grid, block, 0, s, (const unsigned char*)x_t,
                           (unsigned char*)x_snap, (const unsigned char*)wT, y, arrive, g, stats);
    else
        hipLaunchKernelGGL((fc_delta_kernel<RRM_BF16_F32, false>), grid, block, 0, s, (const unsigned char*)x_t,
                           (unsigned char*)x_snap, (const unsigned char*)wT, y, arrive, g, stats);
    return hipGetLastError();
}

int fc_dense_slices(int dtype, const FcGeom& g) {
    const int pv = dtype == RRM_I8_I32 ? 16 : 8;
    return (g.c_out_p + FC_LANES * pv - 1) / (FC_LANES * pv);
}

hipError_t launch_fc_dense(int dtype, int splits, const void* wT, const void* x, void* part, const void* bias, void* y,
                           const FcGeom& g, hipStream_t s) {
    if (splits < 1 || splits > FC_MAX_SPLITS) return hipErrorInvalidValue;
    dim3 grid((unsigned int)fc_dense_slices(dtype, g), (unsigned int)splits, (unsigned int)g.n), block(FC_KG * FC_LANES);
    dim3 rgrid((unsigned int)((g.c_out_p / 4 + 15) / 16), (unsigned int)g.n), rblock(FC_MAX_SPLITS * 16);
    const unsigned char* w = static_cast<const unsigned char*>(wT);
    const unsigned char* xx = static_cast<const unsigned char*>(x);
    if (dtype == RRM_I8_I32) {
        hipLaunchKernelGGL(fc_dense_kernel<RRM_I8_I32>, grid, block, 0, s, w, xx, part, g, splits);
        hipLaunchKernelGGL(fc_reduce_kernel<RRM_I8_I32>, rgrid, rblock, 0, s, part, bias, y, g, splits);
    } else {
        hipLaunchKernelGGL(fc_dense_kernel<RRM_BF16_F32>, grid, block, 0, s, w, xx, part, g, splits);
        hipLaunchKernelGGL(fc_reduce_kernel<RRM_BF16_F32>, rgrid, rblock, 0, s, part, bias, y, g, splits);
    }
    return hipGetLastError();
}

// ---- the dense layer with its partial-sum scratch in a static device array ----------------------------------
// For callers that cannot allocate.  The array exists once per GPU the library runs on and is shared by every
// call on that GPU; its address is looked up once per device (the name below is a host-side stand-in, not a
// device address, so only the looked-up pointer is ever handed to a kernel).
static __device__ __align__(256) unsigned char scratch[FC_STATIC_SCRATCH_BYTES];

hipError_t launch_fc_dense_static(int dtype, int splits, const void* wT, const void* x, const void* bias, void* y,
                                  const FcGeom& g, hipStream_t s) {
    constexpr int MAX_DEV = 64;
    static std::mutex mu;
    static void* dev_ptr[MAX_DEV] = {};
    const size_t need = (size_t)g.n * (size_t)splits * (size_t)g.c_out_p * 4;
    if (need > FC_STATIC_SCRATCH_BYTES) return hipErrorInvalidValue;  // (the caller checks first, with a message)
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEV) return hipErrorInvalidDevice;
    void* ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(mu);
        if (!dev_ptr[dev]) {
            void* p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return e;
            if (!p) return hipErrorInvalidSymbol;
            dev_ptr[dev] = p;
        }
        ptr = dev_ptr[dev];
    }
    // every partial row that the reduction reads is written by the first kernel: nothing has to start at zero
    return launch_fc_dense(dtype, splits, wT, x, ptr, bias, y, g, s);
}

}  // namespace rrm
