// Geometry of the position-gather convolution and the choice of its work-unit shape.  Plain host C++ (no HIP
// types): the kernel, the dispatcher and a host-only test include it.
#pragma once
#include <stddef.h>

#include "rrm.h"

namespace rrm {

constexpr int POS_NUM_CU = 256;  // compute units of the MI355X
constexpr int POS_LDS_BUDGET = 160 * 1024 - 1024;  // dynamic LDS of a workgroup: a compute unit's, minus statics

// Geometry of the position-gather convolution (conv_pos.hip): stride 1, channel runs of 16-byte multiples.
constexpr int POS_THREADS = 512;  // 4 consumer + 4 producer wavefronts
constexpr int POS_PROD = 256;     // producer threads
constexpr int POS_NCB = 4;     // 32-channel blocks per workgroup
constexpr int POS_MAXU = 10;   // staged 16-byte units per producer thread and slab
constexpr int POS_MAXO = 2;    // output positions per thread and work unit
constexpr int POS_COLS = 256;  // columns (output positions) per pass of a workgroup
constexpr int POS_ABUF = 2;    // weight stages in LDS: copies run one stage ahead of the multiplications
struct PosGeom {
    int n, h, w, c_out, kh, kw, pad, groups;
    int ho, wo, og, cg;
    int pos_bytes;       // bytes of one input position (all groups)
    int grp_bytes;       // bytes of one group's channels of a position
    int chunks;          // 16-byte chunks per (position, group): ceil
    int nslab;           // K slabs of 2 chunks
    int ntaps;           // kh * kw
    int ts;              // taps per stage (weights of one stage: ts * POS_NCB KiB in LDS)
    int nstage;          // stages per slab: ceil(ntaps / ts)
    int G, R;            // work unit: G consecutive streams x R output rows (x POS_NCB channel blocks)
    int RB, WP;          // band rows with halo: R + kh - 1; row pitch in positions: w + pad
    int npos;            // staged positions per unit: G * RB * WP + pad
    int nbands;          // ceil(ho / R)
    int nsg;             // ceil(n / G)
    int ncg;             // channel groups (POS_NCB blocks) per filter group
    int total_units;     // nsg * nbands * groups * ncg
    int a_stage_bytes;   // ts * POS_NCB * 1024
    int b_plane_bytes;   // npos * 32, rounded up to 16
    int act_bytes;       // npos rounded up to 16
    int col_cap;         // column list capacity: G * R * wo rounded up to 8
    int full_pct;        // delta launches: units with more than this percentage of active positions recompute
    const unsigned char* xfull;  //   their band from the committed input (nullptr: never)
    unsigned int* fresh;         // see FusedSrc::fresh: cleared at the end of a delta launch
    unsigned int* touched_all;   // see FusedSrc::touched_all: cleared at the end of a delta launch
    unsigned char* touched;      // one byte per output position: written by the last delta step (or nullptr)
};

// dynamic LDS of the position-gather kernel
inline size_t conv_pos_lds_bytes(const PosGeom& g, int terms) {
    return POS_ABUF * (size_t)g.a_stage_bytes + 2 * (size_t)terms * g.b_plane_bytes + (size_t)g.act_bytes + (size_t)g.col_cap * 6;
}

// Fill the geometry of a layer (esize = bytes per input element, terms = difference planes staged per band);
// false if the layer cannot run on the position-gather kernel.
inline bool pos_choose_shape(const rrm_shape& s, int esize, int terms, PosGeom& g) {
    const int cg = s.c_in / s.groups, og = s.c_out / s.groups;
    if (s.stride != 1 || (cg * esize) % 16 != 0 || og % 4 != 0 || s.c_out % 4 != 0) return false;
    g.n = s.n; g.h = s.h; g.w = s.w; g.c_out = s.c_out; g.kh = s.kh; g.kw = s.kw; g.pad = s.pad; g.groups = s.groups;
    g.ho = s.h + 2 * s.pad - s.kh + 1;
    g.wo = s.w + 2 * s.pad - s.kw + 1;
    g.og = og; g.cg = cg;
    g.pos_bytes = s.c_in * esize;
    g.grp_bytes = cg * esize;
    g.chunks = g.grp_bytes / 16;
    g.nslab = (g.chunks + 1) / 2;
    g.ntaps = s.kh * s.kw;
    // taps per stage: the whole window if its weights (POS_NCB KiB per tap) stay within 36 KiB, else a filter row
    g.ts = g.ntaps <= 9 ? g.ntaps : (s.kw <= 5 ? s.kw : 4);
    g.nstage = (g.ntaps + g.ts - 1) / g.ts;
    g.a_stage_bytes = g.ts * POS_NCB * 1024;
    g.WP = s.w + s.pad;
    g.ncg = (og + POS_NCB * 32 - 1) / (POS_NCB * 32);
    if (s.kh > 64 || g.WP > 32000 || g.ho < 1 || g.wo < 1) return false;
    const long long budget = (long long)POS_LDS_BUDGET - (long long)POS_ABUF * g.a_stage_bytes;
    // per staged position: two buffers x terms x 32 bytes and one flag; per output position: 6 bytes of column list
    auto fits = [&](int G, int R) {
        const long long RB = R + s.kh - 1, npos = (long long)G * RB * g.WP + s.pad, ncol = (long long)G * R * g.wo;
        if (npos * 2 > (long long)POS_PROD * POS_MAXU || ncol > (long long)POS_THREADS * POS_MAXO || G > 255 || RB > 255)
            return false;
        return npos * (2 * terms * 32) + 32 * terms + npos + 16 + (ncol + 8) * 6 <= budget;
    };
    const long long chan_units = (long long)s.groups * g.ncg;
    int G = 1, R = 0;
    if (fits(1, g.ho)) {
        // Whole maps, G streams per unit: the G that needs the fewest rounds of the chip's compute units per stream
        // (a unit costs about G; rounds = ceil(units / compute units)).
        R = g.ho;
        long long best = -1;
        for (int c = 1; c <= s.n && fits(c, R); ++c) {
            const long long units = (long long)((s.n + c - 1) / c) * chan_units;
            const long long cost = ((units + POS_NUM_CU - 1) / POS_NUM_CU) * c;
            // (ties: the largest G whose unit still holds at most one and a half passes of columns: more, smaller
            // units balance better when their costs differ, fuller passes multiply better)
            if (best < 0 || cost < best || (cost == best && (long long)c * R * g.wo <= POS_COLS + POS_COLS / 2)) {
                best = cost;
                G = c;
            }
        }
    } else {
        int rmax = 0;
        for (int r = 1; r <= g.ho && fits(1, r); ++r) rmax = r;
        if (rmax == 0) return false;  // not even one row fits
        const int nb = (g.ho + rmax - 1) / rmax;
        R = (g.ho + nb - 1) / nb;
    }
    // few units in all (one stream of a small map): thinner bands spread the work over more compute units
    for (int nb = (g.ho + R - 1) / R + 1;
         R > 1 && (long long)((s.n + G - 1) / G) * ((g.ho + R - 1) / R) * chan_units < POS_NUM_CU; ++nb)
        R = (g.ho + nb - 1) / nb;  // (rows spread evenly over nb bands; ends at one row per band at the latest)
    g.G = G; g.R = R;
    g.RB = R + s.kh - 1;
    g.npos = G * g.RB * g.WP + s.pad;
    g.nbands = (g.ho + R - 1) / R;
    g.nsg = (s.n + G - 1) / G;
    g.total_units = (int)((long long)g.nsg * g.nbands * chan_units);
    g.b_plane_bytes = (g.npos * 32 + 15) & ~15;
    g.act_bytes = (g.npos + 15) & ~15;
    g.col_cap = (G * R * g.wo + 7) & ~7;
    return (long long)conv_pos_lds_bytes(g, terms) <= POS_LDS_BUDGET;
}

}  // namespace rrm
