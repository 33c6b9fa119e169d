// Geometry of the binary (XNOR / popcount) convolution and the choice of the band kernel's bands.  Plain host C++
// (no HIP types): the kernels, the dispatcher and a host-only test include it.
#pragma once
#include <stddef.h>

#include "rrm.h"

namespace rrm {

constexpr int BIN_TILE = 8;        // output tile edge of the tile kernel
constexpr long long BIN_TILE_MAX_LDS = 152 * 1024;  // both window copies of one tile (160 KB per workgroup, less static use)
constexpr int BIN_NUM_CU = 256;    // compute units of the MI355X

struct BinGeom {
    int n, h, w, c_out, kh, kw, stride, pad, groups;
    int wpp;             // 32-bit words per input position (all groups)
    int wg;              // words per position per group
    int og;              // output channels per group
    int ho, wo, tiles_y, tiles_x;
    int th_in, tw_in;
    int pitch;           // LDS words per staged position
    int nslab;           // word slabs of 4 per group
    int nob8;            // packed 8-channel filter blocks per group (og padded to 16)
    unsigned int magic_wg4;    // floor(2^32/d)+1 for d = 4*nslab
    unsigned int magic_tw;     // same for d = tw_in
    // band kernel (delta step): bands of band_rows output rows over the full width; 0 rows = the layer's bands
    // do not fit LDS and the delta step runs the tile kernel
    int band_rows, nbands, bth_in, btw_in;
    unsigned int magic_btw;    // same for d = btw_in
    unsigned int magic_nslab;  // same for d = nslab
    int vec4;                  // 1: a group's words per position are whole 16-byte vectors (wg % 4 == 0, wpp % 4 == 0)
    int fused_ok;              // 1: the band kernel can run the whole step (compare and commit included)
    int wlds;                  // 1: the band kernel keeps its workgroup's filter words in LDS
};


inline unsigned int bin_magic_for(int d) { return d <= 1 ? 0u : (unsigned int)((1ull << 32) / (unsigned long long)d + 1ull); }

// dynamic LDS of a band-kernel workgroup with bands of band_rows output rows: the A and B words of the band's input
// window, one flag byte per window position, the list of active output positions (16 bits each), and (wlds) the
// filter words of 64 output channels
inline size_t bin_band_lds_bytes(const BinGeom& g, int band_rows) {
    const size_t npos = (size_t)((band_rows - 1) * g.stride + g.kh) * (size_t)((g.wo - 1) * g.stride + g.kw);
    const size_t wl = g.wlds ? (size_t)g.nslab * g.kh * g.kw * 64 * 16 : 0;
    return 2 * npos * g.pitch * 4 + ((npos + 15) & ~(size_t)15) + (((size_t)band_rows * g.wo * 2 + 15) & ~(size_t)15) + wl;
}

// Fill the geometry of a binary layer.  False: the input window of one 8x8 output tile does not fit LDS (the layer
// cannot be created).
inline bool bin_choose_shape(const rrm_shape& s, BinGeom& g) {
    g.n = s.n; g.h = s.h; g.w = s.w; g.c_out = s.c_out; g.kh = s.kh; g.kw = s.kw;
    g.stride = s.stride; g.pad = s.pad; g.groups = s.groups;
    g.wpp = s.c_in / 32;
    g.wg = g.wpp / s.groups;
    g.og = s.c_out / s.groups;
    g.ho = (s.h + 2 * s.pad - s.kh) / s.stride + 1;
    g.wo = (s.w + 2 * s.pad - s.kw) / s.stride + 1;
    g.tiles_y = (g.ho + BIN_TILE - 1) / BIN_TILE;
    g.tiles_x = (g.wo + BIN_TILE - 1) / BIN_TILE;
    g.th_in = (BIN_TILE - 1) * s.stride + s.kh;
    g.tw_in = (BIN_TILE - 1) * s.stride + s.kw;
    g.nslab = (g.wg + 3) / 4;
    g.pitch = g.nslab * 4 + 4;
    g.nob8 = 2 * ((g.og + 15) / 16);
    g.magic_wg4 = bin_magic_for(g.nslab * 4);
    g.magic_tw = bin_magic_for(g.tw_in);
    if ((long long)2 * g.th_in * g.tw_in * g.pitch * 4 > BIN_TILE_MAX_LDS) return false;
    // delta step: bands of output rows whose window, flags and list fit the LDS budget (two workgroups per compute
    // unit); as tall as fits when the streams alone fill the chip (a tall band wastes least on its halo rows and
    // fills its 64-lane chunks best), shorter -- down to 4 rows -- while there are fewer than two workgroups per
    // compute unit; no band at all = the tile kernel
    // (the filter words of a workgroup's 64 channels go to LDS too when they take at most 40 KB; the budget is then
    // 79 KB per workgroup, still two per compute unit)
    g.wlds = (long long)g.nslab * s.kh * s.kw * 1024 <= 40 * 1024 ? 1 : 0;
    const long long band_budget = g.wlds ? 79 * 1024 : 64 * 1024 - 64;
    g.band_rows = 0;
    for (int r = g.ho; r >= 1; --r)
        if ((long long)bin_band_lds_bytes(g, r) <= band_budget && (long long)r * g.wo <= 65535) {
            g.band_rows = r;
            break;
        }
    g.nbands = 1;
    if (g.band_rows > 0) {
        g.nbands = (g.ho + g.band_rows - 1) / g.band_rows;
        const long long per_band = (long long)g.n * g.groups * ((g.og + 63) / 64);
        while (per_band * g.nbands < 2 * BIN_NUM_CU && (g.ho + g.nbands) / (g.nbands + 1) >= 4) ++g.nbands;
        g.band_rows = (g.ho + g.nbands - 1) / g.nbands;
        g.nbands = (g.ho + g.band_rows - 1) / g.band_rows;
    }
    if ((long long)g.n * g.nbands > 65535) g.band_rows = 0;  // (stream x band is the grid's z dimension)
    g.vec4 = (g.wg % 4 == 0 && g.wpp % 4 == 0) ? 1 : 0;
    g.magic_nslab = bin_magic_for(g.nslab);
    g.bth_in = ((g.band_rows > 1 ? g.band_rows : 1) - 1) * s.stride + s.kh;
    g.btw_in = (g.wo - 1) * s.stride + s.kw;
    g.magic_btw = bin_magic_for(g.btw_in);
    // The band kernel can run the whole step in one launch when every input position lies inside the window of
    // the band that owns its row (band k owns input rows k*R*stride .. (k+1)*R*stride - 1, the last band the rest):
    // then each position is compared and counted exactly once, and whole 16-byte vectors are compared.
    g.fused_ok = 0;
    if (g.band_rows > 0 && g.vec4) {
        const bool cols = g.btw_in - s.pad >= s.w;
        const bool rows_mid = g.nbands == 1 || s.stride <= s.kh - s.pad;
        const bool rows_last = (g.nbands - 1) * g.band_rows * s.stride - s.pad + g.bth_in >= s.h;
        g.fused_ok = (cols && rows_mid && rows_last) ? 1 : 0;
    }
    return true;
}

}  // namespace rrm
