// Internal declarations shared by the host dispatcher and the gfx950 kernels of the RRM
// library.  Nothing here is part of the public ABI (see include/rrm.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rrm.h"
#include "bin_shape.h"
#include "pos_shape.h"

namespace rrm {

constexpr int TILE = 8;          // output tile side of the binary kernel (positions)
constexpr int WAVE = 64;
constexpr int CONV_THREADS = 256;
constexpr int NUM_CU = 256;       // compute units of the MI355X

enum Mode : int { MODE_DELTA = 0, MODE_DENSE = 1 };

// Device-side counters (totals), updated with atomics by the kernels.  There are STAT_SLOTS copies
// (a workgroup uses slot blockIdx.x % STAT_SLOTS) so that same-address atomics do not serialise
// the scan; rrm_get_stats sums them.
constexpr int STAT_SLOTS = 256;
struct DevStats {
    unsigned long long changed_elems;
    unsigned long long changed_units;
    unsigned long long active_tiles;
    unsigned int range_error;
    unsigned int pad_;
    unsigned long long truncated_elems;  // bf16 with a threshold: differences below it (not applied, not committed)
    double truncated_sumsq;              //   and the sum of their squares
    // counted on the device (by the scan of every delta step), so that they advance under graph replay too
    unsigned long long delta_steps;
    unsigned long long total_tiles;
};

// Geometry of the flat scan over x (delta + change map), one element = int8 / bf16 / u32 word.
struct ScanGeom {
    long long total_elems;   // n*h*w*c (binary: words)
    int c;                   // elements per position
    int h, w;                // input map
    int kh, kw, stride, pad;
    int ho, wo;
    int tiles_y, tiles_x;    // 8x8 output tiles (binary path: stamped words)
    int sty, stx;            // 4x4 output sub-tiles (MFMA path: one byte flag each)
    int per_vec;             // elements per 16-byte unit: 16 / 8 / 4
    // Layout of the difference buffer.  scatter == 0: same as x (16-byte units map one to one).
    // scatter == 1: element (row r = b*h + iy, column ix, channel c) goes to element
    // ((r*wp + ix)*groups + c / cg)*cp + c % cg, i.e. rows padded to wp columns and every group's
    // channels padded to cp, so that the gather kernel only ever sees whole 16-byte chunks.
    int scatter, wp, cp, cg, groups;
    // reciprocals for the scan's index arithmetic: doubles for dividends up to 2^30 (see udiv_big), a
    // 32-bit one for the small dividends of the receptive-field bounds (floor(2^32/stride)+1, 0 for 1)
    double r_c, r_hw, r_w;
    unsigned int magic_stride;
    float eps;  // bf16: truncation threshold of the difference (0 = exact)
    unsigned long long tiles_per_step;  // what a dense step would count as "tiles" (added to the device counters)
};

// A scan whose input is not a tensor in memory but f(P) of the layer before (Algorithm 1 applies the
// non-linear map f to the projection and feeds the result to the next layer): ReLU, right shift, clamp to 127
// and optional 3x3 / 2 max pooling of the producer's stored int32 projection, computed per 16-byte unit, and
// only under the 4x4 blocks of the projection that the producer's last step wrote.
struct FusedSrc {
    const int* y;                 // producer's stored projection [n][hy][wy][c], c = this layer's c_in
    const unsigned char* touched; // producer's byte flags per block of (1 << tshift)^2 positions of (hy, wy)
    int hy, wy, sty, stx;         // sty x stx blocks per image
    int tshift;                   // 2: 4x4 blocks (window-tile kernel), 0: single positions (position-gather kernel)
    int shift, pool;
    // device word, non-zero while the consumer's stored input holds no f(P) yet (fresh or reset layer): `touched`
    // is ignored and every unit is computed and compared.  Set by create / reset, cleared by the consumer's
    // compute kernel at the end of its first delta step (device state: a replayed graph sees it too).
    const unsigned int* fresh;
    // device word, non-zero after a step of the producer that kept no flags (the single-launch scatter path):
    // `touched` is ignored then as well.  Cleared by the producer's next flag-keeping step.
    const unsigned int* touched_all;
};

constexpr int CONV_MAX_STAGE_UNITS = 12;  // 16-byte units a thread stages per slab (half for 2 terms)

// Geometry of the gather-tile implicit-GEMM convolution (int8 / bf16 MFMA path).
struct ConvGeom {
    int n, h, w, c_in, c_out, kh, kw, stride, pad, groups;
    int ho, wo, cg, og;
    // The source as the kernel sees it: a map of src_h x src_w "source positions" of pos_bytes bytes
    // (groups x chunks x 16), with its own strides, padding and window.  For layers with 16-byte
    // channel runs this is x itself.  For few-channel layers `fold` neighbouring columns share one
    // 16-byte chunk (a filter row becomes ceil(kw/fold) taps of 16 bytes).
    int src_h, src_w, str_y, str_x, pad_y, pad_x;
    int pos_bytes, grp_bytes;
    int fold;            // columns per source position (1 unless folded)
    int cp;              // channels per group and column in the source layout
    int wp;              // columns per row in the source layout (w, or w rounded up to fold)
    int kw_eff;          // filter taps per row in source positions: ceil(kw / fold)
    int aligned;         // 1: the source layout is the caller's x layout
    int sty, stx;        // 4x4 output sub-tiles per image
    int n_sub;           // n*sty*stx
    int n_words;         // 32-bit words of the sub-tile flag array (4 byte flags per word)
    int wh, ww;          // input window of one sub-tile: 3*stride + kh, 3*stride + kw
    int wpos;            // wh*ww
    int per_vec;         // elements per 16-byte K chunk (16 int8 / 8 bf16)
    int chunks;          // 16-byte chunks per (position, group): ceil(cg / per_vec)
    int sc;              // chunks per LDS slab
    int nslab;           // ceil(chunks / sc)
    int pitch;           // LDS bytes per staged position: 16*sc
    int slot_bytes;      // wpos*pitch: LDS bytes of one sub-tile's window
    // Bank spreading: within a staged position the first rot_p chunks (a power of two) are rotated by
    // rot_a * (row / str_y) + rot_b * (column / str_x), so that the 16 positions of a sub-tile read
    // different LDS banks for the same (tap, chunk); the reader splits the rotation into a per-lane and a
    // per-tap term (the tap's term is folded into the K-pair table).
    int rot_p, rot_a, rot_b;
    unsigned int magic_sy, magic_sx;  // reciprocals of str_y, str_x
    int last_sc;         // chunks present in the last slab
    int nq;              // K steps (4 K pairs = 2 MFMAs deep) per slab: ceil(kh*kw*sc / 4)
    int ncb;             // 32-wide output-channel blocks per group
    int wg_cb, nt;       // workgroup shape: 32-channel blocks (1 or 2) and gathered sub-tiles (8, 16)
    unsigned int magic_sc[2];   // reciprocals (floor(2^32/d)+1, 0 for d = 1): [0] d = sc
    unsigned int magic_wsc[2];  // [0] d = wpos
    unsigned int magic_wo, magic_ho;  // d = wo, d = ho
    unsigned int magic_ww;      // d = ww
    unsigned int magic_sub;     // d = sty*stx
    unsigned int magic_stx;     // d = stx
    int vec_store;       // 1: y rows allow 16-byte read-modify-write
    unsigned int* fresh;    // see FusedSrc::fresh: cleared at the end of a delta launch
    unsigned int* touched_all;  // see FusedSrc::touched_all: cleared at the end of a delta launch
    unsigned int* touched;  // copy of the sub-tile flags of the last delta step (what it wrote in y), or nullptr
    const unsigned char* xfull;  // delta launches: the committed input in source layout (full recomputation above
    int full_pct;                //   full_pct % active sub-tiles), or nullptr: never
    int xcd_gy;          // set by the launcher: 0 = two-dimensional grid, else the channel-block groups of a
                         // one-dimensional grid dealt XCD by XCD
};

// Geometry of the single-launch scatter convolution (conv_scatter.hip).
constexpr int SCAT_UPT = 8;  // 16-byte units of x per thread of a position block at most
struct ScatGeom {
    int n, h, w, c_out, kh, kw, stride, pad, groups;
    int ho, wo, og;
    int U;               // 16-byte units per input position (all groups)
    int ug;              // units per group
    int nk;              // K steps (2 units each) per group: ceil(ug / 2)
    int nkp;             // parts of at most 8 K steps: ceil(nk / 8)
    int ncb;             // 32-channel output blocks per group
    int npair;           // groups * ncb: (group, channel block) pairs
    int ntaps;           // kh * kw
    int PB;              // input positions per block (at most 64)
    int cs;              // work-item splits: workgroups per position block
    long long npos_total;  // n * h * w
    float eps;           // bf16: truncation threshold of the difference (0 = exact)
    unsigned int* arrive;       // one word per position block (used when cs > 1; rearmed by the kernel)
    unsigned int* touched_all;  // device word set by every step of this path: "treat every output as written"
};

struct FcGeom {
    int n, c_in, c_out;
    int c_out_p;         // row pitch of the transposed weights (elements), multiple of per_vec
    int per_vec;         // output channels per lane per 16-byte load: 16 / 8
    int vec_ok;          // 1: x rows are 16-byte aligned multiples
    float eps;           // bf16: truncation threshold of the difference (0 = exact)
    // pruned weights (delta step only): column j of W holds the non-zeros csc_ptr[j] .. csc_ptr[j + 1] - 1, each a
    // row index and a value (int8 / bf16 bits); csc_ptr == nullptr = the dense columns are walked
    const unsigned int* csc_ptr;
    const unsigned short* csc_row;
    const void* csc_val;
};
constexpr int FC_BATCH_MIN_STREAMS = 16;    // from this many streams on an FC layer runs as one product on the matrix cores
constexpr int FC_BATCH_MAX_STREAMS = 4096;  // (launched in groups of at most 128 streams)
constexpr int FC_CSC_MAX_LDS = 96 * 1024;   // the pruned-weight kernel's update accumulators: c_out <= 24576

// floor(u / d) through the reciprocal magic = floor(2^32 / d) + 1 (0 encodes d == 1).  The product's high word is
// the quotient or one more than it for every u < 2^32 - d (the reciprocal is rounded up), so one
// multiply-and-compare makes the result exact over the whole admitted range; without it the estimate is only
// right while u * (magic * d - 2^32) < 2^32.
#ifdef __HIPCC__
__device__ __forceinline__ unsigned int udiv_magic(unsigned int u, unsigned int d, unsigned int magic) {
    if (!magic) return u;
    const unsigned int q = __umulhi(u, magic);
    return q * d > u ? q - 1u : q;
}
#endif

// ---- launchers implemented in the kernel translation units ------------------------------------
// `marks` is the 8x8-tile stamp array (binary layers, stamp = consumers per tile) or the 4x4
// sub-tile byte-flag array (int8 / bf16 layers, stamp ignored)
hipError_t launch_scan(int dtype, const void* x_t, void* x_snap, void* d0, void* d1, unsigned long long* bitmap,
                       unsigned int* marks, unsigned int stamp, const ScanGeom& g, DevStats* stats,
                       hipStream_t s);
// the same scan with the input computed from the producer's projection (int8 layers in the kernel's own
// layout, c_in a multiple of 16)
hipError_t launch_scan_fused(const FusedSrc& src, void* x_snap, void* d0, unsigned long long* bitmap, unsigned int* marks,
                             const ScanGeom& g, DevStats* stats, hipStream_t s);

size_t conv_lds_bytes(const ConvGeom& g, int ncb, int nt, int terms);  // dynamic LDS of the gather kernel
hipError_t launch_conv(int dtype, int mode, int ncb, int nt, int terms, const void* src0, const void* src1,
                       const void* zero16, unsigned int* subbits, unsigned int* ctrl, const void* wpack, const int* offtab,
                       const void* bias, void* y, const ConvGeom& g, DevStats* stats, hipStream_t s);

// `bitmap`: the scan's changed-unit bitmap (delta mode); ctrl: 4 zeroed words (rearmed by the kernel)
hipError_t launch_conv_pos(int dtype, int mode, int terms, const void* src0, const void* src1, const void* zero16,
                           const unsigned long long* bitmap, unsigned int* ctrl, const void* wpack, const void* bias, void* y,
                           const PosGeom& g, DevStats* stats, hipStream_t s);

// one delta step of a convolution layer in a single launch (compare, products of the changed positions, atomic
// accumulation, commit); wsc: weights in [pair][tap][K step][lane] x 16 bytes order
hipError_t launch_conv_scatter(int dtype, int terms, const void* x_t, void* x_snap, const void* wsc, void* y,
                               const ScatGeom& g, DevStats* stats, hipStream_t s);

// one delta step of an FC layer in a single launch; `arrive`: one zeroed word per stream (rearmed by the kernel)
hipError_t launch_fc_delta(int dtype, const void* x_t, void* x_snap, const void* wT, void* y, unsigned int* arrive,
                           const FcGeom& g, DevStats* stats, hipStream_t s);

// dense FC layer: row/slice split into per-split partial sums (scratch `part`: [n][splits][c_out_p] 4-byte
// values), then y = bias + the sum of the splits in a fixed order
bool fc_batched_ok(int dtype, const FcGeom& g);
int fc_batched_splits(int dtype, const FcGeom& g);  // splits of the k range; part: [splits][n][c_out] 4-byte sums
hipError_t launch_fc_batched_dense(int dtype, const void* w_rm, const void* x, void* part, const void* bias, void* y,
                                   const FcGeom& g, hipStream_t s);
hipError_t launch_fc_batched_delta(int dtype, const void* w_rm, const void* x_t, void* x_snap, void* d0, void* part,
                                   const void* bias, void* y, const FcGeom& g, DevStats* stats, hipStream_t s);
int fc_dense_slices(int dtype, const FcGeom& g);
hipError_t launch_fc_dense(int dtype, int splits, const void* wT, const void* x, void* part, const void* bias, void* y,
                           const FcGeom& g, hipStream_t s);
// the same with the partial sums in a static device array of FC_STATIC_SCRATCH_BYTES (no allocation anywhere)
constexpr size_t FC_STATIC_SCRATCH_BYTES = 4u << 20;
hipError_t launch_fc_dense_static(int dtype, int splits, const void* wT, const void* x, const void* bias, void* y,
                                  const FcGeom& g, hipStream_t s);

hipError_t launch_bin_conv(int mode, int cw, const void* xsrc, const void* flip, unsigned int* tileflag,
                           const void* wpack, const void* bias, void* y, const BinGeom& g, DevStats* stats,
                           hipStream_t s);
int bin_consumers(int cw, const BinGeom& g);     // workgroups per tile of the binary kernel
hipError_t launch_bin_band(int cw, const void* xsrc, const void* flip, const void* wpack, void* y, const BinGeom& g,
                           DevStats* stats, hipStream_t s);
hipError_t launch_bin_band_fused(int cw, const void* x_t, void* x_snap, unsigned int* arrive, const void* wpack, void* y,
                                 const BinGeom& g, DevStats* stats, hipStream_t s);

hipError_t launch_fill_bias(int is_float, void* y, const void* bias, long long rows, int c_out, hipStream_t s);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s);
// x (caller layout) -> the padded / folded source layout described by g (pad elements are left untouched)
hipError_t launch_repack(int esize, const void* x, void* dst, const ScanGeom& g, hipStream_t s);
hipError_t launch_fill_word(void* p, size_t bytes, unsigned int word, hipStream_t s);
// touched: nullptr = every output; else byte flags per block of (1 << tshift)^2 positions of y, only outputs under
// a set flag (every output again while the device word *touched_all is non-zero)
hipError_t launch_probe_mfma(int is_bf16, void* sink, int iters, int workgroups, hipStream_t s);
hipError_t launch_probe_copy(void* dst, const void* src, size_t bytes, hipStream_t s);
hipError_t launch_relu_requant_pool(const void* y, void* out, const void* touched, const unsigned int* touched_all,
                                    int tshift, int n, int h, int w, int c, int shift, int pool, hipStream_t s);

}  // namespace rrm
