// Host dispatcher and C ABI of the RRM library (see include/rrm.h for the contract).
//
// A handle owns: the layer's weights repacked for the kernels that read them, the bias, the two
// snapshots of Sec. 3.2 (stored input I_{t-1}, stored projection P_{t-1}) and the scratch of the
// change map (difference buffer, bitmap, tile stamps, FC column list).  rrm_step enqueues
//   convolution   scan (delta + change map + commit)  ->  tile kernel on stamped tiles
//   FC            scan + ordered compaction           ->  column scatter
// and never touches the host side of the stream.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "rrm_internal.h"

using namespace rrm;

namespace {

thread_local std::string g_last_error;

rrm_status fail(rrm_status st, const std::string& msg) {
    g_last_error = msg;
    return st;
}

#define RRM_HIP(expr)                                                                                       \
    do {                                                                                                    \
        hipError_t e_ = (expr);                                                                             \
        if (e_ != hipSuccess)                                                                               \
            return fail(RRM_ERR_HIP, std::string(#expr) + ": " + hipGetErrorString(e_));                    \
    } while (0)

size_t round16(size_t b) { return (b + 15) & ~size_t(15); }

}  // namespace

struct rrm_layer {
    rrm_shape shape{};
    int dtype = 0;
    int esize = 1;          // bytes per input element (binary: per 32-bit word)
    long long x_elems = 0;  // elements of x (binary: words)
    long long y_elems = 0;
    size_t x_bytes = 0, y_bytes = 0;
    size_t d_bytes = 0;     // bytes of one difference buffer
    ScanGeom sg{};
    ConvGeom cg{};
    PosGeom pg{};           // position-gather kernel (stride-1 layers with 16-byte channel runs)
    bool pos_ok = false;    // the layer can run on the position-gather kernel
    bool use_pos = false;   // ... and does
    int tshift = 2;         // log2 of the side of the output blocks that `touched` flags: 2 (4x4) or 0 (positions)
    void* wpos = nullptr;   // weights packed for the position-gather kernel
    ScatGeom sc{};          // single-launch scatter path
    bool scat_ok = false;   // the layer can run on it
    bool scat_auto = false; // ... and does when "path" is automatic
    void* wsc = nullptr;    // weights packed for it
    unsigned int* sc_arrive = nullptr;  // its arrival counters (one per position block)
    unsigned int* bin_arrive = nullptr;  // binary single-launch step: arrival counter per stream
    size_t touched_bytes = 0;
    BinGeom bg{};
    FcGeom fg{};
    // device memory
    void* wpack = nullptr;   // conv: MFMA fragment order; FC: W^T; binary: scalar-load order
    int* offtab = nullptr;   // conv: K-pair table of a slab, then the staging table of a workgroup
    void* bias = nullptr;
    void* x_snap = nullptr;
    void* y_snap = nullptr;
    void* d0 = nullptr;      // difference (bf16: head; binary: flip mask)
    void* d1 = nullptr;      // bf16: tail of the difference
    void* xpad = nullptr;    // dense path of layers whose channel runs are not 16-byte multiples: repacked x
    unsigned long long* bitmap = nullptr;
    unsigned int* tileflag = nullptr;  // binary: 8x8 tile stamps; int8 / bf16: 4x4 sub-tile byte flags
    unsigned int* touched = nullptr;   // int8 / bf16 conv: the sub-tile flags of the last step (what it wrote in y_snap)
    size_t marks_bytes = 0;
    unsigned int* ctrl = nullptr;      // arrival counter of the gather kernel
    unsigned int* fresh = nullptr;     // conv: device word, non-zero until the first delta step has run (see FusedSrc)
    void* zero16 = nullptr;            // a block of zeros: source of staged units outside the image
    unsigned int* fc_arrive = nullptr;  // FC delta step: arrival counter per stream
    void* fc_bpart = nullptr; // FC as one product (many streams): the k splits' partial sums [splits][n][c_out]
    void* fc_part = nullptr;  // FC dense path: per-split partial sums [n][fc_nsplit][c_out_p]
    void *csc_ptr = nullptr, *csc_row = nullptr, *csc_val = nullptr;  // FC, pruned weights: non-zeros by column
    void* w_rm = nullptr;     // FC with many streams: W in its own row-major layout, for the batched product
    int opt_fc_batched = 1;
    bool csc_ok = false, use_csc = false;
    double w_density = 1.0;  // FC: share of non-zero weights
    int fc_nsplit = 0;
    DevStats* stats = nullptr;
    // state
    bool has_snapshot = false;
    unsigned long long steps = 0;  // rrm_step calls enqueued by the host
    // event brackets of the "profile" option: 3 events per step (before scan, between, after)
    std::vector<hipEvent_t> prof_ev;
    int prof_n = 0;
    bool prof_on = false;
    // options
    int opt_path = 0, opt_wm = 0, opt_fc_splits = 0, opt_terms = 2, opt_bin_cw = 0, opt_conv_kernel = 0, opt_bin_fused = 1;

    ~rrm_layer() {
        void* ptrs[] = {wpack, wpos, wsc, sc_arrive, bin_arrive, offtab, bias, x_snap, y_snap, d0, d1, xpad, bitmap, tileflag, touched, ctrl, fresh, zero16, fc_arrive, fc_part, fc_bpart, csc_ptr, csc_row, csc_val, w_rm, stats};
        for (void* p : ptrs)
            if (p) (void)hipFree(p);
        for (hipEvent_t e : prof_ev) (void)hipEventDestroy(e);
    }
};

namespace {

rrm_status validate(const rrm_shape* s, int dtype) {
    if (dtype != RRM_I8_I32 && dtype != RRM_BF16_F32 && dtype != RRM_BIN_I32)
        return fail(RRM_ERR_DTYPE, "unknown dtype");
    if (s->kind != RRM_CONV && s->kind != RRM_FC) return fail(RRM_ERR_SHAPE, "kind must be RRM_CONV or RRM_FC");
    if (s->n < 1 || s->c_in < 1 || s->c_out < 1) return fail(RRM_ERR_SHAPE, "n, c_in, c_out must be positive");
    if (s->kind == RRM_FC) {
        if (dtype == RRM_BIN_I32) return fail(RRM_ERR_DTYPE, "binary layers are convolutions only");
        if ((long long)s->n * s->c_in > (1ll << 30) || (long long)s->c_in * s->c_out > (1ll << 32))
            return fail(RRM_ERR_SHAPE, "FC layer too large");
        return RRM_OK;
    }
    if (s->h < 1 || s->w < 1 || s->kh < 1 || s->kw < 1 || s->stride < 1 || s->pad < 0 || s->groups < 1)
        return fail(RRM_ERR_SHAPE, "h, w, kh, kw, stride, groups must be positive and pad non-negative");
    if (s->c_in % s->groups || s->c_out % s->groups) return fail(RRM_ERR_SHAPE, "groups must divide c_in and c_out");
    if (s->h + 2 * s->pad < s->kh || s->w + 2 * s->pad < s->kw)
        return fail(RRM_ERR_SHAPE, "filter window larger than the padded input");
    if (dtype == RRM_BIN_I32 && ((s->c_in / s->groups) % 32))
        return fail(RRM_ERR_SHAPE, "binary layers need c_in/groups to be a multiple of 32");
    const long long ho = (s->h + 2 * s->pad - s->kh) / s->stride + 1, wo = (s->w + 2 * s->pad - s->kw) / s->stride + 1;
    // 32-bit byte offsets inside the kernels
    if ((long long)s->n * s->h * s->w * s->c_in > (1ll << 30) || (long long)s->n * ho * wo * s->c_out > (1ll << 30))
        return fail(RRM_ERR_SHAPE, "tensor too large");
    if ((long long)s->kh * s->kw > 4096) return fail(RRM_ERR_SHAPE, "filter window too large");
    return RRM_OK;
}

// copy `bytes` from a host-or-device pointer into a host vector
rrm_status fetch(const void* src, size_t bytes, std::vector<unsigned char>& out) {
    out.resize(bytes);
    if (!bytes) return RRM_OK;
    RRM_HIP(hipMemcpy(out.data(), src, bytes, hipMemcpyDefault));
    return RRM_OK;
}

rrm_status upload(const void* host, size_t bytes, void** dev) {
    const size_t alloc = round16(bytes ? bytes : 16);
    if (hipMalloc(dev, alloc) != hipSuccess) {
        *dev = nullptr;
        return fail(RRM_ERR_ALLOC, "hipMalloc failed");
    }
    RRM_HIP(hipMemset(*dev, 0, alloc));
    if (bytes) RRM_HIP(hipMemcpy(*dev, host, bytes, hipMemcpyHostToDevice));
    return RRM_OK;
}

rrm_status dalloc(size_t bytes, void** dev) {
    const size_t alloc = round16(bytes ? bytes : 16);
    if (hipMalloc(dev, alloc) != hipSuccess) {
        *dev = nullptr;
        return fail(RRM_ERR_ALLOC, "hipMalloc failed");
    }
    RRM_HIP(hipMemset(*dev, 0, alloc));
    return RRM_OK;
}

int pitch_for(int sc) { return sc * 16; }

// reciprocal for the kernels' u / d on small u (0 encodes d == 1)
unsigned int magic_for(int d) { return d <= 1 ? 0u : (unsigned int)((1ull << 32) / (unsigned long long)d + 1ull); }



// Pack the LDS offset table and the weights for the workgroup shape chosen in L->cg.
// K pairs are ordered chunk by chunk: pair e of a slab is (chunk slab*sc + e / ntaps, tap e % ntaps),
// four pairs per K step, nq K steps per slab.  A "tap" is a filter tap in source positions: in a
// folded layer one tap covers `fold` filter columns of cp channels each.
rrm_status pack_conv(rrm_layer* L, const std::vector<unsigned char>& w) {
    const rrm_shape& s = L->shape;
    ConvGeom& g = L->cg;
    const int ntaps = s.kh * g.kw_eff;
    // K-pair table of a slab (the same for every slab), two words per pair:
    //   [0] LDS byte offset of the tap's window position (+ the chunk's, for chunks that are not rotated)
    //   [1] rotated chunks: (chunk + the tap's rotation term) mod rot_p | (rot_p - 1) << 8; others 0
    // Padded pairs point at offset 0 and carry zero weights.
    std::vector<int> tab((size_t)g.nq * 4 * 2, 0);
    for (int e = 0; e < ntaps * g.sc && e < g.nq * 4; ++e) {
        const int cc = e / ntaps, tap = e % ntaps;
        const int ky = tap / g.kw_eff, ku = tap % g.kw_eff;
        const int hp = ky * g.ww + ku;
        if (cc < g.rot_p) {
            const int rt = (g.rot_a * (ky / g.str_y) + g.rot_b * (ku / g.str_x)) & (g.rot_p - 1);
            tab[2 * e] = hp * g.sc * 16;
            tab[2 * e + 1] = ((cc + rt) & (g.rot_p - 1)) | ((g.rot_p - 1) << 8);
        } else {
            tab[2 * e] = hp * g.sc * 16 + cc * 16;
            tab[2 * e + 1] = 0;
        }
    }
    // Staging table, appended: what staged unit v = (slot*wpos + hp)*sc + cs of a workgroup holds, two
    // words per unit:
    //   [0] slot | window row << 5 | window column << 13 | (chunk missing in the last slab) << 21
    //   [1] source byte offset relative to the window origin at slab 0: (row*src_w + column)*pos_bytes + chunk*16
    const int n_units = g.nt * g.wpos * g.sc;
    tab.resize(tab.size() + (size_t)n_units * 2, 0);
    int* ut = tab.data() + (size_t)g.nq * 4 * 2;
    for (int v = 0; v < n_units; ++v) {
        const int r = v / g.sc, cs = v % g.sc;
        const int slot = r / g.wpos, hp = r % g.wpos;
        const int hy = hp / g.ww, hx = hp % g.ww;
        int cc = cs;  // the chunk held by slot cs of this position (see rot_p)
        if (cs < g.rot_p) cc = (cs - g.rot_a * (hy / g.str_y) - g.rot_b * (hx / g.str_x)) & (g.rot_p - 1);
        ut[2 * v] = slot | (hy << 5) | (hx << 13) | ((cc >= g.last_sc ? 1 : 0) << 21);
        ut[2 * v + 1] = (hy * g.src_w + hx) * g.pos_bytes + cc * 16;
    }
    rrm_status st = upload(tab.data(), tab.size() * sizeof(int), (void**)&L->offtab);
    if (st != RRM_OK) return st;

    // Weights in per-lane MFMA operand order: [group][32-channel block][MFMA step][lane] x 16 bytes, with
    // lane l -> output channel 32*block + l%32, K pair 2*step + l/32 (two MFMA steps per K step).  The block
    // dimension is padded to a multiple of the workgroup's block count; padded blocks, channels and pairs
    // are zero.
    const int NCB = g.wg_cb;
    const int ncb_p = (g.ncb + NCB - 1) / NCB * NCB;
    const int nq2 = 2 * g.nq;
    const int kall = g.nslab * nq2;
    const size_t nfrag = (size_t)s.groups * ncb_p * kall;
    std::vector<unsigned char> pack(nfrag * 64 * 16, 0);
    const int es = L->esize;
    const int real_taps = s.kh * s.kw;
    for (int grp = 0; grp < s.groups; ++grp)
        for (int cb = 0; cb < g.ncb; ++cb)
            for (int slab = 0; slab < g.nslab; ++slab)
                for (int q = 0; q < nq2; ++q)
                    for (int lane = 0; lane < 64; ++lane) {
                        const int co = cb * 32 + (lane & 31);
                        const int e = 2 * q + (lane >> 5);
                        if (co >= g.og || e >= ntaps * g.sc) continue;
                        const int chunk = slab * g.sc + e / ntaps, tap = e % ntaps;
                        if (chunk >= g.chunks) continue;
                        const int ky = tap / g.kw_eff, ku = tap % g.kw_eff;
                        const size_t frag = ((size_t)(grp * ncb_p + cb) * kall + (size_t)slab * nq2 + q);
                        unsigned char* dst = pack.data() + (frag * 64 + lane) * 16;
                        const size_t wrow = (size_t)(grp * g.og + co) * real_taps;
                        for (int k = 0; k < g.per_vec; ++k) {
                            // element k of the 16-byte chunk: filter column and channel it stands for
                            int kx, c;
                            if (g.fold > 1) {
                                kx = ku * g.fold + k / g.cp;
                                c = k % g.cp;
                            } else {
                                kx = ku;
                                c = chunk * g.per_vec + k;
                            }
                            if (kx >= s.kw || c >= g.cg) continue;
                            std::memcpy(dst + (size_t)k * es, w.data() + ((wrow + (size_t)ky * s.kw + kx) * g.cg + c) * es, es);
                        }
                    }
    return upload(pack.data(), pack.size(), &L->wpack);
}

// LDS bank spreading for the window reads of the K loop.  The 16 lanes that read the same (tap, chunk)
// for the 16 positions of a sub-tile should hit 16 different 16-byte bank groups of the 256-byte bank
// row.  The rotation coefficients are chosen by exhaustive search over the layer's taps.
void choose_rotation(ConvGeom& t, int ntaps) {
    int P = 1;
    while (P * 2 <= t.sc) P *= 2;
    t.rot_p = P;
    t.rot_a = t.rot_b = 0;
    t.magic_sy = magic_for(t.str_y);
    t.magic_sx = magic_for(t.str_x);
    if (P == 1) return;
    long long best = -1;
    for (int a = 0; a < P; ++a)
        for (int b = 0; b < P; ++b) {
            long long cost = 0;
            for (int tap = 0; tap < ntaps; ++tap) {
                const int ky = tap / t.kw_eff, ku = tap % t.kw_eff;
                for (int cc = 0; cc < P; ++cc) {
                    int addr[16], worst = 1;
                    for (int j = 0; j < 16; ++j) {
                        const int hy = (j >> 2) * t.str_y + ky, hx = (j & 3) * t.str_x + ku;
                        const int cs = (cc + a * (hy / t.str_y) + b * (hx / t.str_x)) & (P - 1);
                        addr[j] = ((hy * t.ww + hx) * t.sc + cs) * 16;
                    }
                    for (int j = 0; j < 16; ++j) {
                        int same = 1;
                        for (int k = 0; k < j; ++k)
                            if ((addr[k] & 255) / 16 == (addr[j] & 255) / 16 && addr[k] != addr[j]) ++same;
                        worst = std::max(worst, same);
                    }
                    cost += worst;
                }
            }
            if (best < 0 || cost < best) {
                best = cost;
                t.rot_a = a;
                t.rot_b = b;
            }
        }
}

// Fill the slab-dependent fields for (blocks, sub-tiles) per workgroup with the largest slab that fits
// the LDS budget; false if none does.  Several slabs: a slab is a whole number of K steps (4 pairs
// each) unless `padded`, which lets every slab end in up to 3 zero-weight pairs.
bool conv_try_shape(ConvGeom& g, int terms, int wg_cb, int nt, int ntaps, long long budget, bool padded = false) {
    const int max_units = CONV_MAX_STAGE_UNITS * CONV_THREADS;
    for (int sc = g.chunks; sc >= 1; --sc) {
        if (!padded && sc < g.chunks && (sc * ntaps) % 4 != 0) continue;
        ConvGeom t = g;
        t.wg_cb = wg_cb;
        t.nt = nt;
        t.sc = sc;
        t.nslab = (t.chunks + sc - 1) / sc;
        t.pitch = pitch_for(sc);
        t.slot_bytes = t.wpos * t.pitch;
        t.nq = (ntaps * sc + 3) / 4;
        if ((long long)conv_lds_bytes(t, wg_cb, nt, terms) > budget) continue;
        if ((long long)nt * t.wpos * sc > max_units) continue;  // staged units per thread are bounded
        t.magic_sc[0] = t.magic_sc[1] = magic_for(sc);
        t.magic_wsc[0] = t.magic_wsc[1] = magic_for(t.wpos);
        choose_rotation(t, ntaps);
        t.last_sc = t.chunks - (t.nslab - 1) * sc;
        g = t;
        return true;
    }
    return false;
}

rrm_status setup_conv(rrm_layer* L, const std::vector<unsigned char>& w) {
    const rrm_shape& s = L->shape;
    ConvGeom& g = L->cg;
    g.n = s.n; g.h = s.h; g.w = s.w; g.c_in = s.c_in; g.c_out = s.c_out;
    g.kh = s.kh; g.kw = s.kw; g.stride = s.stride; g.pad = s.pad; g.groups = s.groups;
    g.ho = (s.h + 2 * s.pad - s.kh) / s.stride + 1;
    g.wo = (s.w + 2 * s.pad - s.kw) / s.stride + 1;
    g.cg = s.c_in / s.groups;
    g.og = s.c_out / s.groups;
    g.sty = (g.ho + 3) / 4;
    g.stx = (g.wo + 3) / 4;
    g.n_sub = s.n * g.sty * g.stx;
    g.n_words = (g.n_sub + 3) / 4;
    g.per_vec = 16 / L->esize;
    g.chunks = (g.cg + g.per_vec - 1) / g.per_vec;
    // Source layout seen by the gather kernel.
    g.src_h = s.h;
    g.str_y = s.stride;
    g.pad_y = s.pad;
    const int run_bytes = g.cg * L->esize;  // one position's channels of one group
    g.aligned = (run_bytes % 16 == 0) ? 1 : 0;
    g.fold = 1;
    g.cp = g.chunks * g.per_vec;
    g.wp = s.w;
    if (!g.aligned && s.groups == 1 && run_bytes < 16) {
        // few channels: 16 / cpb neighbouring columns share one chunk, if the stride and the padding
        // keep every sub-tile's window aligned to that
        int cpb = 4;
        while (cpb < run_bytes) cpb *= 2;
        const int fold = 16 / cpb;
        if (fold > 1 && s.stride % fold == 0 && s.pad % fold == 0) {
            g.fold = fold;
            g.cp = cpb / L->esize;
            g.wp = (s.w + fold - 1) / fold * fold;
        }
    }
    g.kw_eff = (s.kw + g.fold - 1) / g.fold;
    g.src_w = g.wp / g.fold;
    g.str_x = s.stride / g.fold;
    g.pad_x = s.pad / g.fold;
    g.grp_bytes = g.fold > 1 ? 16 : g.chunks * 16;
    g.pos_bytes = g.fold > 1 ? 16 : s.groups * g.chunks * 16;
    g.wh = 3 * g.str_y + s.kh;
    g.ww = 3 * g.str_x + g.kw_eff;
    g.wpos = g.wh * g.ww;
    g.ncb = (g.og + 31) / 32;  // 32-channel MFMA blocks per group
    g.magic_ww = magic_for(g.ww);
    g.magic_sub = magic_for(g.sty * g.stx);
    g.magic_stx = magic_for(g.stx);
    g.magic_wo = magic_for(g.wo);
    g.magic_ho = magic_for(g.ho);
    g.vec_store = (s.c_out % 4 == 0) && (g.og % 4 == 0);
    const int ntaps = s.kh * g.kw_eff;
    const int terms = L->dtype == RRM_BF16_F32 ? 2 : 1;
    // Workgroup shape.  Few sub-tiles in total (one stream of a small map): latency matters, so one
    // 32-channel block and up to 8 sub-tiles per workgroup, the whole K range in as few slabs as fit.
    // Many sub-tiles (many streams): operand reuse matters, so 2 channel blocks x 16 sub-tiles.
    struct Cand { int cb, nt; };
    std::vector<Cand> cands;
    const bool small = (long long)g.n_sub * g.ncb * s.groups <= 1024;
    if (small || g.ncb < 2) {
        cands = {{1, 8}, {1, 16}, {1, 4}};
        if (!small) cands = {{1, 16}, {1, 8}, {1, 4}};
    } else {
        cands = {{2, 16}, {2, 8}, {1, 16}, {1, 8}, {1, 4}};
    }
    bool ok = false;
    // (the kernel's static LDS, about 6 KB, comes on top of the dynamic budget; 160 KB per workgroup in all)
    long long first_budget = (small ? 96ll : 153ll) * 1024;
    if (const char* env = std::getenv("RRM_CONV_LDS_KB")) {  // tuning knob: preferred LDS bytes per workgroup
        const long long kb = std::atoll(env);
        if (kb >= 16 && kb <= 153) first_budget = kb * 1024;
    }
    for (long long budget : {first_budget, 153ll * 1024}) {
        for (const Cand& c : cands) {
            ConvGeom t = g;
            // a slab should hold at least 4 chunks (or all of them) to amortise its barriers
            if (conv_try_shape(t, terms, c.cb, c.nt, ntaps, budget) && (t.sc >= 4 || t.sc == t.chunks)) {
                g = t;
                ok = true;
                break;
            }
        }
        if (ok) break;
    }
    if (!ok)
        for (const Cand& c : cands)
            if (!ok) ok = conv_try_shape(g, terms, c.cb, c.nt, ntaps, 153 * 1024);
    if (!ok)  // large filter windows: slabs of any chunk count, down to one sub-tile per workgroup
        for (const Cand& c : {Cand{1, 8}, Cand{1, 4}, Cand{1, 2}, Cand{1, 1}})
            if (!ok) ok = conv_try_shape(g, terms, c.cb, c.nt, ntaps, 153 * 1024, true);
    if (!ok) return fail(RRM_ERR_SHAPE, "input window of one output sub-tile does not fit LDS");
    return pack_conv(L, w);
}

// Position-gather kernel: eligibility, work-unit shape, weights in per-lane MFMA order
// [group][block of POS_NCB x 32 channels][slab of 2 chunks][tap][32-channel block][lane] x 16 bytes, lane l ->
// output channel l % 32 of the block, chunk 2 * slab + l / 32 of the tap.  Padded channels and chunks are zero.
rrm_status setup_pos(rrm_layer* L, const std::vector<unsigned char>& w) {
    const rrm_shape& s = L->shape;
    PosGeom& g = L->pg;
    L->pos_ok = false;
    const int es = L->esize;
    if (!pos_choose_shape(s, es, L->dtype == RRM_BF16_F32 ? 2 : 1, g)) return RRM_OK;
    const int cg = g.cg, og = g.og;

    const int real_taps = s.kh * s.kw;
    std::vector<unsigned char> pack((size_t)s.groups * g.ncg * g.nslab * g.ntaps * POS_NCB * 1024, 0);
    const int per_vec = 16 / es;
    for (int grp = 0; grp < s.groups; ++grp)
        for (int cgp = 0; cgp < g.ncg; ++cgp)
            for (int slab = 0; slab < g.nslab; ++slab)
                for (int tap = 0; tap < g.ntaps; ++tap)
                    for (int cb = 0; cb < POS_NCB; ++cb)
                        for (int lane = 0; lane < 64; ++lane) {
                            const int co = (cgp * POS_NCB + cb) * 32 + (lane & 31);
                            const int chunk = 2 * slab + (lane >> 5);
                            if (co >= og || chunk >= g.chunks) continue;
                            const size_t frag = ((((size_t)(grp * g.ncg + cgp) * g.nslab + slab) * g.ntaps + tap) * POS_NCB + cb);
                            unsigned char* dst = pack.data() + (frag * 64 + lane) * 16;
                            const size_t wrow = (size_t)(grp * og + co) * real_taps + tap;
                            std::memcpy(dst, w.data() + (wrow * cg + (size_t)chunk * per_vec) * es, 16);
                        }
    rrm_status st = upload(pack.data(), pack.size(), &L->wpos);
    if (st != RRM_OK) return st;
    L->pos_ok = true;
    return RRM_OK;
}

// Single-launch scatter path: eligibility, block shape, weights in per-lane MFMA order
// [(group, 32-channel block)][tap][K step][lane] x 16 bytes, lane l -> output channel l % 32 of the block, unit
// 2 * step + l / 32 of the group's channels at that tap.  Padded channels and units are zero.
rrm_status setup_scatter(rrm_layer* L, const std::vector<unsigned char>& w) {
    const rrm_shape& s = L->shape;
    ScatGeom& g = L->sc;
    L->scat_ok = false;
    const int es = L->esize;
    const int cg = s.c_in / s.groups, og = s.c_out / s.groups;
    if ((cg * es) % 16 != 0) return RRM_OK;
    g.n = s.n; g.h = s.h; g.w = s.w; g.c_out = s.c_out; g.kh = s.kh; g.kw = s.kw; g.stride = s.stride; g.pad = s.pad;
    g.groups = s.groups;
    g.ho = (s.h + 2 * s.pad - s.kh) / s.stride + 1;
    g.wo = (s.w + 2 * s.pad - s.kw) / s.stride + 1;
    g.og = og;
    g.U = s.c_in * es / 16;
    g.ug = cg * es / 16;
    g.nk = (g.ug + 1) / 2;
    g.ncb = (og + 31) / 32;
    g.npair = s.groups * g.ncb;
    g.ntaps = s.kh * s.kw;
    g.npos_total = (long long)s.n * s.h * s.w;
    const int terms = L->dtype == RRM_BF16_F32 ? 2 : 1;
    // positions per block: the block's units fit the threads' registers (SCAT_UPT each) and, times the terms, 64 KB
    g.PB = 0;
    for (int pb : {64, 32, 16, 8})
        if (pb * g.U <= 256 * SCAT_UPT && terms * pb * g.U <= 4000) {
            g.PB = pb;
            break;
        }
    if (g.PB == 0) return RRM_OK;
    const long long nblk = (g.npos_total + g.PB - 1) / g.PB;
    // Work items of a position block: (channel block, tap, part of the K range of at most 8 steps); a workgroup's four
    // wavefronts take one item each per round.  Few position blocks: the items of a block are split over more
    // workgroups (one round each at most), up to about two workgroups per compute unit in all.
    g.nkp = (g.nk + 7) / 8;
    const long long items = (long long)g.npair * g.ntaps * g.nkp;
    g.cs = (int)std::max(1ll, std::min((items + 3) / 4, (2ll * NUM_CU + nblk - 1) / nblk));
    std::vector<unsigned char> pack((size_t)g.npair * g.ntaps * g.nk * 64 * 16, 0);
    const int per_vec = 16 / es;
    for (int pair = 0; pair < g.npair; ++pair)
        for (int tap = 0; tap < g.ntaps; ++tap)
            for (int k = 0; k < g.nk; ++k)
                for (int lane = 0; lane < 64; ++lane) {
                    const int grp = pair / g.ncb, cb = pair % g.ncb;
                    const int co = cb * 32 + (lane & 31), unit = 2 * k + (lane >> 5);
                    if (co >= og || unit >= g.ug) continue;
                    unsigned char* dst = pack.data() + ((((size_t)pair * g.ntaps + tap) * g.nk + k) * 64 + lane) * 16;
                    const size_t wrow = (size_t)(grp * og + co) * g.ntaps + tap;
                    std::memcpy(dst, w.data() + (wrow * cg + (size_t)unit * per_vec) * es, 16);
                }
    rrm_status st = upload(pack.data(), pack.size(), &L->wsc);
    if (st != RRM_OK) return st;
    if ((st = dalloc((size_t)nblk * sizeof(unsigned int), (void**)&L->sc_arrive)) != RRM_OK) return st;
    g.arrive = L->sc_arrive;
    L->scat_ok = true;
    // Automatic: layers with few positions in all (one stream of a small map).  Two dependent launches and the
    // per-workgroup set-up of the tile kernels then cost more than the step's work; measured, the single launch wins
    // there up to about a tenth of the positions changing, and on the smallest maps at any density.
    L->scat_auto = g.npos_total <= 1024;
    return RRM_OK;
}

// choose the convolution kernel of an int8 / bf16 layer: 0 = automatic, 1 = window-tile, 2 = position-gather
rrm_status select_conv_kernel(rrm_layer* L, int which) {
    if (which == 2 && !L->pos_ok) return fail(RRM_ERR_OPTION, "the position-gather kernel needs stride 1 and 16-byte channel runs");
    // Automatic is the window-tile kernel.  The position-gather kernel measured 8-10 % faster on small int8 maps
    // when every stream changes in the same scattered way, and 15-25 % slower on the video recipe, whose streams
    // differ widely (its fixed set-up per (stream, band) unit is paid by the static streams too, and once a
    // third of the positions change the gather saves little over whole windows): it is the caller's choice.
    L->use_pos = which == 2;
    L->tshift = L->use_pos ? 0 : 2;
    ScanGeom& sg = L->sg;
    sg.sty = L->use_pos ? 0 : L->cg.sty;  // (no sub-tile flags for the position-gather kernel: it reads the bitmap)
    sg.stx = L->use_pos ? 0 : L->cg.stx;
    sg.tiles_per_step = L->use_pos ? (unsigned long long)L->shape.n * L->cg.ho * L->cg.wo
                                   : (unsigned long long)L->shape.n * L->cg.sty * L->cg.stx;
    return RRM_OK;
}

rrm_status setup_bin(rrm_layer* L, const std::vector<unsigned char>& w) {
    const rrm_shape& s = L->shape;
    BinGeom& g = L->bg;
    if (!bin_choose_shape(s, g)) return fail(RRM_ERR_SHAPE, "input window of one output tile does not fit LDS");
    if (g.fused_ok) {
        rrm_status st2 = dalloc((size_t)s.n * sizeof(unsigned int), (void**)&L->bin_arrive);
        if (st2 != RRM_OK) return st2;
    }
    const int ntaps = s.kh * s.kw;
    // filter words: [group][co/8][slab][tap][co%8][4 words]
    std::vector<unsigned int> pack((size_t)s.groups * g.nob8 * g.nslab * ntaps * 8 * 4, 0u);
    const unsigned int* ww = reinterpret_cast<const unsigned int*>(w.data());
    for (int grp = 0; grp < s.groups; ++grp)
        for (int co = 0; co < g.og; ++co)
            for (int tap = 0; tap < ntaps; ++tap)
                for (int wd = 0; wd < g.wg; ++wd) {
                    const int slab = wd / 4;
                    const size_t dst = (((((size_t)grp * g.nob8 + co / 8) * g.nslab + slab) * ntaps + tap) * 8 + co % 8) * 4 + wd % 4;
                    pack[dst] = ww[(((size_t)(grp * g.og + co)) * ntaps + tap) * g.wg + wd];
                }
    return upload(pack.data(), pack.size() * 4, &L->wpack);
}

rrm_status setup_fc(rrm_layer* L, const std::vector<unsigned char>& w) {
    const rrm_shape& s = L->shape;
    FcGeom& g = L->fg;
    g.n = s.n; g.c_in = s.c_in; g.c_out = s.c_out;
    g.per_vec = 16 / L->esize;
    g.c_out_p = (s.c_out + g.per_vec - 1) / g.per_vec * g.per_vec;
    g.vec_ok = (s.c_in % g.per_vec) == 0;
    // input-major copy: W^T [c_in][c_out_p], every column of W contiguous
    const int es = L->esize;
    std::vector<unsigned char> t((size_t)s.c_in * g.c_out_p * es, 0);
    for (int o = 0; o < s.c_out; ++o)
        for (int j = 0; j < s.c_in; ++j)
            std::memcpy(t.data() + ((size_t)j * g.c_out_p + o) * es, w.data() + ((size_t)o * s.c_in + j) * es, es);
    rrm_status st = upload(t.data(), t.size(), &L->wpack);
    if (st != RRM_OK) return st;
    // Pruned weights (Sec. 4.3: the compressed models keep 10 % or so of their weights): when at most half of
    // the weights are non-zero the columns are also stored as (row, value) lists, which the delta step walks on
    // request ("fc_sparse_weights").  Not by itself: at one stream the step is bound by latency and by the atomic
    // adds that merge the workgroups' partial updates, not by bytes, and on fc6 with a tenth of the weights the
    // sparse walk measured faster than the whole-column walk only while few inputs change (int8, 5 %: 9.1 against
    // 10.5 us; 25 %: 17.2 against 11.4 us).
    g.csc_ptr = nullptr;
    g.csc_row = nullptr;
    g.csc_val = nullptr;
    {
        auto nonzero = [&](size_t i) {
            if (es == 1) return w[i] != 0;
            return (reinterpret_cast<const unsigned short*>(w.data())[i] & 0x7FFFu) != 0;
        };
        const size_t total = (size_t)s.c_in * s.c_out;
        size_t nnz = 0;
        for (size_t i = 0; i < total; ++i) nnz += nonzero(i) ? 1 : 0;
        L->w_density = total ? (double)nnz / (double)total : 1.0;
        if (2 * nnz <= total && s.c_out <= 65536 && (size_t)s.c_out * 4 <= (size_t)FC_CSC_MAX_LDS && nnz < 0xFFFFFFFFull) {
            std::vector<unsigned int> ptr((size_t)s.c_in + 1, 0u);
            std::vector<unsigned short> rowi(std::max<size_t>(nnz, 1));
            std::vector<unsigned char> val(std::max<size_t>(nnz, 1) * es);
            size_t k = 0;
            for (int j = 0; j < s.c_in; ++j) {
                ptr[j] = (unsigned int)k;
                for (int o = 0; o < s.c_out; ++o) {
                    const size_t i = (size_t)o * s.c_in + j;
                    if (!nonzero(i)) continue;
                    rowi[k] = (unsigned short)o;
                    std::memcpy(val.data() + k * es, w.data() + i * es, es);
                    ++k;
                }
            }
            ptr[s.c_in] = (unsigned int)k;
            if ((st = upload(ptr.data(), ptr.size() * 4, &L->csc_ptr)) != RRM_OK) return st;
            if ((st = upload(rowi.data(), rowi.size() * 2, &L->csc_row)) != RRM_OK) return st;
            if ((st = upload(val.data(), val.size(), &L->csc_val)) != RRM_OK) return st;
            L->csc_ok = true;
        }
    }
    // many streams: the layer runs as one product on the matrix cores, from W in its own layout; int8 steps
    // multiply the difference of all streams (d0), bf16 steps recompute from x_t
    if (fc_batched_ok(L->dtype, g)) {
        if ((st = upload(w.data(), (size_t)s.c_in * s.c_out * es, &L->w_rm)) != RRM_OK) return st;
        if (L->dtype == RRM_I8_I32 && (st = dalloc((size_t)s.n * s.c_in * es, &L->d0)) != RRM_OK) return st;
        if ((st = dalloc((size_t)fc_batched_splits(L->dtype, g) * s.n * s.c_out * 4, &L->fc_bpart)) != RRM_OK) return st;
    }
    // dense path: enough workgroups to keep memory busy (about 256 in total, at most 64 row splits per stream)
    L->fc_nsplit = std::max(1, std::min(64, 256 / (fc_dense_slices(L->dtype, g) * s.n)));
    if ((st = dalloc((size_t)s.n * L->fc_nsplit * g.c_out_p * 4, &L->fc_part)) != RRM_OK) return st;
    return dalloc((size_t)s.n * sizeof(unsigned int), (void**)&L->fc_arrive);  // delta path: arrival counters
}

constexpr int kProfMax = 1024;

// record the k-th (0..2) event of the current profiled step
rrm_status prof_mark(rrm_layer* L, int k, hipStream_t s) {
    if (!L->prof_on || L->prof_n >= kProfMax) return RRM_OK;
    const size_t need = (size_t)3 * (L->prof_n + 1);
    while (L->prof_ev.size() < need) {
        hipEvent_t e;
        RRM_HIP(hipEventCreate(&e));
        L->prof_ev.push_back(e);
    }
    RRM_HIP(hipEventRecord(L->prof_ev[(size_t)3 * L->prof_n + k], s));
    if (k == 2) ++L->prof_n;
    return RRM_OK;
}

int bin_cw(const rrm_layer* L) {
    if (L->opt_bin_cw) return L->opt_bin_cw;
    const BinGeom& g = L->bg;
    return ((long long)g.n * g.tiles_y * g.tiles_x * g.groups * ((g.og + 63) / 64) >= 512) ? 16 : 8;
}

// does this step of a convolution layer take the single-launch scatter path?  ("path" = 3: always where the layer
// is eligible; automatic, with the kernel choice left automatic too: layers with few positions, see setup_scatter)
bool use_scatter(const rrm_layer* L) {
    if (!L->scat_ok || L->dtype == RRM_BIN_I32) return false;
    if (L->opt_path == 3) return true;
    return L->opt_path == 0 && L->opt_conv_kernel == 0 && L->scat_auto;
}

int fc_splits(const rrm_layer* L) { return L->opt_fc_splits > 0 ? L->opt_fc_splits : L->fc_nsplit; }

rrm_status check_ptr(const void* p, const char* what) {
    if (!p) return fail(RRM_ERR_NULL, std::string(what) + " is NULL");
    if (reinterpret_cast<uintptr_t>(p) & 15) return fail(RRM_ERR_ALIGN, std::string(what) + " is not 16-byte aligned");
    return RRM_OK;
}

// dense layer of Eq. 3 from x into y
rrm_status enqueue_dense(rrm_layer* L, const void* x, void* y, hipStream_t st) {
    if (L->shape.kind == RRM_FC) {
        if (L->w_rm && L->opt_fc_batched)
            RRM_HIP(launch_fc_batched_dense(L->dtype, L->w_rm, x, L->fc_bpart, L->bias, y, L->fg, st));
        else
            RRM_HIP(launch_fc_dense(L->dtype, fc_splits(L), L->wpack, x, L->fc_part, L->bias, y, L->fg, st));
    } else if (L->dtype == RRM_BIN_I32) {
        RRM_HIP(launch_bin_conv(MODE_DENSE, bin_cw(L), x, nullptr, nullptr, L->wpack, L->bias, y, L->bg, L->stats, st));
    } else {
        if (L->use_pos) {
            RRM_HIP(launch_conv_pos(L->dtype, MODE_DENSE, 1, x, nullptr, L->zero16, nullptr, L->ctrl, L->wpos, L->bias, y, L->pg,
                                    L->stats, st));
            return RRM_OK;
        }
        const void* src = x;
        if (!L->cg.aligned) {  // bring x into the 16-byte-chunk layout first (its pad elements stay zero)
            RRM_HIP(launch_repack(L->esize, x, L->xpad, L->sg, st));
            src = L->xpad;
        }
        RRM_HIP(launch_conv(L->dtype, MODE_DENSE, L->cg.wg_cb, L->cg.nt, 1, src, nullptr, L->zero16, nullptr, nullptr, L->wpack, L->offtab,
                            L->bias, y, L->cg, L->stats, st));
    }
    return RRM_OK;
}

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

rrm_status rrm_layer_create(const void* weights, const void* bias, const rrm_shape* shape, int dtype, rrm_layer** out) {
    if (!out) return fail(RRM_ERR_NULL, "out is NULL");
    *out = nullptr;
    if (!weights) return fail(RRM_ERR_NULL, "weights is NULL");
    if (!shape) return fail(RRM_ERR_NULL, "shape is NULL");
    rrm_status st = validate(shape, dtype);
    if (st != RRM_OK) return st;
    rrm_layer* L = new (std::nothrow) rrm_layer();
    if (!L) return fail(RRM_ERR_ALLOC, "out of host memory");
    L->shape = *shape;
    if (shape->kind == RRM_FC) {
        L->shape.h = L->shape.w = L->shape.kh = L->shape.kw = L->shape.stride = L->shape.groups = 1;
        L->shape.pad = 0;
    }
    const rrm_shape& s = L->shape;
    L->dtype = dtype;
    L->esize = dtype == RRM_I8_I32 ? 1 : (dtype == RRM_BF16_F32 ? 2 : 4);
    const long long ho = (s.h + 2 * s.pad - s.kh) / s.stride + 1, wo = (s.w + 2 * s.pad - s.kw) / s.stride + 1;
    const long long cin_units = dtype == RRM_BIN_I32 ? s.c_in / 32 : s.c_in;
    L->x_elems = (long long)s.n * s.h * s.w * cin_units;
    L->y_elems = (long long)s.n * ho * wo * s.c_out;
    L->x_bytes = (size_t)L->x_elems * L->esize;
    L->y_bytes = (size_t)L->y_elems * 4;

    const long long w_units = (long long)s.c_out * s.kh * s.kw * (cin_units / s.groups);
    std::vector<unsigned char> hw, hb;
    auto bail = [&](rrm_status e) {
        delete L;
        return e;
    };
    if ((st = fetch(weights, (size_t)w_units * L->esize, hw)) != RRM_OK) return bail(st);
    if (bias) {
        if ((st = fetch(bias, (size_t)s.c_out * 4, hb)) != RRM_OK) return bail(st);
        if ((st = upload(hb.data(), hb.size(), &L->bias)) != RRM_OK) return bail(st);
    }
    if (s.kind == RRM_FC)
        st = setup_fc(L, hw);
    else if (dtype == RRM_BIN_I32)
        st = setup_bin(L, hw);
    else {
        st = setup_conv(L, hw);
        if (st == RRM_OK) st = setup_pos(L, hw);
        if (st == RRM_OK) st = setup_scatter(L, hw);
    }
    if (st != RRM_OK) return bail(st);

    if ((st = dalloc(L->x_bytes, &L->x_snap)) != RRM_OK) return bail(st);
    if ((st = dalloc(L->y_bytes, &L->y_snap)) != RRM_OK) return bail(st);
    if ((st = dalloc(sizeof(DevStats) * STAT_SLOTS, (void**)&L->stats)) != RRM_OK) return bail(st);
    if (s.kind == RRM_CONV) {
        ScanGeom& sg = L->sg;
        sg.total_elems = L->x_elems;
        sg.c = (int)cin_units;
        sg.h = s.h; sg.w = s.w; sg.kh = s.kh; sg.kw = s.kw; sg.stride = s.stride; sg.pad = s.pad;
        sg.ho = (int)ho; sg.wo = (int)wo;
        sg.tiles_y = (int)((ho + TILE - 1) / TILE);
        sg.tiles_x = (int)((wo + TILE - 1) / TILE);
        sg.per_vec = 16 / L->esize;
        sg.r_c = 1.0 / (double)sg.c;
        sg.r_hw = 1.0 / ((double)s.h * (double)s.w);
        sg.r_w = 1.0 / (double)s.w;
        sg.magic_stride = magic_for(s.stride);
        const size_t nvec = round16(L->x_bytes) / 16;
        // difference buffer: x's own layout, or the padded / folded layout of the gather kernel
        L->d_bytes = L->x_bytes;
        sg.scatter = 0;
        if (dtype != RRM_BIN_I32 && !L->cg.aligned) {
            sg.scatter = 1;
            sg.wp = L->cg.wp;
            sg.cp = L->cg.cp;
            sg.cg = L->cg.cg;
            sg.groups = s.groups;
            L->d_bytes = (size_t)s.n * s.h * sg.wp * s.groups * sg.cp * L->esize;
            if ((st = dalloc(L->d_bytes, &L->xpad)) != RRM_OK) return bail(st);  // dense path's repacked x
        }
        if ((st = dalloc(L->d_bytes, &L->d0)) != RRM_OK) return bail(st);
        if (dtype == RRM_BF16_F32 && (st = dalloc(L->d_bytes, &L->d1)) != RRM_OK) return bail(st);
        if ((st = dalloc(((nvec + 63) / 64) * 8, (void**)&L->bitmap)) != RRM_OK) return bail(st);
        sg.sty = (int)((ho + 3) / 4);
        sg.stx = (int)((wo + 3) / 4);
        sg.tiles_per_step = dtype == RRM_BIN_I32 ? (L->bg.band_rows > 0 ? (unsigned long long)s.n * ho * wo
                                                                        : (unsigned long long)s.n * sg.tiles_y * sg.tiles_x)
                                                 : (unsigned long long)s.n * sg.sty * sg.stx;
        // binary: one stamp per 8x8 tile; int8 / bf16: one byte flag per 4x4 sub-tile
        L->marks_bytes = dtype == RRM_BIN_I32 ? (size_t)s.n * sg.tiles_y * sg.tiles_x * 4
                                              : (size_t)((s.n * sg.sty * sg.stx + 3) / 4) * 4;
        if ((st = dalloc(L->marks_bytes, (void**)&L->tileflag)) != RRM_OK) return bail(st);
        if (dtype != RRM_BIN_I32) {
            // everything counts as written until the first step has run (y_snap = bias everywhere)
            // (one byte per 4x4 block for the window-tile kernel, per output position for the position-gather kernel)
            L->touched_bytes = L->pos_ok ? std::max(L->marks_bytes, (size_t)s.n * (size_t)ho * (size_t)wo) : L->marks_bytes;
            if ((st = dalloc(L->touched_bytes, (void**)&L->touched)) != RRM_OK) return bail(st);
            if (hipMemset(L->touched, 1, round16(L->touched_bytes)) != hipSuccess) return bail(fail(RRM_ERR_HIP, "hipMemset failed"));
            L->cg.touched = L->touched;
            L->pg.touched = reinterpret_cast<unsigned char*>(L->touched);
            // Above this share of active sub-tiles a delta step recomputes the layer instead (the stored
            // input, equal to x_t after the scan, is the source: only layers whose x layout is the kernel's)
            L->cg.xfull = L->cg.aligned ? static_cast<const unsigned char*>(L->x_snap) : nullptr;
            // (a bf16 delta multiplies two terms, a recomputation one: it pays off earlier)
            L->cg.full_pct = dtype == RRM_BF16_F32 ? 40 : 75;
            L->pg.xfull = static_cast<const unsigned char*>(L->x_snap);  // (its layers are always in x's layout)
            L->pg.full_pct = dtype == RRM_BF16_F32 ? 50 : 90;
            if ((st = select_conv_kernel(L, 0)) != RRM_OK) return bail(st);
        }
        if ((st = dalloc(16, (void**)&L->ctrl)) != RRM_OK) return bail(st);
        {
            const unsigned int ones[4] = {1u, 1u, 1u, 1u};
            if ((st = upload(ones, 16, (void**)&L->fresh)) != RRM_OK) return bail(st);
            L->cg.fresh = L->fresh;
            L->pg.fresh = L->fresh;
            L->cg.touched_all = L->pg.touched_all = L->sc.touched_all = L->ctrl + 3;
        }
        if ((st = dalloc(256, &L->zero16)) != RRM_OK) return bail(st);
    }
    // P_0 = b (Eq. 3 at I_0 = 0); I_0 = 0 comes from the zeroed allocation
    hipError_t e = launch_fill_bias(dtype == RRM_BF16_F32, L->y_snap, L->bias, L->y_elems / s.c_out, s.c_out, nullptr);
    // A binary tensor has no zero: the all-zero bit pattern of the fresh stored input is the frame of all -1,
    // and the stored projection starts as that frame's projection, so that the recurrence holds from the first
    // delta step on whatever the host knows about the handle's history.
    if (e == hipSuccess && dtype == RRM_BIN_I32 && enqueue_dense(L, L->x_snap, L->y_snap, nullptr) != RRM_OK) e = hipErrorUnknown;
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        delete L;
        return fail(RRM_ERR_HIP, std::string("initialising the projection: ") + hipGetErrorString(e));
    }
    *out = L;
    return RRM_OK;
}

rrm_status rrm_step(rrm_layer* L, const void* x_t, void* y_out, void* hip_stream) {
    if (!L) return fail(RRM_ERR_NULL, "layer is NULL");
    rrm_status st = check_ptr(x_t, "x_t");
    if (st != RRM_OK) return st;
    if (y_out && (reinterpret_cast<uintptr_t>(y_out) & 15)) return fail(RRM_ERR_ALIGN, "y_out is not 16-byte aligned");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const bool first_bin = L->dtype == RRM_BIN_I32 && !L->has_snapshot;
    if (L->opt_path == 2 || first_bin) {
        // full recomputation: P <- b + W (*) x_t, I <- x_t
        if ((st = prof_mark(L, 0, s)) != RRM_OK) return st;
        RRM_HIP(launch_copy(L->x_snap, x_t, L->x_bytes, s));
        if ((st = prof_mark(L, 1, s)) != RRM_OK) return st;
        if ((st = enqueue_dense(L, x_t, L->y_snap, s)) != RRM_OK) return st;
        // a full recomputation writes every output block (enqueued unconditionally: a captured step must not
        // depend on what the host believes the flags hold)
        if (L->touched) RRM_HIP(launch_fill_word(L->touched, round16(L->touched_bytes), 0x01010101u, s));
        if ((st = prof_mark(L, 2, s)) != RRM_OK) return st;
    } else if (L->shape.kind == RRM_FC) {
        if ((st = prof_mark(L, 0, s)) != RRM_OK) return st;
        if (L->w_rm && L->opt_fc_batched && !L->use_csc && L->fg.eps == 0.0f) {
            // many streams: difference (or commit) of all streams, then one product over W (two launches; the events
            // bracket both)
            if ((st = prof_mark(L, 1, s)) != RRM_OK) return st;
            RRM_HIP(launch_fc_batched_delta(L->dtype, L->w_rm, x_t, L->x_snap, L->d0, L->fc_bpart, L->bias, L->y_snap, L->fg, L->stats, s));
            if ((st = prof_mark(L, 2, s)) != RRM_OK) return st;
        } else {
        if ((st = prof_mark(L, 1, s)) != RRM_OK) return st;  // (no separate scan kernel: its time is reported as 0)
        FcGeom fg = L->fg;
        if (L->use_csc) {
            fg.csc_ptr = static_cast<const unsigned int*>(L->csc_ptr);
            fg.csc_row = static_cast<const unsigned short*>(L->csc_row);
            fg.csc_val = L->csc_val;
        }
        RRM_HIP(launch_fc_delta(L->dtype, x_t, L->x_snap, L->wpack, L->y_snap, L->fc_arrive, fg, L->stats, s));
        if ((st = prof_mark(L, 2, s)) != RRM_OK) return st;
        }
    } else {
        if ((st = prof_mark(L, 0, s)) != RRM_OK) return st;
        if (L->dtype == RRM_BIN_I32) {
            const int cw = bin_cw(L);
            if (L->bg.fused_ok && L->opt_bin_fused) {
                // one launch: compare, popcount products of the changed positions, commit
                if ((st = prof_mark(L, 1, s)) != RRM_OK) return st;  // (no separate difference kernel: its time is reported as 0)
                RRM_HIP(launch_bin_band_fused(cw, x_t, L->x_snap, L->bin_arrive, L->wpack, L->y_snap, L->bg, L->stats, s));
            } else {
            const bool band = L->bg.band_rows > 0;  // (the band kernel reads the flip words itself: no tile stamps)
            RRM_HIP(launch_scan(L->dtype, x_t, L->x_snap, L->d0, L->d1, L->bitmap, L->tileflag,
                                band ? 0u : (unsigned int)bin_consumers(cw, L->bg), L->sg, L->stats, s));
            if ((st = prof_mark(L, 1, s)) != RRM_OK) return st;
            if (band)
                RRM_HIP(launch_bin_band(cw, L->x_snap, L->d0, L->wpack, L->y_snap, L->bg, L->stats, s));
            else
                RRM_HIP(launch_bin_conv(MODE_DELTA, cw, L->x_snap, L->d0, L->tileflag, L->wpack, nullptr, L->y_snap, L->bg,
                                        L->stats, s));
            }
        } else if (use_scatter(L)) {
            // one launch: compare, products of the changed positions, atomic accumulation, commit
            if ((st = prof_mark(L, 1, s)) != RRM_OK) return st;  // (no separate scan kernel: its time is reported as 0)
            ScatGeom sc = L->sc;
            sc.eps = L->sg.eps;
            RRM_HIP(launch_conv_scatter(L->dtype, L->opt_terms, x_t, L->x_snap, L->wsc, L->y_snap, sc, L->stats, s));
        } else {
            RRM_HIP(launch_scan(L->dtype, x_t, L->x_snap, L->d0, L->d1, L->bitmap, L->tileflag, 0u, L->sg, L->stats, s));
            if ((st = prof_mark(L, 1, s)) != RRM_OK) return st;
            if (L->use_pos) {
                PosGeom pg = L->pg;
                if (L->opt_path == 1) pg.xfull = nullptr;  // the sparse path always: no switch to recomputation
                RRM_HIP(launch_conv_pos(L->dtype, MODE_DELTA, L->dtype == RRM_BF16_F32 ? L->opt_terms : 1, L->d0, L->d1,
                                        L->zero16, L->bitmap, L->ctrl, L->wpos, L->bias, L->y_snap, pg, L->stats, s));
            } else {
            ConvGeom cg = L->cg;
            if (L->opt_path == 1) cg.xfull = nullptr;  // the sparse path always: no switch to recomputation
            RRM_HIP(launch_conv(L->dtype, MODE_DELTA, L->cg.wg_cb, L->cg.nt, L->dtype == RRM_BF16_F32 ? L->opt_terms : 1,
                                L->d0, L->d1, L->zero16, L->tileflag, L->ctrl, L->wpack, L->offtab, L->bias, L->y_snap, cg,
                                L->stats, s));
            }
        }
        if ((st = prof_mark(L, 2, s)) != RRM_OK) return st;
    }
    L->has_snapshot = true;
    ++L->steps;
    if (y_out) RRM_HIP(launch_copy(y_out, L->y_snap, L->y_bytes, s));
    return RRM_OK;
}

rrm_status rrm_step_from_projection(rrm_layer* L, rrm_layer* P, int shift, int pool, void* y_out, void* hip_stream) {
    if (!L || !P) return fail(RRM_ERR_NULL, "layer / producer is NULL");
    if (L == P) return fail(RRM_ERR_STATE, "a layer cannot be its own producer");
    const rrm_shape& s = L->shape;
    const rrm_shape& ps = P->shape;
    if (s.kind != RRM_CONV || ps.kind != RRM_CONV || L->dtype != RRM_I8_I32 || P->dtype != RRM_I8_I32 || !P->touched)
        return fail(RRM_ERR_DTYPE, "rrm_step_from_projection needs two int8 convolution layers");
    const int hy = P->cg.ho, wy = P->cg.wo;
    const int hx = pool ? (hy - 3) / 2 + 1 : hy, wx = pool ? (wy - 3) / 2 + 1 : wy;
    if (shift < 0 || shift > 31 || (pool && (hy < 3 || wy < 3)) || s.n != ps.n || s.c_in != ps.c_out || s.h != hx || s.w != wx)
        return fail(RRM_ERR_SHAPE, "the producer's projection, mapped by f, does not have this layer's input shape");
    if (s.c_in % 16 != 0 || L->sg.scatter)
        return fail(RRM_ERR_SHAPE, "rrm_step_from_projection needs c_in to be a multiple of 16");
    if (L->opt_path == 2) return fail(RRM_ERR_STATE, "not available with \"path\" = 2: that path needs x_t in memory");
    if (y_out && (reinterpret_cast<uintptr_t>(y_out) & 15)) return fail(RRM_ERR_ALIGN, "y_out is not 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    FusedSrc src{};
    src.y = static_cast<const int*>(P->y_snap);
    src.touched = reinterpret_cast<const unsigned char*>(P->touched);
    src.hy = hy; src.wy = wy;
    src.tshift = P->tshift;
    src.sty = P->tshift ? P->cg.sty : hy;
    src.stx = P->tshift ? P->cg.stx : wy;
    src.shift = shift; src.pool = pool ? 1 : 0;
    src.fresh = L->fresh;  // a fresh / reset layer holds no f(P) yet: everything is compared
    src.touched_all = P->ctrl + 3;
    rrm_status rs;
    if ((rs = prof_mark(L, 0, st)) != RRM_OK) return rs;
    RRM_HIP(launch_scan_fused(src, L->x_snap, L->d0, L->bitmap, L->tileflag, L->sg, L->stats, st));
    if ((rs = prof_mark(L, 1, st)) != RRM_OK) return rs;
    if (L->use_pos)
        RRM_HIP(launch_conv_pos(L->dtype, MODE_DELTA, 1, L->d0, L->d1, L->zero16, L->bitmap, L->ctrl, L->wpos, L->bias,
                                L->y_snap, L->pg, L->stats, st));
    else
        RRM_HIP(launch_conv(L->dtype, MODE_DELTA, L->cg.wg_cb, L->cg.nt, 1, L->d0, L->d1, L->zero16, L->tileflag, L->ctrl,
                            L->wpack, L->offtab, L->bias, L->y_snap, L->cg, L->stats, st));
    if ((rs = prof_mark(L, 2, st)) != RRM_OK) return rs;
    L->has_snapshot = true;
    ++L->steps;
    if (y_out) RRM_HIP(launch_copy(y_out, L->y_snap, L->y_bytes, st));
    return RRM_OK;
}

rrm_status rrm_stack_step(const rrm_stack_entry* entries, int n_layers, const void* x_t, void* f_out, void* hip_stream) {
    if (!entries || n_layers < 1) return fail(RRM_ERR_NULL, "entries is NULL or empty");
    for (int i = 0; i < n_layers; ++i)
        if (!entries[i].layer) return fail(RRM_ERR_NULL, "a stack entry has no layer");
    rrm_status st = rrm_step(entries[0].layer, x_t, nullptr, hip_stream);
    for (int i = 1; i < n_layers && st == RRM_OK; ++i)
        st = rrm_step_from_projection(entries[i].layer, entries[i - 1].layer, entries[i - 1].shift, entries[i - 1].pool, nullptr,
                                      hip_stream);
    if (st == RRM_OK && f_out)
        st = rrm_aux_relu_requant_pool_changed_i8(entries[n_layers - 1].layer, f_out, entries[n_layers - 1].shift,
                                                  entries[n_layers - 1].pool, hip_stream);
    return st;
}

rrm_status rrm_dense(rrm_layer* L, const void* x, void* y, void* hip_stream) {
    if (!L) return fail(RRM_ERR_NULL, "layer is NULL");
    rrm_status st = check_ptr(x, "x");
    if (st != RRM_OK) return st;
    if ((st = check_ptr(y, "y")) != RRM_OK) return st;
    return enqueue_dense(L, x, y, static_cast<hipStream_t>(hip_stream));
}

rrm_status rrm_dense_noalloc(rrm_layer* L, const void* x, void* y, void* hip_stream) {
    if (!L) return fail(RRM_ERR_NULL, "layer is NULL");
    rrm_status st = check_ptr(x, "x");
    if (st != RRM_OK) return st;
    if ((st = check_ptr(y, "y")) != RRM_OK) return st;
    if (L->shape.kind != RRM_FC) return fail(RRM_ERR_SHAPE, "rrm_dense_noalloc is available for FC layers");
    const size_t need = (size_t)L->shape.n * (size_t)fc_splits(L) * (size_t)L->fg.c_out_p * 4;
    if (need > FC_STATIC_SCRATCH_BYTES)
        return fail(RRM_ERR_SHAPE, "rrm_dense_noalloc: the layer needs " + std::to_string(need) +
                                       " bytes of partial sums, the static scratch holds " +
                                       std::to_string(FC_STATIC_SCRATCH_BYTES));
    RRM_HIP(launch_fc_dense_static(L->dtype, fc_splits(L), L->wpack, x, L->bias, y, L->fg, static_cast<hipStream_t>(hip_stream)));
    return RRM_OK;
}

rrm_status rrm_reset(rrm_layer* L, void* hip_stream) {
    if (!L) return fail(RRM_ERR_NULL, "layer is NULL");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    RRM_HIP(launch_fill_zero(L->x_snap, round16(L->x_bytes), s));
    RRM_HIP(launch_fill_bias(L->dtype == RRM_BF16_F32, L->y_snap, L->bias, L->y_elems / L->shape.c_out, L->shape.c_out, s));
    if (L->dtype == RRM_BIN_I32) {  // (see rrm_layer_create: the projection of the all -1 frame)
        rrm_status rs = enqueue_dense(L, L->x_snap, L->y_snap, s);
        if (rs != RRM_OK) return rs;
    }
    RRM_HIP(launch_fill_zero(L->stats, sizeof(DevStats) * STAT_SLOTS, s));
    if (L->shape.kind == RRM_CONV) {
        // the difference buffer is zero wherever the bitmap is clear, and no tile is stamped
        RRM_HIP(launch_fill_zero(L->d0, round16(L->d_bytes), s));
        if (L->d1) RRM_HIP(launch_fill_zero(L->d1, round16(L->d_bytes), s));
        RRM_HIP(launch_fill_zero(L->bitmap, round16(((round16(L->x_bytes) / 16 + 63) / 64) * 8), s));
        RRM_HIP(launch_fill_zero(L->tileflag, round16(L->marks_bytes), s));
        RRM_HIP(launch_fill_zero(L->ctrl, 16, s));
        RRM_HIP(launch_fill_word(L->fresh, 16, 1u, s));
        if (L->touched) RRM_HIP(launch_fill_word(L->touched, round16(L->touched_bytes), 0x01010101u, s));
    }
    if (L->bin_arrive) RRM_HIP(launch_fill_zero(L->bin_arrive, round16((size_t)L->shape.n * sizeof(unsigned int)), s));
    if (L->sc_arrive)
        RRM_HIP(launch_fill_zero(L->sc_arrive, round16((size_t)((L->sc.npos_total + L->sc.PB - 1) / L->sc.PB) * sizeof(unsigned int)), s));
    if (L->fc_arrive) RRM_HIP(launch_fill_zero(L->fc_arrive, round16((size_t)L->shape.n * sizeof(unsigned int)), s));
    L->has_snapshot = false;
    L->steps = 0;
    return RRM_OK;
}

rrm_status rrm_snapshot(rrm_layer* L, const void** x_snap, const void** y_snap) {
    if (!L) return fail(RRM_ERR_NULL, "layer is NULL");
    if (x_snap) *x_snap = L->x_snap;
    if (y_snap) *y_snap = L->y_snap;
    return RRM_OK;
}

rrm_status rrm_read_snapshot(rrm_layer* L, void* x_dst, void* y_dst, void* hip_stream) {
    if (!L) return fail(RRM_ERR_NULL, "layer is NULL");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (x_dst) RRM_HIP(hipMemcpyAsync(x_dst, L->x_snap, L->x_bytes, hipMemcpyDeviceToDevice, s));
    if (y_dst) RRM_HIP(hipMemcpyAsync(y_dst, L->y_snap, L->y_bytes, hipMemcpyDeviceToDevice, s));
    return RRM_OK;
}

rrm_status rrm_set_option(rrm_layer* L, const char* key, long value) {
    if (!L) return fail(RRM_ERR_NULL, "layer is NULL");
    if (!key) return fail(RRM_ERR_NULL, "key is NULL");
    const std::string k(key);
    if (k == "path") {
        if (value < 0 || value > 3) return fail(RRM_ERR_OPTION, "path must be 0, 1, 2 or 3");
        if (value == 3 && !L->scat_ok)
            return fail(RRM_ERR_OPTION, "path 3 (single-launch scatter) needs an int8 / bf16 convolution with 16-byte channel runs");
        L->opt_path = (int)value;
    } else if (k == "fc_splits") {
        // the scratch of the partial sums was sized for fc_nsplit at create: only fewer are allowed
        if (L->shape.kind != RRM_FC || value < 1 || value > L->fc_nsplit)
            return fail(RRM_ERR_OPTION, "fc_splits must be in [1, the layer's default]");
        L->opt_fc_splits = (int)value;
    } else if (k == "bf16_terms") {
        if (value != 1 && value != 2) return fail(RRM_ERR_OPTION, "bf16_terms must be 1 or 2");
        L->opt_terms = (int)value;
    } else if (k == "dense_switch_pct") {
        if (value < 1 || value > 100) return fail(RRM_ERR_OPTION, "dense_switch_pct must be in [1, 100]");
        L->cg.full_pct = (int)value;
        L->pg.full_pct = (int)value;
    } else if (k == "conv_kernel") {
        if (L->shape.kind != RRM_CONV || L->dtype == RRM_BIN_I32 || value < 0 || value > 2)
            return fail(RRM_ERR_OPTION, "conv_kernel is 0, 1 or 2, for int8 / bf16 convolution layers");
        L->opt_conv_kernel = (int)value;
        return select_conv_kernel(L, (int)value);
    } else if (k == "profile") {
        if (value != 0 && value != 1) return fail(RRM_ERR_OPTION, "profile must be 0 or 1");
        L->prof_on = value != 0;
        L->prof_n = 0;
    } else if (k == "fc_batched") {
        if (L->shape.kind != RRM_FC || (value != 0 && value != 1)) return fail(RRM_ERR_OPTION, "fc_batched is 0 or 1, for FC layers");
        L->opt_fc_batched = (int)value;
    } else if (k == "fc_sparse_weights") {
        if (L->shape.kind != RRM_FC || (value != 0 && value != 1)) return fail(RRM_ERR_OPTION, "fc_sparse_weights is 0 or 1, for FC layers");
        if (value == 1 && !L->csc_ok)
            return fail(RRM_ERR_OPTION, "fc_sparse_weights: the layer holds no non-zero lists (more than half of its weights "
                                         "are non-zero, or c_out is above 24576)");
        L->use_csc = value == 1;
    } else if (k == "bin_single_launch") {
        if (L->dtype != RRM_BIN_I32 || (value != 0 && value != 1)) return fail(RRM_ERR_OPTION, "bin_single_launch is 0 or 1, for binary layers");
        L->opt_bin_fused = (int)value;
    } else if (k == "bin_cout_per_wave") {
        if (value != 0 && value != 8 && value != 16) return fail(RRM_ERR_OPTION, "bin_cout_per_wave must be 0, 8 or 16");
        L->opt_bin_cw = (int)value;
    } else {
        return fail(RRM_ERR_OPTION, "unknown option key: " + k);
    }
    return RRM_OK;
}

rrm_status rrm_set_threshold(rrm_layer* L, float epsilon) {
    if (!L) return fail(RRM_ERR_NULL, "layer is NULL");
    if (L->dtype != RRM_BF16_F32) return fail(RRM_ERR_DTYPE, "the truncation threshold is defined for BF16 layers");
    if (!(epsilon >= 0.0f) || epsilon > 3.0e38f) return fail(RRM_ERR_OPTION, "epsilon must be finite and >= 0");
    L->sg.eps = epsilon;
    L->fg.eps = epsilon;
    return RRM_OK;
}

rrm_status rrm_get_stats(rrm_layer* L, rrm_stats* out) {
    if (!L) return fail(RRM_ERR_NULL, "layer is NULL");
    if (!out) return fail(RRM_ERR_NULL, "out is NULL");
    DevStats slots[STAT_SLOTS];
    RRM_HIP(hipMemcpy(slots, L->stats, sizeof(slots), hipMemcpyDeviceToHost));
    DevStats d{};
    for (const DevStats& t : slots) {
        d.changed_elems += t.changed_elems;
        d.changed_units += t.changed_units;
        d.active_tiles += t.active_tiles;
        d.range_error |= t.range_error;
        d.truncated_elems += t.truncated_elems;
        d.truncated_sumsq += t.truncated_sumsq;
        d.delta_steps += t.delta_steps;
        d.total_tiles += t.total_tiles;
    }
    out->steps = L->steps;
    out->delta_steps = d.delta_steps;
    out->changed_elems = d.changed_elems;
    out->changed_units = d.changed_units;
    out->active_tiles = d.active_tiles;
    out->total_tiles = d.total_tiles;
    out->range_error = (int32_t)d.range_error;
    out->tile_positions = L->shape.kind == RRM_FC ? 0 : (L->dtype == RRM_BIN_I32 ? (L->bg.band_rows > 0 ? 1 : TILE * TILE) : (L->use_pos ? 1 : 16));
    out->truncated_elems = d.truncated_elems;
    out->truncated_sumsq = d.truncated_sumsq;
    if (d.range_error) return fail(RRM_ERR_RANGE, "an int8 input difference did not fit int8");
    return RRM_OK;
}

rrm_status rrm_get_kernel_times(rrm_layer* L, double* scan_us, double* compute_us, int* steps) {
    if (!L) return fail(RRM_ERR_NULL, "layer is NULL");
    double a = 0.0, c = 0.0;
    for (int i = 0; i < L->prof_n; ++i) {
        float ms = 0.f;
        RRM_HIP(hipEventSynchronize(L->prof_ev[(size_t)3 * i + 2]));
        RRM_HIP(hipEventElapsedTime(&ms, L->prof_ev[(size_t)3 * i], L->prof_ev[(size_t)3 * i + 1]));
        a += 1e3 * ms;
        RRM_HIP(hipEventElapsedTime(&ms, L->prof_ev[(size_t)3 * i + 1], L->prof_ev[(size_t)3 * i + 2]));
        c += 1e3 * ms;
    }
    if (scan_us) *scan_us = a;
    if (compute_us) *compute_us = c;
    if (steps) *steps = L->prof_n;
    L->prof_n = 0;
    return RRM_OK;
}

void rrm_layer_destroy(rrm_layer* L) { delete L; }

const char* rrm_status_string(int status) {
    switch (status) {
        case RRM_OK: return "ok";
        case RRM_ERR_NULL: return "null pointer";
        case RRM_ERR_SHAPE: return "unsupported shape";
        case RRM_ERR_DTYPE: return "unsupported dtype";
        case RRM_ERR_ALLOC: return "allocation failed";
        case RRM_ERR_HIP: return "HIP runtime error";
        case RRM_ERR_STATE: return "invalid state";
        case RRM_ERR_RANGE: return "int8 difference out of range";
        case RRM_ERR_OPTION: return "unknown option";
        case RRM_ERR_ALIGN: return "misaligned pointer";
        default: return "unknown status";
    }
}

const char* rrm_last_error(void) { return g_last_error.c_str(); }

rrm_status rrm_aux_relu_requant_pool_i8(const void* y, void* out, int n, int h, int w, int c, int shift, int pool,
                                        void* hip_stream) {
    if (!y || !out) return fail(RRM_ERR_NULL, "y / out is NULL");
    if (n < 1 || h < 1 || w < 1 || c < 1 || shift < 0 || shift > 31 || (pool && (h < 3 || w < 3)))
        return fail(RRM_ERR_SHAPE, "bad shape for relu_requant_pool");
    RRM_HIP(launch_relu_requant_pool(y, out, nullptr, nullptr, 0, n, h, w, c, shift, pool, static_cast<hipStream_t>(hip_stream)));
    return RRM_OK;
}

rrm_status rrm_aux_probe_mfma(int dtype, void* sink, int iters, int workgroups, void* hip_stream) {
    if (!sink) return fail(RRM_ERR_NULL, "sink is NULL");
    if (dtype != RRM_I8_I32 && dtype != RRM_BF16_F32) return fail(RRM_ERR_DTYPE, "the matrix-core probe runs int8 or bf16 tiles");
    if (iters < 1 || iters > (1 << 20) || workgroups < 1 || workgroups > (1 << 16))
        return fail(RRM_ERR_SHAPE, "probe: iters in [1, 2^20], workgroups in [1, 2^16]");
    RRM_HIP(launch_probe_mfma(dtype == RRM_BF16_F32, sink, iters, workgroups, static_cast<hipStream_t>(hip_stream)));
    return RRM_OK;
}

rrm_status rrm_aux_probe_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
    if (!dst || !src) return fail(RRM_ERR_NULL, "dst / src is NULL");
    if (((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15) != 0)
        return fail(RRM_ERR_ALIGN, "probe copy: pointers must be 16-byte aligned");
    RRM_HIP(launch_probe_copy(dst, src, bytes, static_cast<hipStream_t>(hip_stream)));
    return RRM_OK;
}

rrm_status rrm_aux_relu_requant_pool_changed_i8(rrm_layer* L, void* out, int shift, int pool, void* hip_stream) {
    if (!L || !out) return fail(RRM_ERR_NULL, "layer / out is NULL");
    const rrm_shape& s = L->shape;
    if (s.kind != RRM_CONV || L->dtype != RRM_I8_I32 || !L->touched || s.c_out % 4 != 0)
        return fail(RRM_ERR_SHAPE, "the incremental nonlinearity needs an int8 conv layer with c_out % 4 == 0");
    const int ho = L->cg.ho, wo = L->cg.wo;
    if (shift < 0 || shift > 31 || (pool && (ho < 3 || wo < 3))) return fail(RRM_ERR_SHAPE, "bad shape for relu_requant_pool");
    if (reinterpret_cast<uintptr_t>(out) & 3) return fail(RRM_ERR_ALIGN, "out must be 4-byte aligned");
    RRM_HIP(launch_relu_requant_pool(L->y_snap, out, L->touched, L->ctrl + 3, L->tshift, s.n, ho, wo, s.c_out, shift, pool,
                                     static_cast<hipStream_t>(hip_stream)));
    return RRM_OK;
}

#pragma GCC visibility pop
}  // extern "C"
