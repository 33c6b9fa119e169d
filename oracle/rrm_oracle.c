/*
 * CPU oracle for the Recurrent Residual Module's per-layer update.  TEST INFRASTRUCTURE ONLY:
 * it is called by the tests, by the smoke check and by the benchmark's CPU-baseline leg, never
 * by the product path, and it shares no code with the HIP library.
 *
 * What it computes, written out as plainly as possible:
 *
 *   orc_dense_*  the projection layer P = F * I + b (convolution) or P = W I + b (fully
 *                connected) of the paper's Eq. 3 (Sec. 3.1), as a direct nested-loop
 *                cross-correlation / matrix-vector product.  Because the method reaches
 *                exactly the dense result ("feature maps of each frame are precisely
 *                computed", abstract; Eq. 4), this definition is the expected value of every
 *                frame.
 *   orc_step_*   one (layer, frame) iteration of Algorithm 1 (Sec. 3.2): the difference
 *                I_t - I_{t-1}, the product of the layer's weights with that difference done
 *                input-stationary (every non-zero difference is scattered into the outputs it
 *                touches, zero entries are skipped as the sparse engine of Sec. 3.5 does), the
 *                sum into the stored projection, and the snapshot of the input.
 *
 * Layouts: activations NHWC, convolution weights [c_out][kh][kw][c_in/groups], FC weights
 * [c_out][c_in], outputs NHWC.  "Convolution" is cross-correlation (no kernel flip); taps that
 * fall outside the image contribute 0.
 *
 * Integer paths accumulate in 64 bits and report (return value 1) if any result does not fit
 * an int32; floating-point paths take doubles (bf16 inputs are widened exactly by the caller)
 * and accumulate in double.
 *
 * Pins (see tests/test_oracle_*.py): impulse response, all-ones tap counts, the 1x1 and
 * full-window special cases that reduce to a matrix-vector product, an independent library
 * convolution in float64, brute force on tiny layers and the linearity invariants of Eq. 4.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int kind;   /* 0 = convolution, 1 = fully connected */
    int n, h, w, c_in, c_out, kh, kw, stride, pad, groups;
} orc_shape;

static int out_h(const orc_shape* s) { return (s->h + 2 * s->pad - s->kh) / s->stride + 1; }
static int out_w(const orc_shape* s) { return (s->w + 2 * s->pad - s->kw) / s->stride + 1; }

int orc_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_threads(int t) {
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

/* ------------------------------------------------------------------------------------------
 * Eq. 3, dense.  Output-stationary: one output element at a time gathers its taps.
 * ---------------------------------------------------------------------------------------- */
int orc_dense_i8(const orc_shape* s, const int8_t* wt, const int32_t* bias, const int8_t* x, int32_t* y) {
    int overflow = 0;
    if (s->kind == 1) {
#pragma omp parallel for collapse(2) reduction(| : overflow)
        for (int b = 0; b < s->n; ++b)
            for (int o = 0; o < s->c_out; ++o) {
                int64_t acc = bias ? bias[o] : 0;
                for (int j = 0; j < s->c_in; ++j)
                    acc += (int64_t)wt[(size_t)o * s->c_in + j] * x[(size_t)b * s->c_in + j];
                if (acc > INT32_MAX || acc < INT32_MIN) overflow = 1;
                y[(size_t)b * s->c_out + o] = (int32_t)acc;
            }
        return overflow;
    }
    const int ho = out_h(s), wo = out_w(s);
    const int cg = s->c_in / s->groups, og = s->c_out / s->groups;
#pragma omp parallel for collapse(2) reduction(| : overflow)
    for (int b = 0; b < s->n; ++b)
        for (int oy = 0; oy < ho; ++oy)
            for (int ox = 0; ox < wo; ++ox)
                for (int o = 0; o < s->c_out; ++o) {
                    const int g = o / og;
                    int64_t acc = bias ? bias[o] : 0;
                    for (int ky = 0; ky < s->kh; ++ky) {
                        const int iy = oy * s->stride - s->pad + ky;
                        if (iy < 0 || iy >= s->h) continue;
                        for (int kx = 0; kx < s->kw; ++kx) {
                            const int ix = ox * s->stride - s->pad + kx;
                            if (ix < 0 || ix >= s->w) continue;
                            const int8_t* xp = x + (((size_t)b * s->h + iy) * s->w + ix) * s->c_in + (size_t)g * cg;
                            const int8_t* wp = wt + (((size_t)o * s->kh + ky) * s->kw + kx) * cg;
                            for (int c = 0; c < cg; ++c) acc += (int64_t)wp[c] * xp[c];
                        }
                    }
                    if (acc > INT32_MAX || acc < INT32_MIN) overflow = 1;
                    y[(((size_t)b * ho + oy) * wo + ox) * s->c_out + o] = (int32_t)acc;
                }
    return overflow;
}

int orc_dense_f64(const orc_shape* s, const double* wt, const double* bias, const double* x, double* y) {
    if (s->kind == 1) {
#pragma omp parallel for collapse(2)
        for (int b = 0; b < s->n; ++b)
            for (int o = 0; o < s->c_out; ++o) {
                double acc = bias ? bias[o] : 0.0;
                for (int j = 0; j < s->c_in; ++j)
                    acc += wt[(size_t)o * s->c_in + j] * x[(size_t)b * s->c_in + j];
                y[(size_t)b * s->c_out + o] = acc;
            }
        return 0;
    }
    const int ho = out_h(s), wo = out_w(s);
    const int cg = s->c_in / s->groups, og = s->c_out / s->groups;
#pragma omp parallel for collapse(2)
    for (int b = 0; b < s->n; ++b)
        for (int oy = 0; oy < ho; ++oy)
            for (int ox = 0; ox < wo; ++ox)
                for (int o = 0; o < s->c_out; ++o) {
                    const int g = o / og;
                    double acc = bias ? bias[o] : 0.0;
                    for (int ky = 0; ky < s->kh; ++ky) {
                        const int iy = oy * s->stride - s->pad + ky;
                        if (iy < 0 || iy >= s->h) continue;
                        for (int kx = 0; kx < s->kw; ++kx) {
                            const int ix = ox * s->stride - s->pad + kx;
                            if (ix < 0 || ix >= s->w) continue;
                            const double* xp = x + (((size_t)b * s->h + iy) * s->w + ix) * s->c_in + (size_t)g * cg;
                            const double* wp = wt + (((size_t)o * s->kh + ky) * s->kw + kx) * cg;
                            for (int c = 0; c < cg; ++c) acc += wp[c] * xp[c];
                        }
                    }
                    y[(((size_t)b * ho + oy) * wo + ox) * s->c_out + o] = acc;
                }
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Algorithm 1, one (layer, frame) iteration.  Input-stationary: every non-zero entry of the
 * difference is multiplied with the weights that see it and added into the stored projection.
 *   i_prev : I_{t-1,l}, overwritten with I_{t,l}
 *   p_prev : P_{(t-1)l}, overwritten with P_{tl}
 *   nnz    : (out, may be NULL) number of non-zero entries of the difference
 * The bias is not touched here: it entered the stored projection when the state was
 * initialised (P_0 = b, the value of Eq. 3 at I_0 = 0).
 * ---------------------------------------------------------------------------------------- */
int orc_step_i8(const orc_shape* s, const int8_t* wt, int8_t* i_prev, int32_t* p_prev, const int8_t* x_t,
                int64_t* nnz) {
    int overflow = 0;
    int64_t count = 0;
    if (s->kind == 1) {
        for (int b = 0; b < s->n; ++b)
            for (int j = 0; j < s->c_in; ++j) {
                const int d = (int)x_t[(size_t)b * s->c_in + j] - (int)i_prev[(size_t)b * s->c_in + j];
                if (d == 0) continue;
                ++count;
                for (int o = 0; o < s->c_out; ++o) {
                    int64_t v = (int64_t)p_prev[(size_t)b * s->c_out + o] + (int64_t)d * wt[(size_t)o * s->c_in + j];
                    if (v > INT32_MAX || v < INT32_MIN) overflow = 1;
                    p_prev[(size_t)b * s->c_out + o] = (int32_t)v;
                }
                i_prev[(size_t)b * s->c_in + j] = x_t[(size_t)b * s->c_in + j];
            }
        if (nnz) *nnz = count;
        return overflow;
    }
    const int ho = out_h(s), wo = out_w(s);
    const int cg = s->c_in / s->groups, og = s->c_out / s->groups;
    for (int b = 0; b < s->n; ++b)
        for (int iy = 0; iy < s->h; ++iy)
            for (int ix = 0; ix < s->w; ++ix)
                for (int ci = 0; ci < s->c_in; ++ci) {
                    const size_t xi = (((size_t)b * s->h + iy) * s->w + ix) * s->c_in + ci;
                    const int d = (int)x_t[xi] - (int)i_prev[xi];
                    if (d == 0) continue;
                    ++count;
                    const int g = ci / cg, c = ci % cg;
                    for (int ky = 0; ky < s->kh; ++ky) {
                        const int ty = iy + s->pad - ky;
                        if (ty < 0 || ty % s->stride) continue;
                        const int oy = ty / s->stride;
                        if (oy >= ho) continue;
                        for (int kx = 0; kx < s->kw; ++kx) {
                            const int tx = ix + s->pad - kx;
                            if (tx < 0 || tx % s->stride) continue;
                            const int ox = tx / s->stride;
                            if (ox >= wo) continue;
                            for (int oo = 0; oo < og; ++oo) {
                                const int o = g * og + oo;
                                const size_t yi = (((size_t)b * ho + oy) * wo + ox) * s->c_out + o;
                                int64_t v = (int64_t)p_prev[yi] +
                                            (int64_t)d * wt[(((size_t)o * s->kh + ky) * s->kw + kx) * cg + c];
                                if (v > INT32_MAX || v < INT32_MIN) overflow = 1;
                                p_prev[yi] = (int32_t)v;
                            }
                        }
                    }
                    i_prev[xi] = x_t[xi];
                }
    if (nnz) *nnz = count;
    return overflow;
}

/* Sparsity enhancement (Sec. 3.4, "Improving sparsity"): a difference whose magnitude is below the threshold
 * eps is truncated to zero.  Reading taken here: only what was applied to P is committed to I, so that
 * P = b + W (*) I stays true and a truncated difference is still pending at the next frame (nothing is lost
 * for good).  The decision is taken on the single-precision difference, the precision the inputs' difference
 * is formed in on the device.  eps = 0 is the exact method.  ntrunc / sumsq (nullable) receive the number
 * of truncated entries and the sum of their squares (the l2 norm of the truncated map of Eq. 7, squared). */
int orc_step_f64(const orc_shape* s, const double* wt, double* i_prev, double* p_prev, const double* x_t,
                 float eps, int64_t* nnz, int64_t* ntrunc, double* sumsq) {
    int64_t count = 0, ntr = 0;
    double ssq = 0.0;
    if (s->kind == 1) {
        for (int b = 0; b < s->n; ++b)
            for (int j = 0; j < s->c_in; ++j) {
                const double d = x_t[(size_t)b * s->c_in + j] - i_prev[(size_t)b * s->c_in + j];
                if (d == 0.0) continue;
                const float d32 = (float)x_t[(size_t)b * s->c_in + j] - (float)i_prev[(size_t)b * s->c_in + j];
                if (fabsf(d32) < eps) {
                    ++ntr;
                    ssq += (double)d32 * (double)d32;
                    continue;
                }
                ++count;
                for (int o = 0; o < s->c_out; ++o)
                    p_prev[(size_t)b * s->c_out + o] += d * wt[(size_t)o * s->c_in + j];
                i_prev[(size_t)b * s->c_in + j] = x_t[(size_t)b * s->c_in + j];
            }
        if (nnz) *nnz = count;
        if (ntrunc) *ntrunc = ntr;
        if (sumsq) *sumsq = ssq;
        return 0;
    }
    const int ho = out_h(s), wo = out_w(s);
    const int cg = s->c_in / s->groups, og = s->c_out / s->groups;
    for (int b = 0; b < s->n; ++b)
        for (int iy = 0; iy < s->h; ++iy)
            for (int ix = 0; ix < s->w; ++ix)
                for (int ci = 0; ci < s->c_in; ++ci) {
                    const size_t xi = (((size_t)b * s->h + iy) * s->w + ix) * s->c_in + ci;
                    const double d = x_t[xi] - i_prev[xi];
                    if (d == 0.0) continue;
                    const float d32 = (float)x_t[xi] - (float)i_prev[xi];
                    if (fabsf(d32) < eps) {
                        ++ntr;
                        ssq += (double)d32 * (double)d32;
                        continue;
                    }
                    ++count;
                    const int g = ci / cg, c = ci % cg;
                    for (int ky = 0; ky < s->kh; ++ky) {
                        const int ty = iy + s->pad - ky;
                        if (ty < 0 || ty % s->stride) continue;
                        const int oy = ty / s->stride;
                        if (oy >= ho) continue;
                        for (int kx = 0; kx < s->kw; ++kx) {
                            const int tx = ix + s->pad - kx;
                            if (tx < 0 || tx % s->stride) continue;
                            const int ox = tx / s->stride;
                            if (ox >= wo) continue;
                            for (int oo = 0; oo < og; ++oo) {
                                const int o = g * og + oo;
                                p_prev[(((size_t)b * ho + oy) * wo + ox) * s->c_out + o] +=
                                    d * wt[(((size_t)o * s->kh + ky) * s->kw + kx) * cg + c];
                            }
                        }
                    }
                    i_prev[xi] = x_t[xi];
                }
    if (nnz) *nnz = count;
    if (ntrunc) *ntrunc = ntr;
    if (sumsq) *sumsq = ssq;
    return 0;
}
