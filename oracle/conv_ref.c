/*
 * conv_ref.c -- CPU oracle for the Convolution op family.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct fp64 definitions of what the GPU path computes:
 *   Convolution forward (+ optional bias / ReLU compound epilogue),
 *   ConvolutionBackpropData, ConvolutionBackpropFilters,
 *   the NCHW <-> 16-channel-blocked layout permutation, and a bf16 rounding helper.
 *
 * The paper (Sec. 2, "Intermediate Representation") only says that an op is a
 * stateless node whose inputs and constant attributes fix the output shape, and
 * (Sec. 3, "Framework Bridges") that derivative ops come from autodiff of the
 * forward op; (Sec. 4, "Transformers") names convolution as a backend kernel.  It
 * prints no formula.  The formulas below are the standard deep-learning
 * definitions: cross-correlation (no filter flip), filters [K,C,R,S], data
 * [N,C,H,W], window strides, padding below (low index side) / above (high index
 * side), window dilation, floor output size; the two backprops are the exact
 * adjoints of forward with respect to data and filters.
 *
 * Nothing in the product (the HIP library, its Python binding) may call this
 * file; only tests, the smoke check and the benchmark's cpu_baseline leg do.
 * It shares no code, header, table or helper with the HIP path.
 *
 * Parallelism: OpenMP over independent outputs only; every output element is
 * produced by one thread with a fixed summation order (c, then r, then s / k, r, s
 * / n, p, q), so results do not depend on the thread count.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>

typedef struct {
    int32_t n, c, h, w;                 /* data batch shape   [N,C,H,W]          */
    int32_t k, r, s;                    /* filters            [K,C,R,S]          */
    int32_t sh, sw;                     /* window movement strides               */
    int32_t dh, dw;                     /* window dilation                       */
    int32_t pbh, pbw;                   /* padding below (top / left)            */
    int32_t pah, paw;                   /* padding above (bottom / right)        */
} ref_attrs;

/* Output extent along one axis: number of window placements that fit (floor). */
int32_t ref_out_dim(int32_t in, int32_t pb, int32_t pa, int32_t dil, int32_t win, int32_t stride)
{
    int32_t span = in + pb + pa - dil * (win - 1) - 1;
    if (span < 0) return 0;
    return span / stride + 1;
}

static int32_t out_p(const ref_attrs *a) { return ref_out_dim(a->h, a->pbh, a->pah, a->dh, a->r, a->sh); }
static int32_t out_q(const ref_attrs *a) { return ref_out_dim(a->w, a->pbw, a->paw, a->dw, a->s, a->sw); }

#define X_AT(a, n_, c_, i_, j_) ((((size_t)(n_) * (a)->c + (c_)) * (a)->h + (i_)) * (a)->w + (j_))
#define W_AT(a, k_, c_, r_, s_) ((((size_t)(k_) * (a)->c + (c_)) * (a)->r + (r_)) * (a)->s + (s_))
#define Y_AT(a, P_, Q_, n_, k_, p_, q_) ((((size_t)(n_) * (a)->k + (k_)) * (P_) + (p_)) * (Q_) + (q_))

/* ---- forward: y[n,k,p,q] = sum_{c,r,s} X(n,c, p*sh-pbh+r*dh, q*sw-pbw+s*dw) * w[k,c,r,s],
 *      X = x inside the image, 0 outside. ------------------------------------------------ */
static double fwd_elem(const ref_attrs *a, const double *x, const double *w,
                       int n, int k, int p, int q)
{
    double acc = 0.0;
    for (int c = 0; c < a->c; ++c)
        for (int r = 0; r < a->r; ++r) {
            int i = p * a->sh - a->pbh + r * a->dh;
            if (i < 0 || i >= a->h) continue;
            for (int s = 0; s < a->s; ++s) {
                int j = q * a->sw - a->pbw + s * a->dw;
                if (j < 0 || j >= a->w) continue;
                acc += x[X_AT(a, n, c, i, j)] * w[W_AT(a, k, c, r, s)];
            }
        }
    return acc;
}

/* compound epilogue on the fp64 result: z = y (+ b[k]) ; z = max(z, 0) */
static double epilogue(double y, const double *bias, int k, int relu)
{
    double z = y;
    if (bias) z += bias[k];
    if (relu && z < 0.0) z = 0.0;
    return z;
}

void ref_conv_fwd(const ref_attrs *a, const double *x, const double *w,
                  const double *bias /* NULL = none */, int relu, double *y)
{
    const int P = out_p(a), Q = out_q(a);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < a->n; ++n)
        for (int k = 0; k < a->k; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q)
                    y[Y_AT(a, P, Q, n, k, p, q)] = epilogue(fwd_elem(a, x, w, n, k, p, q), bias, k, relu);
}

/* the same definition evaluated at a list of flat indices into y[N,K,P,Q] */
void ref_conv_fwd_at(const ref_attrs *a, const double *x, const double *w,
                     const double *bias, int relu, int64_t count, const int64_t *flat, double *out)
{
    const int P = out_p(a), Q = out_q(a);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < count; ++t) {
        int64_t f = flat[t];
        int q = (int)(f % Q); f /= Q;
        int p = (int)(f % P); f /= P;
        int k = (int)(f % a->k); f /= a->k;
        int n = (int)f;
        out[t] = epilogue(fwd_elem(a, x, w, n, k, p, q), bias, k, relu);
    }
}

/* ---- backprop-data, scatter form: every term dy[n,k,p,q]*w[k,c,r,s] of the forward sum is
 *      sent back to the x element it multiplied.  Pixels no window touches stay 0. ---------- */
void ref_conv_bwd_data(const ref_attrs *a, const double *dy, const double *w, double *dx)
{
    const int P = out_p(a), Q = out_q(a);
    memset(dx, 0, sizeof(double) * (size_t)a->n * a->c * a->h * a->w);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < a->n; ++n)              /* images own disjoint slabs of dx */
        for (int k = 0; k < a->k; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double g = dy[Y_AT(a, P, Q, n, k, p, q)];
                    for (int c = 0; c < a->c; ++c)
                        for (int r = 0; r < a->r; ++r) {
                            int i = p * a->sh - a->pbh + r * a->dh;
                            if (i < 0 || i >= a->h) continue;
                            for (int s = 0; s < a->s; ++s) {
                                int j = q * a->sw - a->pbw + s * a->dw;
                                if (j < 0 || j >= a->w) continue;
                                dx[X_AT(a, n, c, i, j)] += g * w[W_AT(a, k, c, r, s)];
                            }
                        }
                }
}

/* ---- backprop-data, gather form (second, independent path):
 *      dx[n,c,i,j] = sum_{k,r,s} dy[n,k,p,q]*w[k,c,r,s] over (p,r) with p*sh-pbh+r*dh = i,
 *      0<=p<P, and (q,s) likewise. ----------------------------------------------------------- */
static double bwd_data_elem(const ref_attrs *a, int P, int Q, const double *dy, const double *w,
                            int n, int c, int i, int j)
{
    double acc = 0.0;
    for (int k = 0; k < a->k; ++k)
        for (int r = 0; r < a->r; ++r) {
            int pn = i + a->pbh - r * a->dh;
            if (pn < 0 || pn % a->sh != 0) continue;
            int p = pn / a->sh;
            if (p >= P) continue;
            for (int s = 0; s < a->s; ++s) {
                int qn = j + a->pbw - s * a->dw;
                if (qn < 0 || qn % a->sw != 0) continue;
                int q = qn / a->sw;
                if (q >= Q) continue;
                acc += dy[Y_AT(a, P, Q, n, k, p, q)] * w[W_AT(a, k, c, r, s)];
            }
        }
    return acc;
}

void ref_conv_bwd_data_gather(const ref_attrs *a, const double *dy, const double *w, double *dx)
{
    const int P = out_p(a), Q = out_q(a);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < a->n; ++n)
        for (int c = 0; c < a->c; ++c)
            for (int i = 0; i < a->h; ++i)
                for (int j = 0; j < a->w; ++j)
                    dx[X_AT(a, n, c, i, j)] = bwd_data_elem(a, P, Q, dy, w, n, c, i, j);
}

void ref_conv_bwd_data_at(const ref_attrs *a, const double *dy, const double *w,
                          int64_t count, const int64_t *flat, double *out)
{
    const int P = out_p(a), Q = out_q(a);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < count; ++t) {
        int64_t f = flat[t];
        int j = (int)(f % a->w); f /= a->w;
        int i = (int)(f % a->h); f /= a->h;
        int c = (int)(f % a->c); f /= a->c;
        int n = (int)f;
        out[t] = bwd_data_elem(a, P, Q, dy, w, n, c, i, j);
    }
}

/* ---- backprop-filters: dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * X(n,c, p*sh-pbh+r*dh, q*sw-pbw+s*dw) */
static double bwd_filters_elem(const ref_attrs *a, int P, int Q, const double *x, const double *dy,
                               int k, int c, int r, int s)
{
    double acc = 0.0;
    for (int n = 0; n < a->n; ++n)
        for (int p = 0; p < P; ++p) {
            int i = p * a->sh - a->pbh + r * a->dh;
            if (i < 0 || i >= a->h) continue;
            for (int q = 0; q < Q; ++q) {
                int j = q * a->sw - a->pbw + s * a->dw;
                if (j < 0 || j >= a->w) continue;
                acc += dy[Y_AT(a, P, Q, n, k, p, q)] * x[X_AT(a, n, c, i, j)];
            }
        }
    return acc;
}

void ref_conv_bwd_filters(const ref_attrs *a, const double *x, const double *dy, double *dw)
{
    const int P = out_p(a), Q = out_q(a);
#pragma omp parallel for collapse(2) schedule(static)
    for (int k = 0; k < a->k; ++k)
        for (int c = 0; c < a->c; ++c)
            for (int r = 0; r < a->r; ++r)
                for (int s = 0; s < a->s; ++s)
                    dw[W_AT(a, k, c, r, s)] = bwd_filters_elem(a, P, Q, x, dy, k, c, r, s);
}

void ref_conv_bwd_filters_at(const ref_attrs *a, const double *x, const double *dy,
                             int64_t count, const int64_t *flat, double *out)
{
    const int P = out_p(a), Q = out_q(a);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < count; ++t) {
        int64_t f = flat[t];
        int s = (int)(f % a->s); f /= a->s;
        int r = (int)(f % a->r); f /= a->r;
        int c = (int)(f % a->c); f /= a->c;
        int k = (int)f;
        out[t] = bwd_filters_elem(a, P, Q, x, dy, k, c, r, s);
    }
}

/* ---- layout permutation: blocked[n][cb][h][w][ci] = nchw[n][16*cb+ci][h][w], tail lanes +0.
 *      Pure copies of bit patterns; elem_bytes is 2 (bf16) or 4 (fp32). ------------------------ */
void ref_nchw_to_blocked16(int32_t n, int32_t c, int32_t h, int32_t w, int32_t elem_bytes,
                           const void *src, void *dst)
{
    const int CB = (c + 15) / 16;
    const unsigned char *s = (const unsigned char *)src;
    unsigned char *d = (unsigned char *)dst;
    for (int in = 0; in < n; ++in)
        for (int cb = 0; cb < CB; ++cb)
            for (int ih = 0; ih < h; ++ih)
                for (int iw = 0; iw < w; ++iw)
                    for (int ci = 0; ci < 16; ++ci) {
                        size_t o = (((((size_t)in * CB + cb) * h + ih) * w + iw) * 16 + ci) * elem_bytes;
                        int ch = 16 * cb + ci;
                        if (ch < c) {
                            size_t i = ((((size_t)in * c + ch) * h + ih) * w + iw) * elem_bytes;
                            memcpy(d + o, s + i, (size_t)elem_bytes);
                        } else {
                            memset(d + o, 0, (size_t)elem_bytes);
                        }
                    }
}

void ref_blocked16_to_nchw(int32_t n, int32_t c, int32_t h, int32_t w, int32_t elem_bytes,
                           const void *src, void *dst)
{
    const int CB = (c + 15) / 16;
    const unsigned char *s = (const unsigned char *)src;
    unsigned char *d = (unsigned char *)dst;
    for (int in = 0; in < n; ++in)
        for (int ch = 0; ch < c; ++ch)
            for (int ih = 0; ih < h; ++ih)
                for (int iw = 0; iw < w; ++iw) {
                    size_t o = ((((size_t)in * c + ch) * h + ih) * w + iw) * elem_bytes;
                    size_t i = (((((size_t)in * CB + ch / 16) * h + ih) * w + iw) * 16 + ch % 16) * elem_bytes;
                    memcpy(d + o, s + i, (size_t)elem_bytes);
                }
}

/* ---- bf16 helper: round an fp32 bit pattern to bf16, round-to-nearest, ties to even.
 *      Written as an explicit case analysis on the discarded 16 bits. ------------------------- */
uint16_t ref_f32_bits_to_bf16_rne(uint32_t u)
{
    uint32_t keep = u >> 16;
    uint32_t drop = u & 0xFFFFu;
    if ((u & 0x7F800000u) == 0x7F800000u) {            /* Inf / NaN: keep class */
        if ((u & 0x007FFFFFu) != 0) keep |= 0x0040u;   /* quiet NaN stays NaN   */
        return (uint16_t)keep;
    }
    if (drop > 0x8000u) keep += 1;                     /* above half: up        */
    else if (drop == 0x8000u && (keep & 1u)) keep += 1;/* tie: to even          */
    return (uint16_t)keep;
}

void ref_f32_to_bf16_rne_array(int64_t count, const uint32_t *f32_bits, uint16_t *bf16_bits)
{
    for (int64_t i = 0; i < count; ++i) bf16_bits[i] = ref_f32_bits_to_bf16_rne(f32_bits[i]);
}

/* ------------------------------------------------------------------------------------------
 * Backward-direction compounding (the derivative of the compounded bias + ReLU forward op;
 * the paper's Sec. 3 obtains derivative graphs by autodiff of the forward ops, Sec. 1 / 4 name
 * the compounding of ops as a backend optimisation; it prints no formula).
 *
 *   ReLU backprop:   g'[i] = g[i] if z[i] > 0 else 0       (z = the ReLU's output or input: same sign test)
 *   bias gradient:   db[k] = sum_{n,p,q} dy[n,k,p,q]       (adjoint of broadcasting b over n, p, q)
 * ------------------------------------------------------------------------------------------ */
void ref_relu_bwd_mask(int64_t count, const double *g, const double *z, double *out)
{
    for (int64_t i = 0; i < count; ++i) out[i] = (z[i] > 0.0) ? g[i] : 0.0;
}

void ref_bias_grad(int32_t n, int32_t k, int32_t p, int32_t q, const double *dy, double *db)
{
    for (int32_t kk = 0; kk < k; ++kk) {
        double acc = 0.0;
        for (int32_t nn = 0; nn < n; ++nn)
            for (int32_t i = 0; i < p * q; ++i) acc += dy[((size_t)nn * k + kk) * p * q + i];
        db[kk] = acc;
    }
}

