// C ABI of the Convolution op family over three spatial axes (include/ngconv.h, second part):
// validation, kernel selection, workspace layout, launches.
//
// Selection per op:
//   1. the window moves over at most one group of adjacent axes while the others are idle (window 1,
//      stride 1, no padding): the op equals the rank-2 op on a reshaped tensor ((D, H*W) with a
//      (T,1) window, or (D*H, W) with a (1,S) window; 1x1x1 is the first with T = 1) and goes to
//      the rank-2 entry point, i.e. to the strip / 1x1 GEMM / per-tap kernels;
//   2. bf16, blocked tensors: the strip kernel with a depth axis (forward / backprop-data; windows of 2..25
//      taps in (h, w), up to 7 depth taps, Cin % 16, Cout % 16), else the gather kernel with a depth axis
//      (Cin % 32, Cout % 64); the per-tap backprop-filters GEMM with a depth axis (C % 16, K % 16);
//   3. the direct kernels (filters [K][C][T][R][S] only).
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "common.h"

namespace {

using namespace ngc;

constexpr size_t MAX_ELEMS3 = (size_t)1 << 31;
constexpr int NUM_CUS3 = 256;

int out_dim3(int extent, int below, int above, int dil, int taps, int stride)
{
    const long long span = (long long)extent + below + above - (long long)dil * (taps - 1) - 1;
    if (span < 0) return 0;
    return (int)(span / stride) + 1;
}

bool layout_ok3(int l) { return l == NGC_NCHW || l == NGC_NCHW16C; }

size_t phys3(int layout, int n, int c, int d, int h, int w)
{
    return (size_t)n * (layout == NGC_NCHW ? c : (c + 15) / 16 * 16) * d * h * w;
}

int validate3(const ngc_conv3d_desc *d, int *O, int *P, int *Q)
{
    if (!d) return NGC_BAD_ARG;
    if (d->dtype != NGC_F32 && d->dtype != NGC_BF16) return NGC_BAD_ARG;
    if (!layout_ok3(d->x_layout) || !layout_ok3(d->y_layout)) return NGC_BAD_ARG;
    if (d->w_layout != NGC_KCRS && d->w_layout != NGC_BLOCKED_FWD && d->w_layout != NGC_BLOCKED_BWD) return NGC_BAD_ARG;
    if (d->epilogue & ~(NGC_EPI_BIAS | NGC_EPI_RELU)) return NGC_BAD_ARG;
    if (d->n < 1 || d->c < 1 || d->d < 1 || d->h < 1 || d->w < 1 || d->k < 1 || d->t < 1 || d->r < 1 || d->s < 1)
        return NGC_BAD_SHAPE;
    if (d->stride_d < 1 || d->stride_h < 1 || d->stride_w < 1 || d->dil_d < 1 || d->dil_h < 1 || d->dil_w < 1) return NGC_BAD_SHAPE;
    if (d->pad_below_d < 0 || d->pad_below_h < 0 || d->pad_below_w < 0 || d->pad_above_d < 0 || d->pad_above_h < 0 ||
        d->pad_above_w < 0)
        return NGC_BAD_SHAPE;
    // keep every intermediate index comfortably inside int32
    const int big[] = {d->d, d->h, d->w, d->pad_below_d, d->pad_below_h, d->pad_below_w, d->pad_above_d, d->pad_above_h, d->pad_above_w};
    for (int v : big)
        if (v > (1 << 20)) return NGC_BAD_SHAPE;
    const int small[] = {d->t, d->r, d->s, d->dil_d, d->dil_h, d->dil_w, d->stride_d, d->stride_h, d->stride_w};
    for (int v : small)
        if (v > 1024) return NGC_BAD_SHAPE;
    const int o = out_dim3(d->d, d->pad_below_d, d->pad_above_d, d->dil_d, d->t, d->stride_d);
    const int p = out_dim3(d->h, d->pad_below_h, d->pad_above_h, d->dil_h, d->r, d->stride_h);
    const int q = out_dim3(d->w, d->pad_below_w, d->pad_above_w, d->dil_w, d->s, d->stride_w);
    if (o < 1 || p < 1 || q < 1) return NGC_BAD_SHAPE;
    if ((double)d->n * ((d->c + 15) / 16 * 16) * d->d * d->h * d->w >= (double)MAX_ELEMS3) return NGC_BAD_SHAPE;
    if ((double)d->n * ((d->k + 15) / 16 * 16) * o * p * q >= (double)MAX_ELEMS3) return NGC_BAD_SHAPE;
    if ((double)((d->k + 15) / 16 * 16) * ((d->c + 15) / 16 * 16) * d->t * d->r * d->s >= (double)MAX_ELEMS3) return NGC_BAD_SHAPE;
    *O = o; *P = p; *Q = q;
    return NGC_OK;
}

bool aligned16_3(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
size_t round256_3(size_t b) { return (b + 255) & ~(size_t)255; }

int status3(hipError_t e)
{
    if (e == hipSuccess) return NGC_OK;
    fprintf(stderr, "ngconv: HIP launch failed: %s\n", hipGetErrorString(e));   // error path only
    return NGC_LAUNCH_FAILED;
}

// Images per launch for operands of 2 GiB or more (bf16, blocked tensors): the ops treat the images of a batch
// independently (backprop-filters up to a final sum), and the MFMA kernels address an operand with 32-bit byte
// offsets.  images == d->n: one launch.
struct BatchSlices3 {
    int images;
    size_t x_bytes, y_bytes;   // of one image
};

BatchSlices3 batch_slices3(const ngc_conv3d_desc *d, int O, int P, int Q)
{
    BatchSlices3 b;
    b.images = d->n;
    b.x_bytes = phys3(d->x_layout, 1, d->c, d->d, d->h, d->w) * 2;
    b.y_bytes = phys3(d->y_layout, 1, d->k, O, P, Q) * 2;
    if (d->dtype != NGC_BF16 || d->x_layout != NGC_NCHW16C || d->y_layout != NGC_NCHW16C) return b;
    const size_t per = b.x_bytes > b.y_bytes ? b.x_bytes : b.y_bytes, lim = (size_t)1 << 31;
    if ((size_t)d->n * per < lim || per >= lim) return b;
    b.images = (int)((lim - 1) / per);
    return b;
}

ngc_conv3d_desc with_batch3(const ngc_conv3d_desc *d, int n)
{
    ngc_conv3d_desc t = *d;
    t.n = n;
    return t;
}

bool idle_axis(int taps, int stride, int below, int above) { return taps == 1 && stride == 1 && below == 0 && above == 0; }

// The rank-2 node this node equals on a reshaped tensor, if there is one.
bool as_rank2(const ngc_conv3d_desc *d, ngc_conv_desc *out)
{
    const char *sw = env_switch(SW_CONV3D_RANK2);         // tests / benchmarks only: 0 = always the rank-3 kernels
    if (sw && atoi(sw) == 0) return false;
    const bool id = idle_axis(d->t, d->stride_d, d->pad_below_d, d->pad_above_d);
    const bool ih = idle_axis(d->r, d->stride_h, d->pad_below_h, d->pad_above_h);
    const bool iw = idle_axis(d->s, d->stride_w, d->pad_below_w, d->pad_above_w);
    ngc_conv_desc t;
    memset(&t, 0, sizeof(t));
    t.n = d->n; t.c = d->c; t.k = d->k;
    t.dtype = d->dtype; t.x_layout = d->x_layout; t.y_layout = d->y_layout; t.w_layout = d->w_layout; t.epilogue = d->epilogue;
    t.stride_h = t.stride_w = t.dil_h = t.dil_w = 1;
    t.r = t.s = 1;
    if (ih && iw) {                                       // (T,1,1): rows = depth slices, columns = H*W
        if ((long long)d->h * d->w > (1 << 20)) return false;
        t.h = d->d; t.w = d->h * d->w;
        t.r = d->t; t.stride_h = d->stride_d; t.dil_h = d->dil_d;
        t.pad_below_h = d->pad_below_d; t.pad_above_h = d->pad_above_d;
    } else if (id && ih) {                                // (1,1,S): rows = D*H, columns = W
        if ((long long)d->d * d->h > (1 << 20)) return false;
        t.h = d->d * d->h; t.w = d->w;
        t.s = d->s; t.stride_w = d->stride_w; t.dil_w = d->dil_w;
        t.pad_below_w = d->pad_below_w; t.pad_above_w = d->pad_above_w;
    } else {
        return false;
    }
    *out = t;
    return true;
}

enum Variant3 { V3_INVALID, V3_UNSUPPORTED, V3_RANK2, V3_STRIP, V3_IGEMM_128, V3_IGEMM_64, V3_WGRAD_GEMM, V3_DIRECT };

bool blocked_bf16_3(const ngc_conv3d_desc *d)
{
    return d->dtype == NGC_BF16 && d->x_layout == NGC_NCHW16C && d->y_layout == NGC_NCHW16C;
}

// Launches of the strip kernel for forward (one) or backprop-data (one per residue class (a, b, c) of the dx voxel
// modulo the strides that has voxels and taps).  The (h, w) part of every launch is planned as the rank-2 node
// over N * OD images; the depth part is the list of depth taps of the class.
struct Strip3Launch {
    StripParams sp;
    int nf;
    size_t lds;
};

struct Strip3Plan {
    int n;
    Strip3Launch l[IGEMM_MAX_CLASSES];
    bool zero;                 // backprop-data: some class with voxels has no tap, dx is cleared first
};

bool strip3_plan(const ngc_conv3d_desc *d, int op, int O, int P, int Q, Strip3Plan *out)
{
    const char *sw = env_switch(SW_CONV3D_STRIP);          // tests / benchmarks only: 0 = the gather kernel instead
    if (sw && atoi(sw) == 0) return false;
    const bool fwd = op == NGC_OP_FWD;
    if (!blocked_bf16_3(d)) return false;
    if (d->w_layout != NGC_KCRS && d->w_layout != (fwd ? NGC_BLOCKED_FWD : NGC_BLOCKED_BWD)) return false;
    const int Cin = fwd ? d->c : d->k, Cout = fwd ? d->k : d->c;
    if (Cin % 16 != 0 || Cout % 16 != 0 || d->t > STRIP_MAX_DT) return false;
    const int sd = d->stride_d, sh = d->stride_h, swd = d->stride_w;
    if (!fwd && sd * sh * swd > IGEMM_MAX_CLASSES) return false;
    const size_t in_bytes = fwd ? (size_t)d->n * d->c * d->d * d->h * d->w * 2 : (size_t)d->n * d->k * O * P * Q * 2;
    const size_t wt_bytes = (size_t)d->t * d->r * d->s * Cin * Cout * 2;
    if (in_bytes >= ((size_t)1 << 31) || wt_bytes >= ((size_t)1 << 31)) return false;

    ngc_conv_desc d2;                                     // the (h, w) part; n is set per launch
    memset(&d2, 0, sizeof(d2));
    d2.c = d->c; d2.h = d->h; d2.w = d->w; d2.k = d->k; d2.r = d->r; d2.s = d->s;
    d2.stride_h = sh; d2.stride_w = swd; d2.dil_h = d->dil_h; d2.dil_w = d->dil_w;
    d2.pad_below_h = d->pad_below_h; d2.pad_below_w = d->pad_below_w;
    d2.pad_above_h = d->pad_above_h; d2.pad_above_w = d->pad_above_w;
    d2.dtype = d->dtype; d2.x_layout = d->x_layout; d2.y_layout = d->y_layout; d2.w_layout = d->w_layout;

    Strip3Plan pl;
    pl.n = 0;
    pl.zero = false;
    const int rs = d->r * d->s;
    for (int a = 0; a < (fwd ? 1 : sd); ++a) {
        int ndt = 0, dt_off[STRIP_MAX_DT], dt_slab[STRIP_MAX_DT];
        for (int t = 0; t < d->t; ++t) {
            if (fwd) {
                dt_off[ndt] = t * d->dil_d - d->pad_below_d;
            } else {
                const int v = a + d->pad_below_d - t * d->dil_d;
                if (((v % sd) + sd) % sd != 0) continue;
                dt_off[ndt] = v / sd;                     // exact
            }
            dt_slab[ndt++] = t * rs;
        }
        const int OD = fwd ? O : (a < d->d ? (d->d - a + sd - 1) / sd : 0);
        if (OD == 0) continue;
        if ((long long)d->n * OD > (1 << 24)) return false;
        d2.n = d->n * OD;
        for (int bc = 0; bc < (fwd ? 1 : sh * swd); ++bc) {
            Strip3Launch L;
            bool empty = false;
            if (!strip_plan_for_class(&d2, op, bc / swd, bc % swd, P, Q, &L.sp, &L.nf, &L.lds, &empty)) return false;
            if (empty || ndt == 0) {
                // no voxel, or voxels no tap reaches (the planner reports both as empty; clearing dx covers the second)
                pl.zero = true;
                continue;
            }
            StripParams &q = L.sp;
            q.r3 = 1;
            q.Din = fwd ? d->d : O;
            q.Dfull = fwd ? O : d->d;
            q.OD = OD;
            q.is_d = fwd ? sd : 1;
            q.os_d = fwd ? 1 : sd;
            q.oa_d = fwd ? 0 : a;
            q.ndt = ndt;
            for (int i = 0; i < ndt; ++i) { q.dt_off[i] = dt_off[i]; q.dt_slab[i] = dt_slab[i]; }
            q.div_od = make_fastdiv((uint32_t)OD);
            q.in_bytes = (uint32_t)in_bytes;
            q.wt_bytes = (uint32_t)wt_bytes;
            pl.l[pl.n++] = L;
        }
    }
    if (fwd) pl.zero = false;
    if (out) *out = pl;
    return true;
}

// tile shape and split of the position axis of the per-tap backprop-filters GEMM
bool wgrad_gemm3_plan(const ngc_conv3d_desc *d, int O, int P, int Q, WgradGemmParams *wp)
{
    const int taps = d->t * d->r * d->s;
    if (!blocked_bf16_3(d) || d->c % 16 != 0 || d->k % 16 != 0 || taps > 64) return false;
    const size_t x_bytes = (size_t)d->n * d->c * d->d * d->h * d->w * 2, dy_bytes = (size_t)d->n * d->k * O * P * Q * 2;
    if (x_bytes >= ((size_t)1 << 31) || dy_bytes >= ((size_t)1 << 31)) return false;
    WgradGemmParams q;
    memset(&q, 0, sizeof(q));
    q.r3 = 1;
    q.N = d->n; q.C = d->c; q.D = d->d; q.H = d->h; q.W = d->w; q.K = d->k; q.O = O; q.P = P; q.Q = Q;
    q.T = d->t; q.R = d->r; q.S = d->s;
    q.sd = d->stride_d; q.sh = d->stride_h; q.sw = d->stride_w;
    q.dil_d = d->dil_d; q.dil_h = d->dil_h; q.dil_w = d->dil_w;
    q.pbd = d->pad_below_d; q.pbh = d->pad_below_h; q.pbw = d->pad_below_w;
    // 128-wide tiles when they waste no more of a partial last tile than 64-wide ones
    auto wide = [](int ch) { return ch > 64 && (ch + 127) / 128 * 128 <= (ch + 63) / 64 * 64; };
    q.wk = wide(d->k) ? 2 : 1;
    q.wc = wide(d->c) ? 2 : 1;
    q.ktiles = (d->k + 64 * q.wk - 1) / (64 * q.wk);
    q.ctiles = (d->c + 64 * q.wc - 1) / (64 * q.wc);
    q.M = (uint32_t)((size_t)d->n * O * P * Q);
    const uint32_t tiles = (uint32_t)q.ktiles * q.ctiles * taps;
    q.sp = (taps > 1 || tiles >= 16) ? 64 : 128;         // the stage-size rule of the rank-2 layers
    const char *fsp = env_switch(SW_WGG_SP);              // tests / benchmarks only
    if (fsp && (atoi(fsp) == 64 || atoi(fsp) == 128)) q.sp = atoi(fsp);
    // The kernel keeps the workgroups of a position chunk on one XCD (chunk % 8): chunks come in multiples of 8.
    // Per XCD m chunks x (tile, tap) sets share its workgroup slots (32 compute units x 1 or 2): of the m that
    // fit one round or leave a chunk at least 4096 positions, take the one that fills whole rounds of slots best (a single round
    // at 84 % leaves compute units with one workgroup idle while others work off two: 3x3x3, 64 -> 128 at
    // 16x56x56, 27 sets: 2 chunks per XCD 330 us, 7 chunks 294 us; with chunks of 900 positions 128 -> 256 at
    // 8x28x28 loses 30 %).
    const uint32_t xcd_slots = (q.sp == 64 ? 2 : 1) * NUM_CUS3 / 8;
    uint32_t best_m = 1;
    double best_fill = 0.0;
    const uint32_t one_round = xcd_slots / tiles > 0 ? xcd_slots / tiles : 1;      // always allowed: what one round holds
    for (uint32_t m = 1; m <= 16 && (m <= one_round || q.M / (8 * m) >= 4096); ++m) {
        const uint32_t wgs = m * tiles, rounds = (wgs + xcd_slots - 1) / xcd_slots;
        const double fill = (double)wgs / (rounds * xcd_slots);
        if (fill > best_fill + 0.02) { best_fill = fill; best_m = m; }
    }
    uint32_t parts = 8 * best_m;
    const char *fp = env_switch(SW_WGG3_PARTS);            // tests / benchmarks only
    if (fp && atoi(fp) >= 1 && atoi(fp) <= 4096) parts = (uint32_t)atoi(fp);
    const uint32_t max_parts = (q.M + 127) / 128;
    if (parts > max_parts) parts = max_parts;
    if (parts < 1) parts = 1;
    uint32_t chunk = (q.M + parts - 1) / parts;
    chunk = (chunk + 127) / 128 * 128;
    q.chunk = chunk;
    q.nparts = (int)((q.M + chunk - 1) / chunk);
    q.x_bytes = (uint32_t)x_bytes;
    q.dy_bytes = (uint32_t)dy_bytes;
    q.div_opq = make_fastdiv((uint32_t)(O * P * Q));
    q.div_pq = make_fastdiv((uint32_t)(P * Q));
    q.div_q = make_fastdiv((uint32_t)Q);
    if (wp) *wp = q;
    return true;
}

Variant3 pick3(const ngc_conv3d_desc *d, int op, ngc_conv_desc *r2)
{
    int O, P, Q;
    if (validate3(d, &O, &P, &Q) != NGC_OK) return V3_INVALID;
    if (op != NGC_OP_FWD && op != NGC_OP_BWD_DATA && op != NGC_OP_BWD_FILTERS) return V3_INVALID;
    ngc_conv_desc t;
    if (as_rank2(d, &t)) {
        if (r2) *r2 = t;
        return V3_RANK2;
    }
    const int taps = d->t * d->r * d->s;
    const bool direct_ok = d->w_layout == NGC_KCRS;
    if ((op == NGC_OP_FWD || op == NGC_OP_BWD_DATA) && strip3_plan(d, op, O, P, Q, nullptr)) return V3_STRIP;
    if (op == NGC_OP_FWD) {
        const bool wl = d->w_layout == NGC_KCRS || d->w_layout == NGC_BLOCKED_FWD;
        if (blocked_bf16_3(d) && wl && d->c % 32 == 0 && d->k % 64 == 0 && taps <= IGEMM_MAX_TAPS)
            return d->k % 128 == 0 ? V3_IGEMM_128 : V3_IGEMM_64;
        return direct_ok ? V3_DIRECT : V3_UNSUPPORTED;
    }
    if (op == NGC_OP_BWD_DATA) {
        const bool wl = d->w_layout == NGC_KCRS || d->w_layout == NGC_BLOCKED_BWD;
        if (blocked_bf16_3(d) && wl && d->k % 32 == 0 && d->c % 64 == 0 && taps <= IGEMM_MAX_TAPS &&
            d->stride_d * d->stride_h * d->stride_w <= IGEMM_MAX_CLASSES)
            return d->c % 128 == 0 ? V3_IGEMM_128 : V3_IGEMM_64;
        return direct_ok ? V3_DIRECT : V3_UNSUPPORTED;
    }
    if (wgrad_gemm3_plan(d, O, P, Q, nullptr)) return V3_WGRAD_GEMM;
    return V3_DIRECT;
}

size_t filter_elems3(const ngc_conv3d_desc *d, int layout)
{
    const size_t taps = (size_t)d->t * d->r * d->s;
    if (layout == NGC_KCRS) return (size_t)d->k * d->c * taps;
    if (layout == NGC_BLOCKED_FWD) return taps * ((d->c + 15) / 16) * d->k * 16;
    if (layout == NGC_BLOCKED_BWD) return taps * ((d->k + 15) / 16) * d->c * 16;
    return 0;
}

size_t workspace3(const ngc_conv3d_desc *d, int op, Variant3 v, const ngc_conv_desc *r2, int O, int P, int Q)
{
    if (v == V3_RANK2) return ngc_conv_workspace_bytes(r2, op);
    if (v == V3_IGEMM_128 || v == V3_IGEMM_64 || v == V3_STRIP) {
        if (d->w_layout != NGC_KCRS) return 0;
        return round256_3(filter_elems3(d, op == NGC_OP_FWD ? NGC_BLOCKED_FWD : NGC_BLOCKED_BWD) * 2);
    }
    if (v == V3_WGRAD_GEMM) {
        WgradGemmParams wp;
        if (!wgrad_gemm3_plan(d, O, P, Q, &wp)) return 0;
        return round256_3((size_t)wp.nparts * d->t * d->r * d->s * wp.ktiles * wp.ctiles * wp.wk * wp.wc * 64 * 64 * sizeof(float));
    }
    return 0;
}

// dx seen as a gradient tensor of [N, C, D*H, W]: its channel sums are a rank-2 bias gradient
ngc_conv_desc dx_as_dy3(const ngc_conv3d_desc *d)
{
    ngc_conv_desc t;
    memset(&t, 0, sizeof(t));
    t.n = d->n; t.c = 1; t.h = d->d * d->h; t.w = d->w; t.k = d->c; t.r = t.s = 1;
    t.stride_h = t.stride_w = t.dil_h = t.dil_w = 1;
    t.dtype = d->dtype; t.x_layout = d->x_layout; t.y_layout = d->x_layout;
    return t;
}

size_t db3_partial_bytes(const ngc_conv3d_desc *d)
{
    const ngc_conv_desc t = dx_as_dy3(d);
    return round256_3((size_t)bias_grad_parts(t, t.h, t.w) * ((d->c + 15) / 16 * 16) * sizeof(float));
}

void fill_class3(IgemmClass &c, int oa_d, int oa_h, int oa_w, int OD, int OP, int OQ, int tap_begin, int tap_count, int N)
{
    c.oa_d = oa_d; c.oa_h = oa_h; c.oa_w = oa_w;
    c.OD = OD; c.OP = OP; c.OQ = OQ;
    c.tap_begin = tap_begin;
    c.tap_count = tap_count;
    const bool empty = OD <= 0 || OP <= 0 || OQ <= 0;
    c.M = empty ? 0u : (uint32_t)((size_t)N * OD * OP * OQ);
    c.div_opq = make_fastdiv(empty ? 1u : (uint32_t)(OD * OP * OQ));
    c.div_pq = make_fastdiv(empty ? 1u : (uint32_t)(OP * OQ));
    c.div_q = make_fastdiv(empty ? 1u : (uint32_t)OQ);
}

}  // namespace

extern "C" {

int ngc_conv3d_out_shape(const ngc_conv3d_desc *desc, int32_t *o, int32_t *p, int32_t *q)
{
    if (!desc || !o || !p || !q) return NGC_BAD_ARG;
    int O, P, Q;
    const int vs = validate3(desc, &O, &P, &Q);
    if (vs != NGC_OK) return vs;
    *o = O; *p = P; *q = Q;
    return NGC_OK;
}

size_t ngc_conv3d_workspace_bytes(const ngc_conv3d_desc *desc, int op)
{
    int O, P, Q;
    if (validate3(desc, &O, &P, &Q) != NGC_OK) return 0;
    if (op == NGC_OP_BIAS_GRAD) {
        ngc_conv_desc t;
        memset(&t, 0, sizeof(t));
        t.n = desc->n; t.k = desc->k; t.dtype = desc->dtype; t.y_layout = desc->y_layout;
        return round256_3((size_t)bias_grad_parts(t, O * P, Q) * ((desc->k + 15) / 16 * 16) * sizeof(float));
    }
    if (op == NGC_OP_BWD_DATA_DB) {
        ngc_conv_desc r2t;
        const Variant3 vb = pick3(desc, NGC_OP_BWD_DATA, &r2t);
        if (vb == V3_INVALID || vb == V3_UNSUPPORTED) return 0;
        return ngc_conv3d_workspace_bytes(desc, NGC_OP_BWD_DATA) + db3_partial_bytes(desc);
    }
    const BatchSlices3 bs = batch_slices3(desc, O, P, Q);
    if (bs.images < desc->n && (op == NGC_OP_FWD || op == NGC_OP_BWD_DATA || op == NGC_OP_BWD_FILTERS)) {
        // groups of images reuse one workspace; backprop-filters keeps one dw per group behind it
        const ngc_conv3d_desc g = with_batch3(desc, bs.images);
        const size_t base = ngc_conv3d_workspace_bytes(&g, op);
        if (op != NGC_OP_BWD_FILTERS) return base;
        const size_t groups = (size_t)(desc->n + bs.images - 1) / bs.images;
        const size_t row = ((size_t)desc->k * desc->c * desc->t * desc->r * desc->s + 15) / 16 * 16;
        return round256_3(base) + round256_3(groups * row * sizeof(float));
    }
    ngc_conv_desc r2;
    const Variant3 v = pick3(desc, op, &r2);
    if (v == V3_INVALID || v == V3_UNSUPPORTED) return 0;
    return workspace3(desc, op, v, &r2, O, P, Q);
}

size_t ngc_conv3d_filter_elems(const ngc_conv3d_desc *desc, int32_t layout)
{
    int O, P, Q;
    if (validate3(desc, &O, &P, &Q) != NGC_OK) return 0;
    return filter_elems3(desc, layout);
}

size_t ngc_conv3d_data_elems(const ngc_conv3d_desc *desc, int which)
{
    int O, P, Q;
    if (validate3(desc, &O, &P, &Q) != NGC_OK) return 0;
    if (which == 0) return phys3(desc->x_layout, desc->n, desc->c, desc->d, desc->h, desc->w);
    if (which == 1) return phys3(desc->y_layout, desc->n, desc->k, O, P, Q);
    return 0;
}

int ngc_conv3d_filter_convert(const ngc_conv3d_desc *desc, const void *w_kctrs, void *w_blocked, int32_t dst_layout,
                              void *hip_stream)
{
    int O, P, Q;
    const int vs = validate3(desc, &O, &P, &Q);
    if (vs != NGC_OK) return vs;
    if (!w_kctrs || !w_blocked || (dst_layout != NGC_BLOCKED_FWD && dst_layout != NGC_BLOCKED_BWD)) return NGC_BAD_ARG;
    if (!aligned16_3(w_kctrs) || !aligned16_3(w_blocked)) return NGC_BAD_ARG;
    // the blocked layouts keep the taps outermost in (t, r, s) order: the rank-2 re-layout with T*R rows of S taps
    return status3(launch_filter_convert(desc->dtype == NGC_BF16 ? 2 : 4, desc->k, desc->c, desc->t * desc->r, desc->s, w_kctrs,
                                         w_blocked, dst_layout, static_cast<hipStream_t>(hip_stream)));
}

const char *ngc_conv3d_variant(const ngc_conv3d_desc *desc, int op)
{
    static thread_local char name[96];
    ngc_conv_desc r2;
    {
        int O, P, Q;
        if (validate3(desc, &O, &P, &Q) == NGC_OK && (op == NGC_OP_FWD || op == NGC_OP_BWD_DATA || op == NGC_OP_BWD_FILTERS)) {
            const BatchSlices3 bs = batch_slices3(desc, O, P, Q);
            if (bs.images < desc->n) {                       // groups of images: the kernel of a group
                static thread_local char sliced[112];
                const ngc_conv3d_desc g = with_batch3(desc, bs.images);
                snprintf(sliced, sizeof(sliced), "sliced:%s", ngc_conv3d_variant(&g, op));
                return sliced;
            }
        }
    }
    switch (pick3(desc, op, &r2)) {
    case V3_RANK2: snprintf(name, sizeof(name), "rank2:%s", ngc_conv_variant(&r2, op)); return name;
    case V3_STRIP: return "strip3_bf16";
    case V3_IGEMM_128: return "igemm3_bf16_128x128";
    case V3_IGEMM_64: return "igemm3_bf16_256x64";
    case V3_WGRAD_GEMM: return "wgrad_gemm3_bf16";
    case V3_DIRECT: return "direct3";
    case V3_UNSUPPORTED: return "unsupported";
    default: return "invalid";
    }
}

int ngc_conv3d_fwd(const ngc_conv3d_desc *desc, const void *x, const void *w, const float *bias, void *y, void *ws,
                   size_t ws_bytes, void *hip_stream)
{
    int O, P, Q;
    const int vs = validate3(desc, &O, &P, &Q);
    if (vs != NGC_OK) return vs;
    if (!x || !w || !y) return NGC_BAD_ARG;
    if ((desc->epilogue & NGC_EPI_BIAS) && !bias) return NGC_BAD_ARG;
    if (!aligned16_3(x) || !aligned16_3(w) || !aligned16_3(y) || !aligned16_3(ws) || !aligned16_3(bias)) return NGC_BAD_ARG;
    const BatchSlices3 bs = batch_slices3(desc, O, P, Q);
    if (bs.images < desc->n) {                                // operands of 2 GiB or more: one launch per group of images
        for (int n0 = 0; n0 < desc->n; n0 += bs.images) {
            const ngc_conv3d_desc g = with_batch3(desc, desc->n - n0 < bs.images ? desc->n - n0 : bs.images);
            const int rc = ngc_conv3d_fwd(&g, static_cast<const unsigned char *>(x) + (size_t)n0 * bs.x_bytes, w, bias,
                                          static_cast<unsigned char *>(y) + (size_t)n0 * bs.y_bytes, ws, ws_bytes, hip_stream);
            if (rc != NGC_OK) return rc;
        }
        return NGC_OK;
    }
    ngc_conv_desc r2;
    const Variant3 v = pick3(desc, NGC_OP_FWD, &r2);
    if (v == V3_RANK2) return ngc_conv_fwd(&r2, x, w, bias, y, ws, ws_bytes, hip_stream);
    if (v == V3_UNSUPPORTED) return NGC_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const float *b = (desc->epilogue & NGC_EPI_BIAS) ? bias : nullptr;
    if (v == V3_DIRECT) return status3(launch_direct3_fwd(*desc, O, P, Q, x, w, b, y, st));

    const size_t need = workspace3(desc, NGC_OP_FWD, v, nullptr, O, P, Q);
    if (need > 0 && (!ws || ws_bytes < need)) return NGC_WORKSPACE_TOO_SMALL;
    const void *wt = w;
    if (desc->w_layout == NGC_KCRS) {
        const hipError_t e = launch_filter_convert(2, desc->k, desc->c, desc->t * desc->r, desc->s, w, ws, NGC_BLOCKED_FWD, st);
        if (e != hipSuccess) return status3(e);
        wt = ws;
    }
    if (v == V3_STRIP) {
        Strip3Plan pl;
        if (!strip3_plan(desc, NGC_OP_FWD, O, P, Q, &pl) || pl.n != 1) return NGC_UNSUPPORTED;
        StripParams &sp = pl.l[0].sp;
        sp.in = static_cast<const uint16_t *>(x);
        sp.wt = static_cast<const uint16_t *>(wt);
        sp.out = static_cast<uint16_t *>(y);
        sp.bias = b;
        sp.relu = (desc->epilogue & NGC_EPI_RELU) ? 1 : 0;
        return status3(launch_strip(sp, pl.l[0].nf, pl.l[0].lds, st));
    }
    IgemmParams p;
    memset(&p, 0, sizeof(p));
    p.in = static_cast<const uint16_t *>(x);
    p.wt = static_cast<const uint16_t *>(wt);
    p.out = static_cast<uint16_t *>(y);
    p.bias = b;
    p.N = desc->n; p.Cin = desc->c; p.Din = desc->d; p.Hin = desc->h; p.Win = desc->w;
    p.Cout = desc->k; p.Dout = O; p.Hout = P; p.Wout = Q;
    p.os_d = p.os_h = p.os_w = 1;
    p.is_d = desc->stride_d; p.is_h = desc->stride_h; p.is_w = desc->stride_w;
    p.relu = (desc->epilogue & NGC_EPI_RELU) ? 1 : 0;
    p.ncls = 1;
    int n = 0;
    for (int t = 0; t < desc->t; ++t)
        for (int r = 0; r < desc->r; ++r)
            for (int s = 0; s < desc->s; ++s) {
                p.taps[n].dd = t * desc->dil_d - desc->pad_below_d;
                p.taps[n].dh = r * desc->dil_h - desc->pad_below_h;
                p.taps[n].dw = s * desc->dil_w - desc->pad_below_w;
                p.taps[n].slab = n;
                ++n;
            }
    fill_class3(p.cls[0], 0, 0, 0, O, P, Q, 0, n, desc->n);
    return status3(launch_igemm3(p, v == V3_IGEMM_128 ? 128 : 64, p.cls[0].M, st));
}

}  // extern "C"

namespace {

// ConvolutionBackpropData; mask (may be null): same shape / layout / type as dx, dx = (mask > 0) ? dx : 0
int bwd_data3_core(const ngc_conv3d_desc *desc, const void *dy, const void *w, const void *mask, void *dx, void *ws,
                   size_t ws_bytes, void *hip_stream)
{
    int O, P, Q;
    const int vs = validate3(desc, &O, &P, &Q);
    if (vs != NGC_OK) return vs;
    if (!dy || !w || !dx) return NGC_BAD_ARG;
    if (!aligned16_3(dy) || !aligned16_3(w) || !aligned16_3(dx) || !aligned16_3(ws) || !aligned16_3(mask)) return NGC_BAD_ARG;
    const BatchSlices3 bs = batch_slices3(desc, O, P, Q);
    if (bs.images < desc->n) {                                // operands of 2 GiB or more: one launch per group of images
        for (int n0 = 0; n0 < desc->n; n0 += bs.images) {
            const ngc_conv3d_desc g = with_batch3(desc, desc->n - n0 < bs.images ? desc->n - n0 : bs.images);
            const size_t xo = (size_t)n0 * bs.x_bytes, yo = (size_t)n0 * bs.y_bytes;
            const int rc = bwd_data3_core(&g, static_cast<const unsigned char *>(dy) + yo, w,
                                          mask ? static_cast<const unsigned char *>(mask) + xo : nullptr,
                                          static_cast<unsigned char *>(dx) + xo, ws, ws_bytes, hip_stream);
            if (rc != NGC_OK) return rc;
        }
        return NGC_OK;
    }
    ngc_conv_desc r2;
    const Variant3 v = pick3(desc, NGC_OP_BWD_DATA, &r2);
    if (v == V3_RANK2)
        return mask ? ngc_conv_bwd_data_relu(&r2, dy, w, mask, dx, ws, ws_bytes, hip_stream)
                    : ngc_conv_bwd_data(&r2, dy, w, dx, ws, ws_bytes, hip_stream);
    if (v == V3_UNSUPPORTED) return NGC_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (v == V3_DIRECT) return status3(launch_direct3_bwd_data(*desc, O, P, Q, dy, w, mask, dx, st));

    const size_t need = workspace3(desc, NGC_OP_BWD_DATA, v, nullptr, O, P, Q);
    if (need > 0 && (!ws || ws_bytes < need)) return NGC_WORKSPACE_TOO_SMALL;
    const void *wt = w;
    if (desc->w_layout == NGC_KCRS) {
        const hipError_t e = launch_filter_convert(2, desc->k, desc->c, desc->t * desc->r, desc->s, w, ws, NGC_BLOCKED_BWD, st);
        if (e != hipSuccess) return status3(e);
        wt = ws;
    }
    if (v == V3_STRIP) {
        Strip3Plan pl;
        if (!strip3_plan(desc, NGC_OP_BWD_DATA, O, P, Q, &pl)) return NGC_UNSUPPORTED;
        if (pl.zero) {
            const hipError_t e = launch_zero_fill(dx, (size_t)desc->n * desc->c * desc->d * desc->h * desc->w * 2, st);
            if (e != hipSuccess) return status3(e);
        }
        // the classes share grids, up to STRIP_MULTI_MAX launches each (launches with column tiles go alone)
        bool col_tiles = false;
        for (int i = 0; i < pl.n; ++i) col_tiles = col_tiles || pl.l[i].sp.ncolt > 1;
        const int per_grid = col_tiles ? 1 : STRIP_MULTI_MAX;
        for (int first = 0; first < pl.n; first += per_grid) {
            const int cnt = pl.n - first < per_grid ? pl.n - first : per_grid;
            StripMulti mp;
            mp.n = cnt;
            int nf_max = 0;
            size_t lds_max = 0;
            for (int i = 0; i < cnt; ++i) {
                StripParams &sp = pl.l[first + i].sp;
                sp.in = static_cast<const uint16_t *>(dy);
                sp.wt = static_cast<const uint16_t *>(wt);
                sp.out = static_cast<uint16_t *>(dx);
                sp.mask = static_cast<const uint16_t *>(mask);
                mp.c[i] = sp;
                mp.wg_end[i] = (i ? mp.wg_end[i - 1] : 0) + sp.groups * sp.strips;
                if (pl.l[first + i].nf > nf_max) nf_max = pl.l[first + i].nf;
                if (pl.l[first + i].lds > lds_max) lds_max = pl.l[first + i].lds;
            }
            const hipError_t e = cnt == 1 ? launch_strip(mp.c[0], nf_max, lds_max, st) : launch_strip_multi(mp, nf_max, lds_max, st);
            if (e != hipSuccess) return status3(e);
        }
        return NGC_OK;
    }
    IgemmParams p;
    memset(&p, 0, sizeof(p));
    p.in = static_cast<const uint16_t *>(dy);
    p.wt = static_cast<const uint16_t *>(wt);
    p.out = static_cast<uint16_t *>(dx);
    p.mask = static_cast<const uint16_t *>(mask);
    p.N = desc->n; p.Cin = desc->k; p.Din = O; p.Hin = P; p.Win = Q;
    p.Cout = desc->c; p.Dout = desc->d; p.Hout = desc->h; p.Wout = desc->w;
    const int sd = desc->stride_d, sh = desc->stride_h, sw = desc->stride_w;
    p.os_d = sd; p.os_h = sh; p.os_w = sw;
    p.is_d = p.is_h = p.is_w = 1;
    p.ncls = sd * sh * sw;
    // One class per residue (a, b, c) of the dx voxel modulo the strides: its taps are those with
    // (a + pad_below - t dil) divisible by the stride on every axis, and the quotient is the offset into dy.
    // A class without taps still runs and writes the zeros no window reaches.
    int n = 0;
    uint32_t max_m = 0;
    auto lattice = [](int extent, int a, int stride) { return a < extent ? (extent - a + stride - 1) / stride : 0; };
    auto hits = [](int v, int stride) { return ((v % stride) + stride) % stride == 0; };
    for (int a = 0; a < sd; ++a)
        for (int b = 0; b < sh; ++b)
            for (int c = 0; c < sw; ++c) {
                const int begin = n;
                for (int t = 0; t < desc->t; ++t) {
                    const int vd = a + desc->pad_below_d - t * desc->dil_d;
                    if (!hits(vd, sd)) continue;
                    for (int r = 0; r < desc->r; ++r) {
                        const int vh = b + desc->pad_below_h - r * desc->dil_h;
                        if (!hits(vh, sh)) continue;
                        for (int s = 0; s < desc->s; ++s) {
                            const int vw = c + desc->pad_below_w - s * desc->dil_w;
                            if (!hits(vw, sw)) continue;
                            p.taps[n].dd = vd / sd;              // exact
                            p.taps[n].dh = vh / sh;
                            p.taps[n].dw = vw / sw;
                            p.taps[n].slab = (t * desc->r + r) * desc->s + s;
                            ++n;
                        }
                    }
                }
                IgemmClass &cl = p.cls[(a * sh + b) * sw + c];
                fill_class3(cl, a, b, c, lattice(desc->d, a, sd), lattice(desc->h, b, sh), lattice(desc->w, c, sw), begin,
                            n - begin, desc->n);
                if (cl.M > max_m) max_m = cl.M;
            }
    return status3(launch_igemm3(p, v == V3_IGEMM_128 ? 128 : 64, max_m, st));
}

// db (may be null): [C] fp32 channel sums of the dx written, from a second pass over dx whose partials sit
// in the workspace behind the backprop-data part
int bwd_data3_impl(const ngc_conv3d_desc *desc, const void *dy, const void *w, const void *mask, void *dx, float *db, void *ws,
                   size_t ws_bytes, void *hip_stream)
{
    if (!db) return bwd_data3_core(desc, dy, w, mask, dx, ws, ws_bytes, hip_stream);
    int O, P, Q;
    const int vs = validate3(desc, &O, &P, &Q);
    if (vs != NGC_OK) return vs;
    if (!aligned16_3(db) || !aligned16_3(ws)) return NGC_BAD_ARG;
    if ((size_t)desc->n * desc->d * desc->h * desc->w >= 0xFFFF0000ull) return NGC_BAD_SHAPE;
    const size_t base = ngc_conv3d_workspace_bytes(desc, NGC_OP_BWD_DATA);
    const size_t need = base + db3_partial_bytes(desc);
    if (!ws || ws_bytes < need) return NGC_WORKSPACE_TOO_SMALL;
    const int rc = bwd_data3_core(desc, dy, w, mask, dx, ws, base, hip_stream);
    if (rc != NGC_OK) return rc;
    const ngc_conv_desc t = dx_as_dy3(desc);
    float *partial = reinterpret_cast<float *>(static_cast<unsigned char *>(ws) + base);
    return status3(launch_bias_grad(t, t.h, t.w, dx, db, partial, bias_grad_parts(t, t.h, t.w), static_cast<hipStream_t>(hip_stream)));
}

}  // namespace

extern "C" {

int ngc_conv3d_bwd_data(const ngc_conv3d_desc *desc, const void *dy, const void *w, void *dx, void *ws, size_t ws_bytes,
                        void *hip_stream)
{
    return bwd_data3_impl(desc, dy, w, nullptr, dx, nullptr, ws, ws_bytes, hip_stream);
}

int ngc_conv3d_bwd_data_relu(const ngc_conv3d_desc *desc, const void *dy, const void *w, const void *x_in, void *dx, void *ws,
                             size_t ws_bytes, void *hip_stream)
{
    if (!x_in) return NGC_BAD_ARG;
    return bwd_data3_impl(desc, dy, w, x_in, dx, nullptr, ws, ws_bytes, hip_stream);
}

int ngc_conv3d_bwd_data_relu_db(const ngc_conv3d_desc *desc, const void *dy, const void *w, const void *x_in, void *dx, float *db,
                                void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!x_in || !db) return NGC_BAD_ARG;
    return bwd_data3_impl(desc, dy, w, x_in, dx, db, ws, ws_bytes, hip_stream);
}

int ngc_conv3d_bias_grad(const ngc_conv3d_desc *desc, const void *dy, float *db, void *ws, size_t ws_bytes, void *hip_stream)
{
    int O, P, Q;
    const int vs = validate3(desc, &O, &P, &Q);
    if (vs != NGC_OK) return vs;
    if (!dy || !db || !ws) return dy && db ? NGC_WORKSPACE_TOO_SMALL : NGC_BAD_ARG;
    if (!aligned16_3(dy) || !aligned16_3(db) || !aligned16_3(ws)) return NGC_BAD_ARG;
    if ((size_t)desc->n * O * P * Q >= 0xFFFF0000ull) return NGC_BAD_SHAPE;
    if (ws_bytes < ngc_conv3d_workspace_bytes(desc, NGC_OP_BIAS_GRAD)) return NGC_WORKSPACE_TOO_SMALL;
    // dy [N, K, O, P, Q] keeps (o, p, q) contiguous in both layouts: the rank-2 reduction over [N, K, O*P, Q]
    ngc_conv_desc t;
    memset(&t, 0, sizeof(t));
    t.n = desc->n; t.k = desc->k; t.dtype = desc->dtype; t.y_layout = desc->y_layout;
    return status3(launch_bias_grad(t, O * P, Q, dy, db, static_cast<float *>(ws), bias_grad_parts(t, O * P, Q),
                                    static_cast<hipStream_t>(hip_stream)));
}

int ngc_conv3d_bwd_filters(const ngc_conv3d_desc *desc, const void *x, const void *dy, float *dw, void *ws, size_t ws_bytes,
                           void *hip_stream)
{
    int O, P, Q;
    const int vs = validate3(desc, &O, &P, &Q);
    if (vs != NGC_OK) return vs;
    if (!x || !dy || !dw) return NGC_BAD_ARG;
    if (!aligned16_3(x) || !aligned16_3(dy) || !aligned16_3(dw) || !aligned16_3(ws)) return NGC_BAD_ARG;
    const BatchSlices3 bs = batch_slices3(desc, O, P, Q);
    if (bs.images < desc->n) {
        // operands of 2 GiB or more: dw of each group of images into the workspace, then their sum in index order
        const ngc_conv3d_desc g0 = with_batch3(desc, bs.images);
        const size_t base = round256_3(ngc_conv3d_workspace_bytes(&g0, NGC_OP_BWD_FILTERS));
        if (!ws || ws_bytes < ngc_conv3d_workspace_bytes(desc, NGC_OP_BWD_FILTERS)) return NGC_WORKSPACE_TOO_SMALL;
        const int elems = desc->k * desc->c * desc->t * desc->r * desc->s, row = (elems + 15) / 16 * 16;
        float *rows = reinterpret_cast<float *>(static_cast<unsigned char *>(ws) + base);
        int groups = 0;
        for (int n0 = 0; n0 < desc->n; n0 += bs.images, ++groups) {
            const ngc_conv3d_desc g = with_batch3(desc, desc->n - n0 < bs.images ? desc->n - n0 : bs.images);
            const int rc = ngc_conv3d_bwd_filters(&g, static_cast<const unsigned char *>(x) + (size_t)n0 * bs.x_bytes,
                                                  static_cast<const unsigned char *>(dy) + (size_t)n0 * bs.y_bytes,
                                                  rows + (size_t)groups * row, ws, base, hip_stream);
            if (rc != NGC_OK) return rc;
        }
        return status3(launch_bias_grad_reduce(rows, dw, groups, elems, row, static_cast<hipStream_t>(hip_stream)));
    }
    ngc_conv_desc r2;
    const Variant3 v = pick3(desc, NGC_OP_BWD_FILTERS, &r2);
    if (v == V3_RANK2) return ngc_conv_bwd_filters(&r2, x, dy, dw, ws, ws_bytes, hip_stream);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (v == V3_DIRECT) return status3(launch_direct3_bwd_filters(*desc, O, P, Q, x, dy, dw, st));
    if (v != V3_WGRAD_GEMM) return NGC_UNSUPPORTED;
    WgradGemmParams wp;
    if (!wgrad_gemm3_plan(desc, O, P, Q, &wp)) return NGC_UNSUPPORTED;
    const size_t need = workspace3(desc, NGC_OP_BWD_FILTERS, v, nullptr, O, P, Q);
    if (!ws || ws_bytes < need) return NGC_WORKSPACE_TOO_SMALL;
    wp.x = static_cast<const uint16_t *>(x);
    wp.dy = static_cast<const uint16_t *>(dy);
    wp.partial = static_cast<float *>(ws);
    wp.dw = dw;
    return status3(launch_wgrad_gemm(wp, st));
}

}  // extern "C"
