// C ABI of libngconv: argument validation, shape inference, kernel selection, launches.
// Host code only.  Kernel selection is the small analogue of what the paper's Sec. 4 gives the
// backend transformer to do (layout and shape decisions taken together with the choice of a
// backend kernel): the descriptor (shape, attributes, element type, layouts) picks a hand-written
// kernel variant; a descriptor without a kernel is reported as NGC_UNSUPPORTED, never routed to
// a CPU path.
#include "common.h"

#include <limits.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <unordered_map>

using namespace ngc;

namespace {

// ---- plan cache -------------------------------------------------------------------------------------------
// Planning a launch (kernel selection, strip / tile geometry, split of a reduction) is a pure function of the
// descriptor, a few integers and the environment switches.  Each planning function below keeps what it
// computed per thread, keyed by its arguments, so that the second call with a descriptor costs a few table
// look-ups instead of the geometry loops; ngc_reload_switches() invalidates everything.
struct PlanKey {
    ngc_conv_desc d;
    int32_t a[4];
};
static_assert(sizeof(PlanKey) == 24 * sizeof(int32_t), "hashed and compared as 24 words, no padding");

struct PlanKeyHash {
    size_t operator()(const PlanKey &k) const
    {
        const uint32_t *w = reinterpret_cast<const uint32_t *>(&k);
        uint64_t h = 0xcbf29ce484222325ull;
        for (int i = 0; i < 24; ++i) h = (h ^ w[i]) * 0x100000001b3ull;
        return (size_t)(h ^ (h >> 29));
    }
};
struct PlanKeyEq {
    bool operator()(const PlanKey &x, const PlanKey &y) const { return memcmp(&x, &y, sizeof(PlanKey)) == 0; }
};

PlanKey plan_key(const ngc_conv_desc *d, int a0 = 0, int a1 = 0, int a2 = 0, int a3 = 0)
{
    PlanKey k;
    k.d = *d;
    k.a[0] = a0; k.a[1] = a1; k.a[2] = a2; k.a[3] = a3;
    return k;
}

template <class V>
struct PlanCache {
    std::unordered_map<PlanKey, V, PlanKeyHash, PlanKeyEq> map;
    uint32_t epoch = 0xFFFFFFFFu;
    V *find(const PlanKey &k)
    {
        if (epoch != sw_epoch()) {
            map.clear();
            epoch = sw_epoch();
        }
        auto it = map.find(k);
        return it == map.end() ? nullptr : &it->second;
    }
    V &put(const PlanKey &k, const V &v)
    {
        if (map.size() >= 2048) map.clear();             // a process cycling through more nodes than that replans
        return map[k] = v;
    }
};

constexpr size_t MAX_ELEMS = (size_t)1 << 31;

int out_dim(int in, int pb, int pa, int dil, int win, int stride)
{
    const long span = (long)in + pb + pa - (long)dil * (win - 1) - 1;
    if (span < 0) return 0;
    return (int)(span / stride) + 1;
}

bool layout_ok(int l) { return l == NGC_NCHW || l == NGC_NCHW16C; }

size_t phys(int layout, size_t n, size_t c, size_t h, size_t w)
{
    return layout == NGC_NCHW ? n * c * h * w : n * ((c + 15) / 16) * h * w * 16;
}

// Validates everything that does not depend on the op.  Fills P, Q.
int validate(const ngc_conv_desc *d, int *P, int *Q)
{
    if (!d) return NGC_BAD_ARG;
    if (d->dtype != NGC_F32 && d->dtype != NGC_BF16) return NGC_BAD_ARG;
    if (!layout_ok(d->x_layout) || !layout_ok(d->y_layout)) return NGC_BAD_ARG;
    if (d->w_layout != NGC_KCRS && d->w_layout != NGC_BLOCKED_FWD && d->w_layout != NGC_BLOCKED_BWD) return NGC_BAD_ARG;
    if (d->epilogue & ~(NGC_EPI_BIAS | NGC_EPI_RELU)) return NGC_BAD_ARG;
    if (d->n < 1 || d->c < 1 || d->h < 1 || d->w < 1 || d->k < 1 || d->r < 1 || d->s < 1) return NGC_BAD_SHAPE;
    if (d->stride_h < 1 || d->stride_w < 1 || d->dil_h < 1 || d->dil_w < 1) return NGC_BAD_SHAPE;
    if (d->pad_below_h < 0 || d->pad_below_w < 0 || d->pad_above_h < 0 || d->pad_above_w < 0) return NGC_BAD_SHAPE;
    // keep every intermediate index comfortably inside int32
    if (d->h > (1 << 20) || d->w > (1 << 20) || d->r > 1024 || d->s > 1024 || d->dil_h > 1024 || d->dil_w > 1024 ||
        d->stride_h > 1024 || d->stride_w > 1024 || d->pad_below_h > (1 << 20) || d->pad_below_w > (1 << 20) ||
        d->pad_above_h > (1 << 20) || d->pad_above_w > (1 << 20))
        return NGC_BAD_SHAPE;
    const int p = out_dim(d->h, d->pad_below_h, d->pad_above_h, d->dil_h, d->r, d->stride_h);
    const int q = out_dim(d->w, d->pad_below_w, d->pad_above_w, d->dil_w, d->s, d->stride_w);
    if (p < 1 || q < 1) return NGC_BAD_SHAPE;
    if (phys(d->x_layout, d->n, d->c, d->h, d->w) >= MAX_ELEMS) return NGC_BAD_SHAPE;
    if (phys(d->y_layout, d->n, d->k, p, q) >= MAX_ELEMS) return NGC_BAD_SHAPE;
    if ((size_t)((d->k + 15) / 16) * 16 * ((d->c + 15) / 16) * 16 * d->r * d->s >= MAX_ELEMS) return NGC_BAD_SHAPE;
    *P = p;
    *Q = q;
    return NGC_OK;
}

size_t round256(size_t b) { return (b + 255) & ~(size_t)255; }

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// Forward and backprop-data treat the images of a batch independently.  The MFMA kernels address an operand with
// 32-bit byte offsets, so a bf16 node with blocked tensors whose x or y has 2 GiB or more runs as several
// launches over groups of images that stay below.  Returns the images per group (d->n: one launch).
struct BatchSlices {
    int images;                // per group
    size_t x_bytes, y_bytes;   // of one image
};

BatchSlices batch_slices(const ngc_conv_desc *d, int P, int Q)
{
    BatchSlices b;
    b.images = d->n;
    b.x_bytes = phys(d->x_layout, 1, d->c, d->h, d->w) * 2;
    b.y_bytes = phys(d->y_layout, 1, d->k, P, Q) * 2;
    if (d->dtype != NGC_BF16 || d->x_layout != NGC_NCHW16C || d->y_layout != NGC_NCHW16C) return b;
    const size_t per = b.x_bytes > b.y_bytes ? b.x_bytes : b.y_bytes, lim = (size_t)1 << 31;
    if ((size_t)d->n * per < lim || per >= lim) return b;             // small enough, or one image alone is too large
    b.images = (int)((lim - 1) / per);
    return b;
}

ngc_conv_desc with_batch(const ngc_conv_desc *d, int n)
{
    ngc_conv_desc t = *d;
    t.n = n;
    return t;
}

enum Variant { V_INVALID, V_UNSUPPORTED, V_DIRECT, V_IGEMM_128, V_IGEMM_64, V_WGRAD_64, V_STRIP, V_WGRAD_STRIP, V_STEM_FWD, V_WGRAD_STEM, V_STEM_BWD, V_WGRAD_GEMM, V_GEMM1X1, V_ROWS, V_STAGED };

constexpr int NUM_CUS = 256;                      // MI355X
constexpr size_t LDS_LIMIT = 160 * 1024;

// Tiling of the output-stationary strip kernel: picks the strip size (nf = 32-position fragments
// per SIMD) and fills the geometry fields of `out` for a lattice of N x Hout x Wout positions whose
// taps span span_h x span_w input pixels beyond the position's own pixel (position stride out.sh,
// out.sw in input pixels).  Returns false if nothing fits.
bool strip_geometry(StripParams &out, int N, int Hout, int Wout, int span_h, int span_w, int ntaps, int Cout,
                    int *nf_out, size_t *lds_out)
{
    // NGC_STRIP_NF (tests / benchmarks only): 0 disables this kernel, 7 / 4 / 2 forces a strip size
    const char *force = env_switch(SW_STRIP_NF);
    const int forced_nf = force ? atoi(force) : -1;
    if (forced_nf == 0) return false;
    constexpr int MAXPATCH = 24 * 64;                                    // patch pixels per plane (24 blocks of 64)
    const int sh = out.sh, sw = out.sw;
    StripParams best;
    int best_nf = 0;
    size_t best_lds = 0;
    const int nfs[3] = {7, 4, 2};
    for (int nf : nfs) {
        if (forced_nf > 0 && nf != forced_nf) continue;
        const int maxpix = 4 * nf * 32;
        StripParams q = out;
        q.ncolt = 1;
        q.BW = Wout;
        q.PC = (Wout - 1) * sw + span_w + 1;
        const int pr_full = (Hout - 1) * sh + span_h + 1;
        if (Wout > maxpix || MAXPATCH / q.PC < span_h + 1) {
            // Rows wider than a strip (or its patch) holds: column tiles.  Of the tile widths (multiples of 8 lattice
            // columns) take the one whose strips read the fewest patch pixels over the image.
            if (out.out_mode != 0) continue;
            // Among equal costs: the widest tile (longer contiguous runs per patch row), but for a node below half the
            // machine balance in flop per tensor byte the widest whose strip fits the smallest kernel variant (256
            // positions) - such a node wants many workgroups in flight, not large ones (3x1 window, 128 -> 64
            // channels, rows of 3136 pixels: tiles of 8 / 16 / 32 / 56 columns cost the same patch traffic and run
            // forward in 42 / 37 / 36 / 37 us, backprop-data in 49 / 37 / 38 / 43 us).
            long best_cost = -1;
            int best_bw = 0, best_tp = 0;
            const bool mem_bound = (double)out.Cin * ntaps * Cout / (out.Cin + Cout) < 157.0;
            auto rank = [&](int bw, int tp) { return mem_bound && bw * tp > 256 ? -bw : bw; };
            const char *fbw = env_switch(SW_STRIP_BW);                    // tests / benchmarks only: tile width
            for (int bw = 8; bw <= maxpix && bw < Wout + 8; bw += 8) {
                if (fbw && atoi(fbw) >= 8 && bw != atoi(fbw)) continue;
                const int pc = (bw - 1) * sw + span_w + 1;
                int tp = maxpix / bw;
                const int prows = MAXPATCH / pc;
                if (prows < span_h + 1) break;
                const int rows_patch = (prows - span_h - 1) / sh + 1;
                if (tp > rows_patch) tp = rows_patch;
                if (tp > Hout) tp = Hout;
                if (tp < 1) continue;
                const long tiles = (long)((Hout + tp - 1) / tp) * ((Wout + bw - 1) / bw);
                const long cost = tiles * ((long)(tp - 1) * sh + span_h + 1) * pc;
                if (best_cost < 0 || cost < best_cost || (cost == best_cost && rank(bw, tp) > rank(best_bw, best_tp))) {
                    best_cost = cost; best_bw = bw; best_tp = tp;
                }
            }
            if (best_cost < 0) continue;
            q.BW = best_bw;
            q.ncolt = (Wout + best_bw - 1) / best_bw;
            q.PC = (best_bw - 1) * sw + span_w + 1;
            q.TN = 1;
            const int rstrips = (Hout + best_tp - 1) / best_tp;
            q.TP = (Hout + rstrips - 1) / rstrips;
            q.strips = ((Hout + q.TP - 1) / q.TP) * q.ncolt;
        } else {
        int tn = maxpix / (Hout * Wout);
        if (tn > MAXPATCH / (pr_full * q.PC)) tn = MAXPATCH / (pr_full * q.PC);
        if (tn >= 1) {
            q.TP = Hout;
            q.TN = tn > N ? N : tn;
            q.strips = 1;
        } else {
            int rows_fit = maxpix / Wout;
            const char *fr = env_switch(SW_STRIP_ROWS);                   // experiments: cap on the rows of a strip
            if (fr && atoi(fr) >= 1 && rows_fit > atoi(fr)) rows_fit = atoi(fr);
            const int prows = MAXPATCH / q.PC;                           // patch rows that fit
            if (prows < span_h + 1) continue;
            const int rows_patch = (prows - span_h - 1) / sh + 1;
            if (rows_fit > rows_patch) rows_fit = rows_patch;
            if (rows_fit < 1) continue;
            q.TN = 1;
            q.strips = (Hout + rows_fit - 1) / rows_fit;
            q.TP = (Hout + q.strips - 1) / q.strips;
            q.strips = (Hout + q.TP - 1) / q.TP;
        }
        }
        q.div_ncolt = make_fastdiv((uint32_t)q.ncolt);
        q.groups = (N + q.TN - 1) / q.TN;
        q.PR = (q.TP - 1) * sh + span_h + 1;
        q.npix = q.TN * q.TP * q.BW;
        q.npatch = q.TN * q.PR * q.PC;
        const int nblocks = (q.npatch + 63) / 64;
        if (nblocks > 24) continue;
        q.xpitch = nblocks * 1024 + 128;
        const size_t lds = 2 * ((size_t)2 * q.xpitch + (size_t)(out.half_cols ? 1 : 2) * ntaps * (64 * 16 + 128));
        if (lds > LDS_LIMIT) continue;
        q.div_tpq = make_fastdiv((uint32_t)(q.TP * q.BW));
        q.div_q = make_fastdiv((uint32_t)q.BW);
        q.div_prpc = make_fastdiv((uint32_t)(q.PR * q.PC));
        q.div_pc = make_fastdiv((uint32_t)q.PC);
        const long wgs = (long)q.groups * q.strips * ((Cout + 63) / 64);
        // the patch limit may leave the strip smaller than the candidate: smallest variant that holds it
        int nf_eff = nf;
        if (forced_nf <= 0) {
            if (q.npix <= 4 * 2 * 32) nf_eff = 2;
            else if (q.npix <= 4 * 4 * 32) nf_eff = 4;
        }
        best = q; best_nf = nf_eff; best_lds = lds;
        if (wgs >= NUM_CUS) break;                                   // largest strip that still fills the chip
    }
    if (!best_nf) return false;
    out = best;
    if (nf_out) *nf_out = best_nf;
    if (lds_out) *lds_out = best_lds;
    return true;
}

// Strip kernel for forward (op 0; any stride) or for residue class (ca, cb) of the output pixels of
// backprop-data (op 1; stride-1 layers have the single class (0,0)) of a multi-tap convolution.
// *empty is set when the class has no output pixel (nothing to launch).
bool strip_plan_class_uncached(const ngc_conv_desc *d, int op, int ca, int cb, int P, int Q, StripParams *sp, int *nf_out,
                               size_t *lds_out, bool *empty)
{
    if (empty) *empty = false;
    const int all_taps = d->r * d->s;
    if (all_taps < 2 || all_taps > STRIP_MAX_TAPS) return false;
    const bool fwd = op == NGC_OP_FWD;
    const int Cin = fwd ? d->c : d->k, Cout = fwd ? d->k : d->c;
    if (Cin % 16 != 0 || Cout % 16 != 0) return false;       // the last 64-channel tile of the output may be partial
    const int Hin = fwd ? d->h : P, Win = fwd ? d->w : Q;
    const int Hfull = fwd ? P : d->h, Wfull = fwd ? Q : d->w;
    const size_t in_bytes = (size_t)d->n * Cin * Hin * Win * 2;
    const size_t wt_bytes = (size_t)all_taps * Cin * Cout * 2;
    if (in_bytes >= ((size_t)1 << 31) || wt_bytes >= ((size_t)1 << 31)) return false;

    // taps of this launch: offset (dh, dw) of the input pixel relative to the position's own pixel
    int tdh[STRIP_MAX_TAPS], tdw[STRIP_MAX_TAPS], tslab[STRIP_MAX_TAPS];
    int ntaps = 0;
    const int sh = d->stride_h, sw = d->stride_w;
    for (int r = 0; r < d->r; ++r)
        for (int s2 = 0; s2 < d->s; ++s2) {
            int dh, dw;
            if (fwd) {
                dh = r * d->dil_h - d->pad_below_h;
                dw = s2 * d->dil_w - d->pad_below_w;
            } else {
                const int vh = ca + d->pad_below_h - r * d->dil_h, vw = cb + d->pad_below_w - s2 * d->dil_w;
                if (((vh % sh) + sh) % sh != 0 || ((vw % sw) + sw) % sw != 0) continue;
                dh = vh / sh;                                            // exact
                dw = vw / sw;
            }
            tdh[ntaps] = dh; tdw[ntaps] = dw; tslab[ntaps] = r * d->s + s2;
            ++ntaps;
        }
    if (ntaps == 0) {                                                    // backprop-data class no tap reaches: its pixels are
        if (empty) *empty = true;                                        // zero (strip_zero_fill), nothing to launch
        return true;
    }
    int min_dh = tdh[0], max_dh = tdh[0], min_dw = tdw[0], max_dw = tdw[0];
    for (int t = 1; t < ntaps; ++t) {
        if (tdh[t] < min_dh) min_dh = tdh[t];
        if (tdh[t] > max_dh) max_dh = tdh[t];
        if (tdw[t] < min_dw) min_dw = tdw[t];
        if (tdw[t] > max_dw) max_dw = tdw[t];
    }
    // position lattice
    const int Hout = fwd ? P : (ca < d->h ? (d->h - ca + sh - 1) / sh : 0);
    const int Wout = fwd ? Q : (cb < d->w ? (d->w - cb + sw - 1) / sw : 0);
    if (Hout == 0 || Wout == 0) {
        if (empty) *empty = true;
        return true;
    }

    StripParams q;
    memset(&q, 0, sizeof(q));
    q.N = d->n; q.Cin = Cin; q.Hin = Hin; q.Win = Win; q.Cout = Cout; q.Hout = Hout; q.Wout = Wout;
    q.Hfull = Hfull; q.Wfull = Wfull;
    q.sh = fwd ? sh : 1; q.sw = fwd ? sw : 1;
    q.os_h = fwd ? 1 : sh; q.os_w = fwd ? 1 : sw;
    q.oa_h = fwd ? 0 : ca; q.oa_w = fwd ? 0 : cb;
    q.min_dh = min_dh; q.min_dw = min_dw;
    q.ntaps = ntaps;
    q.in_bytes = (uint32_t)in_bytes;
    q.wt_bytes = (uint32_t)wt_bytes;
    {
        const size_t out_bytes = (size_t)d->n * ((Cout + 15) / 16) * Hfull * Wfull * 32;
        q.out_bytes = out_bytes < ((size_t)1 << 31) ? (uint32_t)out_bytes : 0;
    }
    if (!strip_geometry(q, d->n, Hout, Wout, max_dh - min_dh, max_dw - min_dw, ntaps, Cout, nf_out, lds_out)) return false;
    for (int t = 0; t < ntaps; ++t) {
        q.tap_off[t] = (tdh[t] - min_dh) * q.PC + (tdw[t] - min_dw);
        q.tap_slab[t] = tslab[t];
    }
    if (sp) *sp = q;
    return true;
}

struct StripClassPlan {
    bool ok, empty;
    int nf;
    size_t lds;
    StripParams sp;
};

bool strip_plan_class(const ngc_conv_desc *d, int op, int ca, int cb, int P, int Q, StripParams *sp, int *nf_out,
                      size_t *lds_out, bool *empty)
{
    static thread_local PlanCache<StripClassPlan> cache;
    const PlanKey key = plan_key(d, op, ca, cb);
    StripClassPlan *e = cache.find(key);
    if (!e) {
        StripClassPlan v;
        memset(&v, 0, sizeof(v));
        v.ok = strip_plan_class_uncached(d, op, ca, cb, P, Q, &v.sp, &v.nf, &v.lds, &v.empty);
        e = &cache.put(key, v);
    }
    if (empty) *empty = e->empty;
    if (e->ok && !e->empty) {
        if (sp) *sp = e->sp;
        if (nf_out) *nf_out = e->nf;
        if (lds_out) *lds_out = e->lds;
    }
    return e->ok;
}

}  // namespace

namespace ngc {
bool strip_plan_for_class(const ngc_conv_desc *d, int op, int ca, int cb, int P, int Q, StripParams *sp, int *nf_out,
                          size_t *lds_out, bool *empty)
{
    return strip_plan_class(d, op, ca, cb, P, Q, sp, nf_out, lds_out, empty);
}
}  // namespace ngc

namespace {

// number of residue classes of backprop-data launches (1 for forward)
int strip_classes(const ngc_conv_desc *d, int op) { return op == NGC_OP_FWD ? 1 : d->stride_h * d->stride_w; }

// true if some launch of the op cuts its rows into column tiles
bool strip_col_tiles(const ngc_conv_desc *d, int op, int P, int Q)
{
    const int ncls = strip_classes(d, op);
    for (int c = 0; c < ncls; ++c) {
        StripParams sp;
        bool empty = false;
        if (strip_plan_class(d, op, c / d->stride_w, c % d->stride_w, P, Q, &sp, nullptr, nullptr, &empty) && !empty && sp.ncolt > 1)
            return true;
    }
    return false;
}

// backprop-data: true if some residue class of the stride is reached by no tap (stride larger than the
// dilated window covers); dx is then cleared before the launches of the other classes
bool strip_zero_fill(const ngc_conv_desc *d)
{
    const int sh = d->stride_h, sw = d->stride_w;
    for (int ca = 0; ca < sh; ++ca)
        for (int cb = 0; cb < sw; ++cb) {
            bool any = false;
            for (int r = 0; r < d->r && !any; ++r)
                for (int s2 = 0; s2 < d->s && !any; ++s2) {
                    const int vh = ca + d->pad_below_h - r * d->dil_h, vw = cb + d->pad_below_w - s2 * d->dil_w;
                    any = ((vh % sh) + sh) % sh == 0 && ((vw % sw) + sw) % sw == 0;
                }
            if (!any) return true;
        }
    return false;
}

// true if every launch of the op can go through the strip kernel
bool strip_plan(const ngc_conv_desc *d, int op, int P, int Q)
{
    const char *sw = env_switch(SW_STRIP_STRIDED);                        // tests / benchmarks only: 0 = stride-1 layers only
    if (sw && atoi(sw) == 0 && (d->stride_h != 1 || d->stride_w != 1)) return false;
    const int ncls = strip_classes(d, op);
    if (ncls > 16) return false;
    for (int c = 0; c < ncls; ++c)
        if (!strip_plan_class(d, op, c / d->stride_w, c % d->stride_w, P, Q, nullptr, nullptr, nullptr, nullptr)) return false;
    return true;
}

// Filter-resident strip kernel: stride-1 forward (op 0) or backprop-data (op 1) of a multi-tap node whose filter
// tile (all taps x Cin x 64 output channels) fits the LDS next to three stage buffers of the input patch.
bool rows_plan_uncached(const ngc_conv_desc *d, int op, int P, int Q, RowsParams *rp, size_t *lds_out)
{
    // Built and measured, not selected by default: on the 56x56, 64 -> 64 layers it is level with the strip kernel at
    // batch 128 (40.1 / 40.4 us against 42.0 / 40.2 us) and behind it at batch 64 (22.5 against 21.3 / 19.9 us).
    // NGC_ROWS=1 selects it (tests / experiments).
    const char *sw = env_switch(SW_ROWS);
    if (!sw || atoi(sw) != 1) return false;
    if (env_switch(SW_STRIP_NF)) return false;   // forced strip-kernel variant
    if (d->stride_h != 1 || d->stride_w != 1) return false;
    const int ntaps = d->r * d->s;
    if (ntaps != 9) return false;                                        // the kernel's tap loop is unrolled for 9 taps
    const bool fwd = op == NGC_OP_FWD;
    const int Cin = fwd ? d->c : d->k, Cout = fwd ? d->k : d->c;
    if (Cin % 16 != 0 || Cout % 16 != 0) return false;
    const int Hin = fwd ? d->h : P, Win = fwd ? d->w : Q;
    const int Hout = fwd ? P : d->h, Wout = fwd ? Q : d->w;
    const size_t in_bytes = (size_t)d->n * Cin * Hin * Win * 2, wt_bytes = (size_t)ntaps * Cin * Cout * 2;
    if (in_bytes >= ((size_t)1 << 31) || wt_bytes >= ((size_t)1 << 31)) return false;
    const int CB = Cin / 16;
    const size_t filter_lds = (size_t)CB * ntaps * 2 * (64 * 16 + 128);
    if (filter_lds > 96 * 1024) return false;
    if (Wout < 8 || Hout < 2) return false;
    RowsParams q;
    memset(&q, 0, sizeof(q));
    int min_dh = INT_MAX, max_dh = INT_MIN, min_dw = INT_MAX, max_dw = INT_MIN;
    int tdh[STRIP_MAX_TAPS], tdw[STRIP_MAX_TAPS];
    int t = 0;
    for (int r = 0; r < d->r; ++r)
        for (int s2 = 0; s2 < d->s; ++s2) {
            tdh[t] = fwd ? r * d->dil_h - d->pad_below_h : d->pad_below_h - r * d->dil_h;
            tdw[t] = fwd ? s2 * d->dil_w - d->pad_below_w : d->pad_below_w - s2 * d->dil_w;
            if (tdh[t] < min_dh) min_dh = tdh[t];
            if (tdh[t] > max_dh) max_dh = tdh[t];
            if (tdw[t] < min_dw) min_dw = tdw[t];
            if (tdw[t] > max_dw) max_dw = tdw[t];
            q.tap_slab[t] = r * d->s + s2;
            ++t;
        }
    const int span_h = max_dh - min_dh, span_w = max_dw - min_dw;
    q.PC = Wout + span_w;
    // rows per sub-strip: at most 512 positions, a patch of at most 24 blocks of 64 pixels, everything in the LDS
    int srb = 0, nblocks = 0;
    for (int cand = 512 / Wout < Hout ? 512 / Wout : Hout; cand >= 1; --cand) {
        const int nb = ((cand + span_h) * q.PC + 63) / 64;
        if (nb > 24) continue;
        if (filter_lds + (size_t)ROWS_NBUF * 2 * ((size_t)nb * 1024 + 128) + 256 > LDS_LIMIT) continue;   // + bias
        srb = cand;
        nblocks = nb;
        break;
    }
    // worth it only while the halo rows of a sub-strip stay a minor part of its patch (wide images: strip kernel)
    if (srb < 1 || srb * Wout < 64 || srb < 2 * span_h) return false;
    // workgroups per image: enough to fill the chip, strips of whole sub-strips where possible
    const int ktiles = (Cout + 63) / 64;
    int strips = (NUM_CUS + d->n * ktiles - 1) / (d->n * ktiles);
    const int max_strips = (Hout + srb - 1) / srb;
    if (strips > max_strips) strips = max_strips;
    if (strips < 1) strips = 1;
    q.TP = (Hout + strips - 1) / strips;
    q.strips = (Hout + q.TP - 1) / q.TP;
    q.SRB = srb;
    q.N = d->n; q.Cin = Cin; q.Hin = Hin; q.Win = Win; q.Cout = Cout; q.Hout = Hout; q.Wout = Wout;
    q.min_dh = min_dh; q.min_dw = min_dw; q.span_h = span_h;
    q.nblocks = nblocks;
    q.xpitch = nblocks * 1024 + 128;
    q.ntaps = ntaps;
    for (int i = 0; i < ntaps; ++i) q.tap_off[i] = (tdh[i] - min_dh) * q.PC + (tdw[i] - min_dw);
    q.in_bytes = (uint32_t)in_bytes;
    q.wt_bytes = (uint32_t)wt_bytes;
    const size_t out_bytes = (size_t)d->n * Cout * Hout * Wout * 2;
    if (out_bytes >= ((size_t)1 << 31)) return false;
    q.out_bytes = (uint32_t)out_bytes;
    const char *fl = env_switch(SW_ROWS_LATE);                          // tests / experiments only: wave mask
    q.late_mask = fl ? (int)strtol(fl, nullptr, 0) & 0xFF : 0;
    q.div_q = make_fastdiv((uint32_t)Wout);
    q.div_pc = make_fastdiv((uint32_t)q.PC);
    if ((size_t)d->n * q.strips > 0x7FFFFFFF) return false;
    if (rp) *rp = q;
    if (lds_out) *lds_out = filter_lds + (size_t)ROWS_NBUF * 2 * q.xpitch;
    return true;
}

// Backprop-data of a low-channel stride-2 convolution (the stem) through the strip kernel.
// Output pixels are grouped into BH x BW blocks (i,j) -> (BH i + a, BW j + b); block (i,j), "channel"
// col = (a BW + b)*C + c is a convolution of dy, read at pixel (BH/2 i, BW/2 j), over the union of the
// classes' tap offsets, with a combined filter (zeros where a class has no tap) built by
// launch_subpixel_filter.  Columns are padded to 64; the strip kernel stores them as NCHW pixels.
// Blocks of 4 x 2 pixels: 24 columns for C = 3 (the kernel then skips the upper 32), 20 union taps
// for 7x7 - fewer MFMAs and LDS operand fetches per output pixel than 2 x 2 blocks with 16 taps.
struct StemBwdPlan {
    StripParams sp;
    int nf;
    size_t lds;
    int dr_min, ndr, ds_min, nds, BH, BW;
    size_t wu_bytes;
};

bool stem_bwd_plan_uncached(const ngc_conv_desc *d, int P, int Q, StemBwdPlan *out)
{
    if (d->dtype != NGC_BF16 || d->x_layout != NGC_NCHW || d->y_layout != NGC_NCHW16C || d->w_layout != NGC_KCRS)
        return false;
    if (d->stride_h != 2 || d->stride_w != 2 || d->dil_h != 1 || d->dil_w != 1) return false;
    if (d->k % 16 != 0) return false;
    StemBwdPlan pl;
    pl.BW = 2;
    pl.BH = (4 * 2 * d->c <= 32) ? 4 : 2;
    const char *fb = env_switch(SW_STEM_BH);                               // tests / experiments only
    if (fb && atoi(fb) == 2) pl.BH = 2;
    if (pl.BH * pl.BW * d->c > 64) return false;
    int dr_min = INT_MAX, dr_max = INT_MIN, ds_min = INT_MAX, ds_max = INT_MIN;
    for (int a = 0; a < pl.BH; ++a)
        for (int r = 0; r < d->r; ++r) {
            const int v = a + d->pad_below_h - r;
            if (v & 1) continue;
            const int dr = v / 2;                                  // exact (v may be negative and even)
            if (dr < dr_min) dr_min = dr;
            if (dr > dr_max) dr_max = dr;
        }
    for (int b = 0; b < pl.BW; ++b)
        for (int s2 = 0; s2 < d->s; ++s2) {
            const int v = b + d->pad_below_w - s2;
            if (v & 1) continue;
            const int ds = v / 2;
            if (ds < ds_min) ds_min = ds;
            if (ds > ds_max) ds_max = ds;
        }
    if (dr_min > dr_max || ds_min > ds_max) return false;
    pl.dr_min = dr_min; pl.ndr = dr_max - dr_min + 1;
    pl.ds_min = ds_min; pl.nds = ds_max - ds_min + 1;
    const int ntaps = pl.ndr * pl.nds;
    if (ntaps < 2 || ntaps > STRIP_MAX_TAPS) return false;
    const size_t in_bytes = (size_t)d->n * d->k * P * Q * 2;
    pl.wu_bytes = (size_t)ntaps * d->k * 64 * 2;
    if (in_bytes >= ((size_t)1 << 31)) return false;
    StripParams q;
    memset(&q, 0, sizeof(q));
    const int Hout = (d->h + pl.BH - 1) / pl.BH, Wout = (d->w + pl.BW - 1) / pl.BW;
    q.N = d->n; q.Cin = d->k; q.Hin = P; q.Win = Q; q.Cout = 64; q.Hout = Hout; q.Wout = Wout;
    q.min_dh = dr_min; q.min_dw = ds_min;
    q.ntaps = ntaps;
    q.in_bytes = (uint32_t)in_bytes;
    q.wt_bytes = (uint32_t)pl.wu_bytes;
    q.out_mode = 1;
    q.sub_C = d->c; q.sub_H = d->h; q.sub_W = d->w; q.sub_BH = pl.BH; q.sub_BW = pl.BW;
    q.sh = pl.BH / 2; q.sw = pl.BW / 2;                                  // dy pixels per block step
    q.half_cols = pl.BH * pl.BW * d->c <= 32 ? 1 : 0;
    q.os_h = q.os_w = 1; q.Hfull = Hout; q.Wfull = Wout;
    if (!strip_geometry(q, d->n, Hout, Wout, pl.ndr - 1, pl.nds - 1, ntaps, 64, &pl.nf, &pl.lds)) return false;
    // rows of the strip can go through LDS if they fit the stage buffers and are made of 16-byte pieces
    q.sub_stage = (d->w % 8 == 0 && pl.BW * Wout == d->w &&
                   (size_t)q.TN * d->c * pl.BH * q.TP * d->w * 2 <= pl.lds) ? 1 : 0;
    {
        const int ROWS = pl.BH * q.TP, WP = pl.BW * Wout;
        for (int col = 0; col < 64; ++col) {
            q.sub_off[col] = -1;
            if (col < pl.BH * pl.BW * d->c) {
                const int ab = col / d->c, c = col - ab * d->c;
                const int a = ab / pl.BW, b = ab - a * pl.BW;
                q.sub_off[col] = (c * ROWS + a) * WP + b;
            }
        }
        q.div_chunks = make_fastdiv((uint32_t)(d->w / 8 > 0 ? d->w / 8 : 1));
        q.div_rows = make_fastdiv((uint32_t)ROWS);
        q.div_subc = make_fastdiv((uint32_t)d->c);
    }
    int t = 0;
    for (int i = 0; i < pl.ndr; ++i)
        for (int j = 0; j < pl.nds; ++j) {
            q.tap_off[t] = i * q.PC + j;
            q.tap_slab[t] = t;
            ++t;
        }
    pl.sp = q;
    if (out) *out = pl;
    return true;
}

// Geometry of the all-taps backprop-filters kernel (stride 1, exactly 9 taps, C and K multiples of 64).
bool wgrad_strip_plan_uncached(const ngc_conv_desc *d, int P, int Q, WgradStripParams *wp, size_t *lds_out)
{
    const char *force = env_switch(SW_WGRAD_STRIP);
    if (force && atoi(force) == 0) return false;
    if (d->stride_h != 1 || d->stride_w != 1 || d->r * d->s != 9) return false;
    if (d->c % 64 != 0 || d->k % 64 != 0) return false;
    const size_t x_bytes = (size_t)d->n * d->c * d->h * d->w * 2, dy_bytes = (size_t)d->n * d->k * P * Q * 2;
    if (x_bytes >= ((size_t)1 << 31) || dy_bytes >= ((size_t)1 << 31)) return false;
    if (Q > 224) return false;
    WgradStripParams q;
    memset(&q, 0, sizeof(q));
    const int span_h = d->dil_h * (d->r - 1), span_w = d->dil_w * (d->s - 1);
    q.SR = 224 / Q;
    if (q.SR > P) q.SR = P;
    q.PRS = q.SR + span_h;
    q.PC = Q + span_w;
    // channel groups per workgroup: few (k,c) tiles -> narrower c per workgroup, longer position chunks
    const int tiles64 = (d->k / 64) * (d->c / 64);
    q.ncq = tiles64 <= 4 ? 2 : 4;
    const char *fq = env_switch(SW_WGRAD_NCQ);
    if (fq && (atoi(fq) == 1 || atoi(fq) == 2 || atoi(fq) == 4)) q.ncq = atoi(fq);
    // small images: several whole images per stage (a stage of one 7x7 image would be 1.5 steps),
    // as many as a workgroup's share of the batch allows
    q.G = 1;
    {
        const int tiles_g = (d->k / 64) * (d->c / (16 * q.ncq));
        const int parts_g = tiles_g >= NUM_CUS ? 1 : (NUM_CUS + tiles_g - 1) / tiles_g;
        const char *fg = env_switch(SW_WGRAD_G1);                        // tests / experiments only: one image per stage
        if (q.SR == P && 2 * P * Q <= 224 && parts_g <= d->n && !(fg && atoi(fg) == 1)) {
            q.G = 224 / (P * Q);
            if (q.G > d->n / parts_g) q.G = d->n / parts_g;
        }
    }
    const int nblk_x = (q.G * q.PRS * q.PC + 31) / 32;
    const int nblk_dy = (q.G > 1 ? q.G * P * Q + 31 : q.SR * Q + 31) / 32;   // 32-position steps per stage
    q.dyplane = nblk_dy * 1024 + 128;
    q.xplane = nblk_x * 1024 + 128;
    if (nblk_dy > 7 || q.ncq * nblk_x > 56) return false;               // load slots per wave and stage: 4 of dy, 7 of x
    const size_t stage = (size_t)4 * q.dyplane + (size_t)q.ncq * q.xplane;
    q.nring = 3 * stage <= LDS_LIMIT ? 3 : 2;
    const char *fr = env_switch(SW_WGRAD_RING);                          // tests / benchmarks only
    if (fr && atoi(fr) == 2) q.nring = 2;
    // waves 0-3 (one wave of each SIMD) issue their loads after their MFMAs, waves 4-7 right after the barrier;
    // NGC_WGRAD_LATE (tests / benchmarks only) sets another wave mask, 0 = every wave issues right after the barrier
    const char *fl = env_switch(SW_WGRAD_LATE);
    q.late_mask = fl ? (int)strtol(fl, nullptr, 0) & 0xFF : 0x0F;
    size_t lds = q.nring * stage;
    const size_t red = (size_t)4 * 144 * 64 * sizeof(float);           // final cross-wave sum
    if (lds < red) lds = red;
    if (lds > LDS_LIMIT) return false;
    const int tiles = (d->k / 64) * (d->c / (16 * q.ncq));
    // enough workgroups to fill the chip, as few partial copies of dw as possible
    int parts_wanted = (NUM_CUS + tiles - 1) / tiles;
    if (tiles >= NUM_CUS) parts_wanted = 1;
    const int max_strips = (P + q.SR - 1) / q.SR;
    if (parts_wanted <= d->n) {
        q.strips = 1;
        q.NI = d->n / parts_wanted;                                      // >= 1
    } else {
        q.NI = 1;
        q.strips = (parts_wanted + d->n - 1) / d->n;
        if (q.strips > max_strips) q.strips = max_strips;
    }
    q.TP = (P + q.strips - 1) / q.strips;
    q.strips = (P + q.TP - 1) / q.TP;
    q.nstages = (q.TP + q.SR - 1) / q.SR;
    q.nparts = ((d->n + q.NI - 1) / q.NI) * q.strips;
    q.N = d->n; q.C = d->c; q.H = d->h; q.W = d->w; q.K = d->k; q.P = P; q.Q = Q;
    q.min_dh = -d->pad_below_h;
    q.min_dw = -d->pad_below_w;
    int t = 0;
    for (int r = 0; r < d->r; ++r)
        for (int s2 = 0; s2 < d->s; ++s2) q.tap_off[t++] = r * d->dil_h * q.PC + s2 * d->dil_w;
    q.ctiles = d->c / (16 * q.ncq);
    {
        // NGC_WGRAD_NT (tests / experiments): 0 / 1 = never / always
        const size_t part_bytes = (size_t)q.nparts * 9 * d->k * d->c * sizeof(float);
        const char *fn = env_switch(SW_WGRAD_NT);
        q.stream_partials = fn ? (atoi(fn) != 0) : (part_bytes <= ((size_t)24 << 20));
    }
    q.x_bytes = (uint32_t)x_bytes;
    q.dy_bytes = (uint32_t)dy_bytes;
    q.div_q = make_fastdiv((uint32_t)Q);
    q.div_pc = make_fastdiv((uint32_t)q.PC);
    q.div_pq = make_fastdiv((uint32_t)(P * Q));
    q.div_patch = make_fastdiv((uint32_t)(q.PRS * q.PC));
    if (wp) *wp = q;
    if (lds_out) *lds_out = lds;
    return true;
}

// low-channel stem forward: C <= 3, 7x7, stride 2, pad_below_w 3, NCHW input, blocked output
bool stem_fwd_plan_uncached(const ngc_conv_desc *d, int P, int Q, StemFwdParams *sp, size_t *lds_out)
{
    if (d->dtype != NGC_BF16 || d->x_layout != NGC_NCHW || d->y_layout != NGC_NCHW16C || d->w_layout != NGC_KCRS)
        return false;
    if (d->c > 3 || d->r != 7 || d->s != 7 || d->stride_h != 2 || d->stride_w != 2 || d->dil_h != 1 || d->dil_w != 1)
        return false;
    if (d->pad_below_w != 3 || d->w % 8 != 0 || d->k % 64 != 0 || 2 * Q > d->w + 2) return false;
    StemFwdParams q;
    memset(&q, 0, sizeof(q));
    q.N = d->n; q.C = d->c; q.H = d->h; q.W = d->w; q.K = d->k; q.P = P; q.Q = Q;
    q.pbh = d->pad_below_h;
    // Output rows per workgroup.  Two workgroups share a compute unit (registers), so a launch runs in rounds of
    // 2 * NUM_CUS workgroups; a workgroup costs its rows plus a fixed part (filter fragments, patch set-up, about 2.5
    // rows' worth).  Take the tile height with the least rounds x cost that fits the LDS: N = 64, 224x224 runs as one
    // round of 512 workgroups of 14 rows (29.3 us) instead of 1.75 rounds of 8 rows (35.2 us).
    auto stem_lds = [&](int tp) {
        const size_t patch = (size_t)d->c * (2 * tp + 5) * (2 * d->w + 16);
        return ((patch + 15) & ~(size_t)15) + (size_t)64 * d->c * 49 * 2;
    };
    q.TP = P < 8 ? P : 8;
    {
        double best = 0;
        for (int tp = P < 4 ? P : 4; tp <= 16 && tp <= P; ++tp) {
            if (stem_lds(tp) > 64 * 1024) break;
            const size_t wgs = (size_t)d->n * ((P + tp - 1) / tp) * (d->k / 64);
            const double cost = (double)((wgs + 2 * NUM_CUS - 1) / (2 * NUM_CUS)) * (tp + 2.5);
            if (best == 0 || cost <= best) {
                best = cost;
                q.TP = tp;
            }
        }
    }
    const char *ftp = env_switch(SW_STEM_TP);                            // tests / benchmarks only: output rows per workgroup
    if (ftp && atoi(ftp) >= 1 && atoi(ftp) <= 16 && atoi(ftp) <= P) q.TP = atoi(ftp);
    q.tiles_per_img = (P + q.TP - 1) / q.TP;
    q.div_q = make_fastdiv((uint32_t)Q);
    q.div_cpr = make_fastdiv((uint32_t)(d->w / 8));
    q.div_rows = make_fastdiv((uint32_t)(2 * q.TP + 5));
    {
        const size_t y_bytes = (size_t)d->n * d->k * P * Q * 2;
        q.y_bytes = y_bytes < ((size_t)1 << 31) ? (uint32_t)y_bytes : 0;
    }
    const size_t lds = stem_lds(q.TP);
    if (lds > 64 * 1024) return false;
    if ((size_t)d->n * q.tiles_per_img > 0x7FFFFFFF) return false;
    if (sp) *sp = q;
    if (lds_out) *lds_out = lds;
    return true;
}

// low-channel stem backprop-filters: same shapes as stem forward, plus Q % 8 == 0
bool wgrad_stem_plan_uncached(const ngc_conv_desc *d, int P, int Q, WgradStemParams *wp, size_t *lds_out)
{
    if (d->dtype != NGC_BF16 || d->x_layout != NGC_NCHW || d->y_layout != NGC_NCHW16C) return false;
    if (d->c > 3 || d->r != 7 || d->s != 7 || d->stride_h != 2 || d->stride_w != 2 || d->dil_h != 1 || d->dil_w != 1)
        return false;
    if (d->pad_below_w != 3 || d->w % 8 != 0 || d->k % 64 != 0 || 2 * Q > d->w || Q % 8 != 0) return false;
    const size_t dy_bytes = (size_t)d->n * d->k * P * Q * 2;
    if (dy_bytes >= ((size_t)1 << 31)) return false;
    WgradStemParams q;
    memset(&q, 0, sizeof(q));
    const size_t x_bytes = (size_t)d->n * d->c * d->h * d->w * 2;
    if (x_bytes >= ((size_t)1 << 31)) return false;
    int sr0 = 1;
    while ((sr0 * Q) % 32 != 0) ++sr0;                                  // <= 4 since Q % 8 == 0
    // positions per stage (NGC_WSTEM_POS, experiments): a stage costs a load latency whatever its size
    int stage_pos = 512;
    const char *fp = env_switch(SW_WSTEM_POS);
    if (fp && atoi(fp) >= 32 && atoi(fp) <= 1024) stage_pos = atoi(fp);
    // LDS of a workgroup with `nbuf` stage buffers of sr dy rows (+ two staging areas for the raw input rows when
    // there are three); 0 if the input rows of a stage need more than 3 pieces per thread
    // LDS pitches of the input rows: a parity plane holds W + 16 bytes; with the plane pitch = 8 and the row pitch = 64
    // (mod 256 bytes) the lanes of one operand read - two (c, r) rows, both planes, four position groups 16 bytes apart,
    // two neighbouring dwords - hit 64 different banks (with W + 16 and twice that, plane and group offsets collide)
    q.PL = (d->w + 16 - 8 + 255) / 256 * 256 + 8;
    q.RPX = (2 * q.PL - 64 + 255) / 256 * 256 + 64;
    const int rpx = q.RPX;
    auto lds_need = [&](int sr, int nbuf) -> size_t {
        const int rows_in = 2 * sr + 5;
        const int xchunks = d->c * rows_in * (d->w / 8);
        if (xchunks > 1536) return 0;
        const size_t dyplane = (size_t)(sr * Q / 32) * 1024 + 128;
        const size_t xbytes = (size_t)d->c * rows_in * rpx;
        size_t lds = nbuf * (4 * dyplane + ((xbytes + 15) & ~(size_t)15));
        if (nbuf == 3) lds += 2 * (size_t)((xchunks + 63) & ~63) * 16;
        return lds < 98304 ? 98304 : lds;                               // final cross-wave tree
    };
    auto largest_sr = [&](int nbuf) {
        if (lds_need(sr0, nbuf) == 0 || lds_need(sr0, nbuf) > LDS_LIMIT) return 0;
        int sr = sr0;
        while (2 * sr * Q <= stage_pos && 2 * sr <= P && lds_need(2 * sr, nbuf) != 0 && lds_need(2 * sr, nbuf) <= LDS_LIMIT) sr *= 2;
        return sr;
    };
    // Three buffers (the loads of two stages in flight behind the one being multiplied) when they fit, else two.
    // NGC_WSTEM_RING (tests / benchmarks only): 2 = two buffers.
    const char *fr = env_switch(SW_WSTEM_RING);
    int sr = (fr && atoi(fr) == 2) ? 0 : largest_sr(3);
    q.ring = sr > 0;
    if (!q.ring) sr = largest_sr(2);
    if (sr == 0) return false;
    q.SR = sr;
    q.dyplane = (sr * Q / 32) * 1024 + 128;
    const size_t lds = lds_need(sr, q.ring ? 3 : 2);
    q.x_bytes = (uint32_t)x_bytes;
    const int ktiles = d->k / 64;
    int strips = (NUM_CUS + d->n * ktiles - 1) / (d->n * ktiles);
    const int max_strips = (P + sr - 1) / sr;
    if (strips > max_strips) strips = max_strips;
    if (strips < 1) strips = 1;
    int tp = (P + strips - 1) / strips;
    tp = (tp + sr - 1) / sr * sr;
    q.TP = tp;
    q.strips = (P + tp - 1) / tp;
    q.N = d->n; q.C = d->c; q.H = d->h; q.W = d->w; q.K = d->k; q.P = P; q.Q = Q;
    q.pbh = d->pad_below_h;
    q.dy_bytes = (uint32_t)dy_bytes;
    q.div_q = make_fastdiv((uint32_t)Q);
    if (wp) *wp = q;
    if (lds_out) *lds_out = lds;
    return true;
}

// backprop-filters as a per-tap GEMM over positions (1x1 layers, strided multi-tap layers)
bool wgrad_gemm_plan_uncached(const ngc_conv_desc *d, int P, int Q, WgradGemmParams *wp)
{
    const char *force = env_switch(SW_WGRAD_GEMM);
    if (force && atoi(force) == 0) return false;
    if (d->c % 16 != 0 || d->k % 16 != 0 || d->r * d->s > 64 || d->dtype != NGC_BF16) return false;
    const size_t x_bytes = (size_t)d->n * d->c * d->h * d->w * 2, dy_bytes = (size_t)d->n * d->k * P * Q * 2;
    if (x_bytes >= ((size_t)1 << 31) || dy_bytes >= ((size_t)1 << 31)) return false;
    WgradGemmParams q;
    memset(&q, 0, sizeof(q));
    // layout propagation: either operand may be NCHW when positions map one to one (1x1, stride 1, no
    // padding) and 8 consecutive positions never straddle two images
    q.x_nchw = d->x_layout == NGC_NCHW;
    q.dy_nchw = d->y_layout == NGC_NCHW;
    if (q.x_nchw || q.dy_nchw) {
        const char *lp = env_switch(SW_G1_NCHW);          // tests / benchmarks only: 0 = NCHW tensors take the direct kernels
        if (lp && atoi(lp) == 0) return false;
        if (d->r != 1 || d->s != 1 || d->stride_h != 1 || d->stride_w != 1 || d->pad_below_h || d->pad_below_w ||
            d->pad_above_h || d->pad_above_w || (d->h * d->w) % 8 != 0)
            return false;
    }
    q.N = d->n; q.C = d->c; q.H = d->h; q.W = d->w; q.K = d->k; q.P = P; q.Q = Q; q.R = d->r; q.S = d->s;
    q.sh = d->stride_h; q.sw = d->stride_w; q.dil_h = d->dil_h; q.dil_w = d->dil_w;
    q.pbh = d->pad_below_h; q.pbw = d->pad_below_w;
    // 128-wide tiles when they waste no more of a partial last tile than 64-wide ones (channel counts % 16 == 0)
    auto wide = [](int ch) { return ch > 64 && (ch + 127) / 128 * 128 <= (ch + 63) / 64 * 64; };
    q.wk = wide(d->k) ? 2 : 1;
    q.wc = wide(d->c) ? 2 : 1;
    const char *ft = env_switch(SW_WGG_TILE);                             // tests / benchmarks only: "11", "12", "21", "22"
    if (ft && (ft[0] == '1' || ft[0] == '2') && (ft[1] == '1' || ft[1] == '2')) {
        q.wk = ft[0] - '0';
        q.wc = ft[1] - '0';
    }
    q.ktiles = (d->k + 64 * q.wk - 1) / (64 * q.wk);
    q.ctiles = (d->c + 64 * q.wc - 1) / (64 * q.wc);
    q.M = (uint32_t)d->n * P * Q;
    const uint32_t tiles = (uint32_t)q.ktiles * q.ctiles * d->r * d->s;
    // Stage size: 64-position stages take half the LDS, so two workgroups fit a compute unit and
    // twice as many position chunks are cut.  That pays when there are many (tile, tap) pairs, i.e.
    // few chunks and little extra partial traffic, and for multi-tap layers; the large-image 1x1
    // layers are HBM-bound and keep 128-position stages.  NGC_WGG_SP (experiments only) forces 64 / 128.
    const char *fsp = env_switch(SW_WGG_SP);
    // Measured per layer over the ResNet-50 stack (reproducible to 1 %): 64 wins from 16 tiles on, and
    // by 20-24 % where one operand is read by a single tile row / column and the other by four or more
    // (128 -> 512 and 512 -> 128 at 28x28); with 2 x 4 tiles it loses 35-65 %.
    const int tmin = q.ktiles < q.ctiles ? q.ktiles : q.ctiles, tmax = q.ktiles < q.ctiles ? q.ctiles : q.ktiles;
    q.sp = (d->r * d->s > 1 || tiles >= 16 || (tmin == 1 && tmax >= 4)) ? 64 : 128;
    if (fsp && (atoi(fsp) == 64 || atoi(fsp) == 128)) q.sp = atoi(fsp);
    uint32_t slots = q.sp == 64 ? 2 * NUM_CUS : NUM_CUS;
    const char *fs = env_switch(SW_WGG_SLOTS);                            // tests / benchmarks only: workgroups aimed at
    if (fs && atoi(fs) >= 32 && atoi(fs) <= 4096) slots = (uint32_t)atoi(fs);
    uint32_t parts = (slots + tiles - 1) / tiles;
    // many (tile, tap) pairs: a few workgroups more than the slots cost a whole extra round of long workgroups
    // (3x3 stride 2, 512 -> 512: 576 workgroups 78 us, 432 workgroups 57 us), so round down there
    if (tiles >= 64 && slots / tiles >= 1) parts = slots / tiles;
    // Multi-tap layers on large tensors: XCD-ordered one-dimensional grid (the (tile, tap) workgroups of a position
    // chunk on one XCD, sharing the chunk through its L2 instead of re-reading it from HBM once per tap).  It needs
    // the chunk count in multiples of 8, so only where that changes the workgroup count by at most a tenth.  Measured:
    // (3,1) window over 16 x 3136 rows, 128 -> 64: 73 -> 59 us; 3x3/2 128 -> 128 at 56x56: 33 -> 25 us (N = 32),
    // 47 -> 48 us (N = 128); small tensors and layers with 25-36 (tile, tap) pairs lose 3-40 %.
    // NGC_WGG_XCD (tests / benchmarks only): 0 = never, 1 = every multi-tap layer.
    if (d->r * d->s > 1 && !q.x_nchw && !q.dy_nchw) {
        const uint32_t xcd_slots = slots / 8;
        const uint32_t parts8 = 8 * (xcd_slots / tiles > 0 ? xcd_slots / tiles : 1);
        const char *fx = env_switch(SW_WGG_XCD);
        bool on = x_bytes + dy_bytes >= ((size_t)24 << 20) && parts8 * 10 >= parts * 9 && parts8 * 10 <= parts * 11;
        if (fx) on = atoi(fx) == 1;
        if (on) {
            q.xcd_order = 1;
            parts = parts8;
        }
    }
    const uint32_t max_parts = (q.M + 127) / 128;
    if (parts > max_parts) parts = max_parts;
    if (parts < 1) parts = 1;
    uint32_t chunk = (q.M + parts - 1) / parts;
    chunk = (chunk + 127) / 128 * 128;
    q.chunk = chunk;
    q.nparts = (int)((q.M + chunk - 1) / chunk);
    // One-tap layers with several tiles: the tiles of a chunk share x or dy; with many chunks whose count is no
    // multiple of 8 the two-dimensional grid spreads them over the XCDs, the XCD-ordered grid does not.  Measured
    // on the 56x56 layers of the ResNet-50 stack (126 chunks, two tiles): 64 -> 256 53.2 -> 49.7 us, 256 -> 64
    // 52.4 -> 46.9 us, but 256 -> 128 (128 x 128 tiles) 72.0 -> 75.5 us, so not for that tile shape.
    if (d->r * d->s == 1 && tiles > 1 && q.wk * q.wc < 4 && q.nparts >= 64 && q.nparts % 8 != 0) {
        const char *fx = env_switch(SW_WGG_XCD);
        if (!(fx && atoi(fx) == 0)) q.xcd_order = 1;
    }
    q.x_bytes = (uint32_t)x_bytes;
    q.dy_bytes = (uint32_t)dy_bytes;
    q.div_pq = make_fastdiv((uint32_t)(P * Q));
    q.div_q = make_fastdiv((uint32_t)Q);
    if (wp) *wp = q;
    return true;
}

// One-tap GEMM kernel for forward (op 0) or backprop-data (op 1) of a 1x1 convolution, any stride.
// Backprop-data with stride > 1 computes the one residue class of pixels the tap reaches; `zero`
// reports that the rest of dx has to be cleared first.
bool gemm1x1_plan_uncached(const ngc_conv_desc *d, int op, int P, int Q, Gemm1x1Params *gp, bool *zero)
{
    const char *sw = env_switch(SW_GEMM1X1);              // tests / benchmarks only: 0 disables this kernel
    if (sw && atoi(sw) == 0) return false;
    if (d->r != 1 || d->s != 1) return false;
    const bool fwd = op == NGC_OP_FWD;
    const int Cin = fwd ? d->c : d->k, Cout = fwd ? d->k : d->c;
    if (Cin % 16 != 0 || Cout % 16 != 0 || d->dtype != NGC_BF16) return false;   // partial last tiles / stages are masked
    Gemm1x1Params q;
    memset(&q, 0, sizeof(q));
    q.Cin = Cin; q.Cout = Cout;
    // layout propagation: either side may be NCHW when positions map one to one (stride 1, no padding)
    // and 8 consecutive positions never straddle two images
    q.in_nchw = (fwd ? d->x_layout : d->y_layout) == NGC_NCHW;
    q.out_nchw = (fwd ? d->y_layout : d->x_layout) == NGC_NCHW;
    if (q.in_nchw || q.out_nchw) {
        const char *lp = env_switch(SW_G1_NCHW);          // tests / benchmarks only: 0 = NCHW tensors take the direct kernels
        if (lp && atoi(lp) == 0) return false;
        if (d->stride_h != 1 || d->stride_w != 1 || d->pad_below_h || d->pad_below_w || d->pad_above_h || d->pad_above_w ||
            (d->h * d->w) % 8 != 0)
            return false;
    }
    int OP, OQ;
    bool z = false;
    if (fwd) {
        q.Hin = d->h; q.Win = d->w; q.Hout = P; q.Wout = Q;
        q.is_h = d->stride_h; q.is_w = d->stride_w;
        q.dh = -d->pad_below_h; q.dw = -d->pad_below_w;
        q.os_h = q.os_w = 1; q.oa_h = q.oa_w = 0;
        OP = P; OQ = Q;
    } else {
        const int sh = d->stride_h, sw_ = d->stride_w;
        const int a = (sh - d->pad_below_h % sh) % sh, b = (sw_ - d->pad_below_w % sw_) % sw_;
        q.Hin = P; q.Win = Q; q.Hout = d->h; q.Wout = d->w;
        q.is_h = q.is_w = 1;
        q.dh = (a + d->pad_below_h) / sh; q.dw = (b + d->pad_below_w) / sw_;      // exact
        q.os_h = sh; q.os_w = sw_; q.oa_h = a; q.oa_w = b;
        OP = a < d->h ? (d->h - a + sh - 1) / sh : 0;
        OQ = b < d->w ? (d->w - b + sw_ - 1) / sw_ : 0;
        z = sh > 1 || sw_ > 1;
        // the lattice starts at pixel (0, 0) and its blocks of sh x sw pixels tile the image: the kernel writes the
        // zeros of a block next to its one computed pixel, no fill pass
        if (z && a == 0 && b == 0 && sh * sw_ <= 4 && !q.out_nchw && OP * sh >= d->h && OQ * sw_ >= d->w) {
            q.zero_sib = 1;
            z = false;
        }
    }
    const size_t in_bytes = (size_t)d->n * Cin * q.Hin * q.Win * 2, wt_bytes = (size_t)Cin * Cout * 2;
    const size_t m = (size_t)d->n * OP * OQ;
    if (in_bytes >= 0x80000000ull || wt_bytes >= 0x80000000ull || m >= 0x7fff0000ull) return false;
    q.M = (uint32_t)m;
    q.in_bytes = (uint32_t)in_bytes;
    q.wt_bytes = (uint32_t)wt_bytes;
    {
        const size_t out_bytes = (size_t)d->n * ((Cout + 15) / 16) * q.Hout * q.Wout * 32;
        q.out_bytes = (!q.out_nchw && out_bytes < 0x80000000ull) ? (uint32_t)out_bytes : 0;
    }
    q.div_pq = make_fastdiv((uint32_t)(OP * OQ > 0 ? OP * OQ : 1));
    q.div_q = make_fastdiv((uint32_t)(OQ > 0 ? OQ : 1));
    if (gp) *gp = q;
    if (zero) *zero = z;
    return true;
}

// cached forms of the planning functions above (same signatures)
template <class T>
struct CachedPlan {
    bool ok;
    size_t lds;
    bool flag;
    T v;
};

bool stem_bwd_plan(const ngc_conv_desc *d, int P, int Q, StemBwdPlan *out)
{
    static thread_local PlanCache<CachedPlan<StemBwdPlan>> cache;
    const PlanKey key = plan_key(d);
    auto *e = cache.find(key);
    if (!e) {
        CachedPlan<StemBwdPlan> v;
        memset(&v, 0, sizeof(v));
        v.ok = stem_bwd_plan_uncached(d, P, Q, &v.v);
        e = &cache.put(key, v);
    }
    if (e->ok && out) *out = e->v;
    return e->ok;
}

#define NGC_CACHED_PLAN_LDS(NAME, TYPE)                                                  \
    bool NAME(const ngc_conv_desc *d, int P, int Q, TYPE *out, size_t *lds_out)          \
    {                                                                                    \
        static thread_local PlanCache<CachedPlan<TYPE>> cache;                           \
        const PlanKey key = plan_key(d);                                                 \
        auto *e = cache.find(key);                                                       \
        if (!e) {                                                                        \
            CachedPlan<TYPE> v;                                                          \
            memset(&v, 0, sizeof(v));                                                    \
            v.ok = NAME##_uncached(d, P, Q, &v.v, &v.lds);                               \
            e = &cache.put(key, v);                                                      \
        }                                                                                \
        if (e->ok && out) *out = e->v;                                                   \
        if (e->ok && lds_out) *lds_out = e->lds;                                         \
        return e->ok;                                                                    \
    }
NGC_CACHED_PLAN_LDS(wgrad_strip_plan, WgradStripParams)
NGC_CACHED_PLAN_LDS(stem_fwd_plan, StemFwdParams)
NGC_CACHED_PLAN_LDS(wgrad_stem_plan, WgradStemParams)
#undef NGC_CACHED_PLAN_LDS

bool wgrad_gemm_plan(const ngc_conv_desc *d, int P, int Q, WgradGemmParams *wp)
{
    static thread_local PlanCache<CachedPlan<WgradGemmParams>> cache;
    const PlanKey key = plan_key(d);
    auto *e = cache.find(key);
    if (!e) {
        CachedPlan<WgradGemmParams> v;
        memset(&v, 0, sizeof(v));
        v.ok = wgrad_gemm_plan_uncached(d, P, Q, &v.v);
        e = &cache.put(key, v);
    }
    if (e->ok && wp) *wp = e->v;
    return e->ok;
}

bool gemm1x1_plan(const ngc_conv_desc *d, int op, int P, int Q, Gemm1x1Params *gp, bool *zero)
{
    static thread_local PlanCache<CachedPlan<Gemm1x1Params>> cache;
    const PlanKey key = plan_key(d, op);
    auto *e = cache.find(key);
    if (!e) {
        CachedPlan<Gemm1x1Params> v;
        memset(&v, 0, sizeof(v));
        v.ok = gemm1x1_plan_uncached(d, op, P, Q, &v.v, &v.flag);
        e = &cache.put(key, v);
    }
    if (e->ok && gp) *gp = e->v;
    if (e->ok && zero) *zero = e->flag;
    return e->ok;
}

bool rows_plan(const ngc_conv_desc *d, int op, int P, int Q, RowsParams *rp, size_t *lds_out)
{
    static thread_local PlanCache<CachedPlan<RowsParams>> cache;
    const PlanKey key = plan_key(d, op);
    auto *e = cache.find(key);
    if (!e) {
        CachedPlan<RowsParams> v;
        memset(&v, 0, sizeof(v));
        v.ok = rows_plan_uncached(d, op, P, Q, &v.v, &v.lds);
        e = &cache.put(key, v);
    }
    if (e->ok && rp) *rp = e->v;
    if (e->ok && lds_out) *lds_out = e->lds;
    return e->ok;
}

bool blocked_bf16(const ngc_conv_desc *d)
{
    return d->dtype == NGC_BF16 && d->x_layout == NGC_NCHW16C && d->y_layout == NGC_NCHW16C;
}

Variant pick_base(const ngc_conv_desc *d, int op)
{
    int P, Q;
    if (validate(d, &P, &Q) != NGC_OK) return V_INVALID;
    if (op == NGC_OP_FWD) {
        if (stem_fwd_plan(d, P, Q, nullptr, nullptr)) return V_STEM_FWD;
        const bool wl = d->w_layout == NGC_KCRS || d->w_layout == NGC_BLOCKED_FWD;
        const bool base = blocked_bf16(d) && wl;
        const bool mf = base && d->c % 32 == 0 && d->k % 64 == 0 && d->r * d->s <= IGEMM_MAX_TAPS;
        if (base && strip_plan(d, op, P, Q)) return rows_plan(d, op, P, Q, nullptr, nullptr) ? V_ROWS : V_STRIP;
        if (wl && gemm1x1_plan(d, op, P, Q, nullptr, nullptr)) return V_GEMM1X1;
        if (mf) return d->k % 128 == 0 ? V_IGEMM_128 : V_IGEMM_64;
        return d->w_layout == NGC_KCRS ? V_DIRECT : V_UNSUPPORTED;
    }
    if (op == NGC_OP_BWD_DATA) {
        if (stem_bwd_plan(d, P, Q, nullptr)) return V_STEM_BWD;
        const bool wl = d->w_layout == NGC_KCRS || d->w_layout == NGC_BLOCKED_BWD;
        const bool base = blocked_bf16(d) && wl;
        const bool mf = base && d->k % 32 == 0 && d->c % 64 == 0 && d->r * d->s <= IGEMM_MAX_TAPS &&
                        d->stride_h * d->stride_w <= IGEMM_MAX_CLASSES;
        if (base && strip_plan(d, op, P, Q)) return rows_plan(d, op, P, Q, nullptr, nullptr) ? V_ROWS : V_STRIP;
        if (wl && gemm1x1_plan(d, op, P, Q, nullptr, nullptr)) return V_GEMM1X1;
        if (mf) return d->c % 128 == 0 ? V_IGEMM_128 : V_IGEMM_64;
        return d->w_layout == NGC_KCRS ? V_DIRECT : V_UNSUPPORTED;
    }
    if (op == NGC_OP_BWD_FILTERS) {
        if (wgrad_stem_plan(d, P, Q, nullptr, nullptr)) return V_WGRAD_STEM;
        if (blocked_bf16(d) && wgrad_strip_plan(d, P, Q, nullptr, nullptr)) return V_WGRAD_STRIP;
        if ((blocked_bf16(d) || d->r * d->s == 1) && wgrad_gemm_plan(d, P, Q, nullptr)) return V_WGRAD_GEMM;
        if (blocked_bf16(d) && d->c % 64 == 0 && d->k % 64 == 0 && d->r * d->s <= 65535) return V_WGRAD_64;
        return V_DIRECT;
    }
    return V_INVALID;
}

// ---- NCHW tensors that no MFMA kernel reads or writes in place ----------------------------------------------
// The layout a kernel works in is the backend's choice, and the conversion at a node's boundary is the backend's job
// (Sec. 2, Sec. 4).  A bf16 node whose NCHW tensors would otherwise leave only the one-thread-per-output kernels
// (several taps, strides, images whose H*W is not a multiple of 8) runs on blocked copies in the workspace: the inputs
// are converted, the node runs with blocked tensors, the result is converted back.  Only the tensors that have to
// change are copied (the low-channel stem kernels read an NCHW x themselves).
bool fast_variant(Variant v) { return v != V_INVALID && v != V_UNSUPPORTED && v != V_DIRECT && v != V_STAGED; }

struct StagedPlan {
    ngc_conv_desc inner;       // the node as it runs
    bool cx, cy;               // x / y have a blocked copy
    size_t x_off, y_off, m_off;    // of the copies in the workspace (m: the ReLU mask of backprop-data, x-shaped)
    size_t inner_off;          // the inner node's own workspace starts here
};

bool staged_plan(const ngc_conv_desc *d, int op, StagedPlan *out)
{
    if (d->dtype != NGC_BF16) return false;
    if (env_switch(SW_STAGED) && atoi(env_switch(SW_STAGED)) == 0) return false;    // tests / benchmarks only
    const bool xn = d->x_layout == NGC_NCHW, yn = d->y_layout == NGC_NCHW;
    for (int cand = 0; cand < 3; ++cand) {
        const bool cx = cand != 0, cy = cand != 1;
        if ((cx && !xn) || (cy && !yn)) continue;
        StagedPlan sp;
        sp.inner = *d;
        if (cx) sp.inner.x_layout = NGC_NCHW16C;
        if (cy) sp.inner.y_layout = NGC_NCHW16C;
        int P, Q;
        if (validate(&sp.inner, &P, &Q) != NGC_OK) continue;
        // operands of 2 GiB or more run as groups of images: what counts is the kernel of a group
        const ngc_conv_desc g = with_batch(&sp.inner, batch_slices(&sp.inner, P, Q).images);
        if (!fast_variant(pick_base(&g, op))) continue;
        sp.cx = cx;
        sp.cy = cy;
        size_t off = 0;
        const size_t xb = round256(phys(NGC_NCHW16C, d->n, d->c, d->h, d->w) * 2);
        const size_t yb = round256(phys(NGC_NCHW16C, d->n, d->k, P, Q) * 2);
        sp.x_off = off;
        if (cx) off += xb;
        sp.y_off = off;
        if (cy) off += yb;
        sp.m_off = off;
        if (cx && op == NGC_OP_BWD_DATA) off += xb;
        sp.inner_off = off;
        if (out) *out = sp;
        return true;
    }
    return false;
}

Variant pick_uncached(const ngc_conv_desc *d, int op)
{
    const Variant v = pick_base(d, op);
    if ((v == V_DIRECT || v == V_UNSUPPORTED) && staged_plan(d, op, nullptr)) return V_STAGED;
    return v;
}

Variant pick(const ngc_conv_desc *d, int op)
{
    static thread_local PlanCache<Variant> cache;
    const PlanKey key = plan_key(d, op);
    Variant *e = cache.find(key);
    if (!e) e = &cache.put(key, pick_uncached(d, op));
    return *e;
}

size_t filter_elems(const ngc_conv_desc *d, int layout)
{
    if (layout == NGC_KCRS) return (size_t)d->k * d->c * d->r * d->s;
    if (layout == NGC_BLOCKED_FWD) return (size_t)d->r * d->s * ((d->c + 15) / 16) * d->k * 16;
    if (layout == NGC_BLOCKED_BWD) return (size_t)d->r * d->s * ((d->k + 15) / 16) * d->c * 16;
    return 0;
}

// split of the N*P*Q reduction of backprop-filters over workgroups
void wgrad_split(const ngc_conv_desc *d, int P, int Q, uint32_t *chunk, int *splits)
{
    const uint32_t M = (uint32_t)d->n * P * Q;
    const uint32_t base = (uint32_t)(d->k / 64) * (d->c / 64) * d->r * d->s;
    uint32_t want = (1024 + base - 1) / base;
    const uint32_t max_splits = (M + 63) / 64;
    if (want > max_splits) want = max_splits;
    if (want < 1) want = 1;
    uint32_t ch = (M + want - 1) / want;
    ch = (ch + 63) / 64 * 64;
    *chunk = ch;
    *splits = (int)((M + ch - 1) / ch);
}

// descriptor of "dx seen as a gradient tensor": its channel sums are what ngc_bias_grad computes for dy
ngc_conv_desc dx_as_dy(const ngc_conv_desc *d)
{
    ngc_conv_desc t = *d;
    t.k = d->c;
    t.y_layout = d->x_layout;
    return t;
}

bool db_fusable(const ngc_conv_desc *d, Variant v)
{
    if (env_switch(SW_DB_FUSE) && atoi(env_switch(SW_DB_FUSE)) == 0) return false;   // tests / benchmarks only
    if (v == V_ROWS) v = V_STRIP;                         // channel sums come from the strip kernel's launches
    if (v == V_STRIP) {                                   // the kernels with column tiles write no channel sums
        int P, Q;
        return validate(d, &P, &Q) == NGC_OK && !strip_col_tiles(d, NGC_OP_BWD_DATA, P, Q);
    }
    if (v == V_GEMM1X1) return d->x_layout == NGC_NCHW16C && d->y_layout == NGC_NCHW16C;
    return false;
}

// rows of partial channel sums the fused launches write
int db_fused_rows(const ngc_conv_desc *d, Variant v, int P, int Q)
{
    int rows = 0;
    if (v == V_ROWS) v = V_STRIP;
    if (v == V_STRIP) {
        const int ncls = strip_classes(d, NGC_OP_BWD_DATA);
        for (int c = 0; c < ncls; ++c) {
            StripParams sp;
            int nf;
            size_t lds;
            bool empty;
            if (!strip_plan_class(d, NGC_OP_BWD_DATA, c / d->stride_w, c % d->stride_w, P, Q, &sp, &nf, &lds, &empty)) return 0;
            if (!empty) rows += sp.groups * sp.strips * 8;                // one row per wave
        }
    } else if (v == V_GEMM1X1) {
        Gemm1x1Params gp;
        if (!gemm1x1_plan(d, NGC_OP_BWD_DATA, P, Q, &gp, nullptr)) return 0;
        gp.dbp = reinterpret_cast<float *>(1);
        const int bm = gemm1x1_dbp_tile_m(gp);
        rows = (int)((gp.M + bm - 1) / bm) * (bm / 64);                  // one row per MFMA wave row
    }
    return rows;
}

size_t workspace_bytes(const ngc_conv_desc *d, int op, Variant v, int P, int Q);

size_t workspace_bytes_uncached(const ngc_conv_desc *d, int op, Variant v, int P, int Q)
{
    if (v == V_STAGED) {
        // the blocked copies, then whatever the node needs when it runs on them
        StagedPlan sp;
        if (!staged_plan(d, op == NGC_OP_BWD_DATA_DB ? NGC_OP_BWD_DATA : op, &sp)) return 0;
        return sp.inner_off + ngc_conv_workspace_bytes(&sp.inner, op);
    }
    if (op == NGC_OP_BWD_DATA_DB) {
        // backprop-data part, then the partial channel sums of dx: rows of the fused launches, or the
        // partials of a second pass over dx where the kernel does not produce them
        const size_t base = workspace_bytes(d, NGC_OP_BWD_DATA, v, P, Q);
        if (db_fusable(d, v))
            return base + round256((size_t)db_fused_rows(d, v, P, Q) * ((d->c + 63) / 64 * 64) * sizeof(float));
        const ngc_conv_desc t = dx_as_dy(d);
        return base + round256((size_t)bias_grad_parts(t, d->h, d->w) * ((d->c + 15) / 16 * 16) * sizeof(float));
    }
    if (op == NGC_OP_BIAS_GRAD) return round256((size_t)bias_grad_parts(*d, P, Q) * ((d->k + 15) / 16 * 16) * sizeof(float));
    if (op == NGC_OP_FWD && (v == V_IGEMM_128 || v == V_IGEMM_64 || v == V_STRIP || v == V_ROWS || v == V_GEMM1X1))
        return d->w_layout == NGC_KCRS ? round256(filter_elems(d, NGC_BLOCKED_FWD) * 2) : 0;
    if (op == NGC_OP_BWD_DATA && (v == V_IGEMM_128 || v == V_IGEMM_64 || v == V_STRIP || v == V_ROWS || v == V_GEMM1X1))
        return d->w_layout == NGC_KCRS ? round256(filter_elems(d, NGC_BLOCKED_BWD) * 2) : 0;
    if (op == NGC_OP_BWD_DATA && v == V_STEM_BWD) {
        StemBwdPlan pl;
        stem_bwd_plan(d, P, Q, &pl);
        return round256(pl.wu_bytes);
    }
    if (op == NGC_OP_BWD_FILTERS && v == V_WGRAD_STEM) {
        WgradStemParams wp;
        wgrad_stem_plan(d, P, Q, &wp, nullptr);
        return round256((size_t)d->n * wp.strips * (d->k / 64) * 2 * 4 * 6 * 64 * 16);
    }
    if (op == NGC_OP_BWD_FILTERS && v == V_WGRAD_GEMM) {
        WgradGemmParams wp;
        wgrad_gemm_plan(d, P, Q, &wp);
        return round256((size_t)wp.nparts * d->r * d->s * wp.ktiles * wp.ctiles * wp.wk * wp.wc * 64 * 64 * sizeof(float));
    }
    if (op == NGC_OP_BWD_FILTERS && v == V_WGRAD_STRIP) {
        WgradStripParams wp;
        wgrad_strip_plan(d, P, Q, &wp, nullptr);
        return round256((size_t)wp.nparts * 9 * d->k * d->c * sizeof(float));
    }
    if (op == NGC_OP_BWD_FILTERS && v == V_WGRAD_64) {
        uint32_t chunk;
        int splits;
        wgrad_split(d, P, Q, &chunk, &splits);
        return round256((size_t)splits * d->r * d->s * d->k * d->c * sizeof(float));
    }
    return 0;
}

size_t workspace_bytes(const ngc_conv_desc *d, int op, Variant v, int P, int Q)
{
    static thread_local PlanCache<size_t> cache;
    const PlanKey key = plan_key(d, op, (int)v);
    size_t *e = cache.find(key);
    if (!e) e = &cache.put(key, workspace_bytes_uncached(d, op, v, P, Q));
    return *e;
}

// Workspace one group of a node that runs as several launches over groups of images needs: the groups reuse one
// workspace, and the split of a backprop-filters reduction is not monotone in the batch, so the last (smaller)
// group can need more than the full ones.
size_t sliced_group_workspace(const ngc_conv_desc *d, int op, const BatchSlices &bs, int P, int Q)
{
    const ngc_conv_desc g = with_batch(d, bs.images);
    size_t need = workspace_bytes(&g, op, pick(&g, op), P, Q);
    const int rem = d->n % bs.images;
    if (rem) {
        const ngc_conv_desc r = with_batch(d, rem);
        const size_t b = workspace_bytes(&r, op, pick(&r, op), P, Q);
        if (b > need) need = b;
    }
    return need;
}

int launch_status(hipError_t e)
{
    if (e == hipSuccess) return NGC_OK;
    fprintf(stderr, "ngconv: HIP launch failed: %s\n", hipGetErrorString(e));   // error path only
    return NGC_LAUNCH_FAILED;
}

void fill_class(IgemmClass &c, int oa_h, int oa_w, int OP, int OQ, int tap_begin, int tap_count, int N)
{
    c.oa_h = oa_h;
    c.oa_w = oa_w;
    c.OP = OP;
    c.OQ = OQ;
    c.tap_begin = tap_begin;
    c.tap_count = tap_count;
    c.M = (uint32_t)N * OP * OQ;
    c.div_pq = make_fastdiv((uint32_t)(OP * OQ > 0 ? OP * OQ : 1));
    c.div_q = make_fastdiv((uint32_t)(OQ > 0 ? OQ : 1));
}

}  // namespace

extern "C" {

int ngc_conv_out_shape(const ngc_conv_desc *desc, int32_t *p, int32_t *q)
{
    if (!desc || !p || !q) return NGC_BAD_ARG;
    int P, Q;
    const int st = validate(desc, &P, &Q);
    if (st != NGC_OK) return st;
    *p = P;
    *q = Q;
    return NGC_OK;
}

size_t ngc_data_elems(const ngc_conv_desc *desc, int which)
{
    int P, Q;
    if (validate(desc, &P, &Q) != NGC_OK) return 0;
    if (which == 0) return phys(desc->x_layout, desc->n, desc->c, desc->h, desc->w);
    if (which == 1) return phys(desc->y_layout, desc->n, desc->k, P, Q);
    return 0;
}

size_t ngc_filter_elems(const ngc_conv_desc *desc, int32_t layout)
{
    int P, Q;
    if (validate(desc, &P, &Q) != NGC_OK) return 0;
    return filter_elems(desc, layout);
}

// Both derivative ops of a 1x1 stride-1 node in one pass over dy (bwd1x1_fused.hip)
static bool bwd1x1_fused_plan(const ngc_conv_desc *d, int P, int Q, Bwd1x1FusedParams *fp)
{
    if (d->dtype != NGC_BF16 || d->x_layout != NGC_NCHW16C || d->y_layout != NGC_NCHW16C || d->w_layout != NGC_BLOCKED_BWD)
        return false;
    if (d->r != 1 || d->s != 1 || d->stride_h != 1 || d->stride_w != 1) return false;
    if (d->pad_below_h || d->pad_below_w || d->pad_above_h || d->pad_above_w) return false;
    if (d->c % 64 != 0 || (d->k != 64 && d->k != 128 && d->k != 256 && d->k != 512)) return false;
    const size_t hw = (size_t)P * Q, m = (size_t)d->n * hw;
    const size_t x_bytes = m * d->c * 2, dy_bytes = m * d->k * 2;
    if (x_bytes >= ((size_t)1 << 31) || dy_bytes >= ((size_t)1 << 31)) return false;
    Bwd1x1FusedParams q;
    memset(&q, 0, sizeof(q));
    q.N = d->n; q.C = d->c; q.K = d->k; q.HW = (int32_t)hw; q.M = (uint32_t)m;
    q.nstages = (int32_t)((m + 63) / 64);
    const int ctiles = d->c / 64;
    int parts = (NUM_CUS + ctiles - 1) / ctiles;
    if (parts > q.nstages) parts = q.nstages;
    q.stages_per_part = (q.nstages + parts - 1) / parts;
    q.nparts = (q.nstages + q.stages_per_part - 1) / q.stages_per_part;
    q.x_bytes = (uint32_t)x_bytes; q.dy_bytes = (uint32_t)dy_bytes;
    q.div_hw = make_fastdiv((uint32_t)hw);
    if (fp) *fp = q;
    return true;
}

size_t ngc_conv_workspace_bytes(const ngc_conv_desc *desc, int op)
{
    int P, Q;
    if (validate(desc, &P, &Q) != NGC_OK) return 0;
    if (op == NGC_OP_BWD_DATA_FILTERS) {
        Bwd1x1FusedParams fp;
        return bwd1x1_fused_plan(desc, P, Q, &fp) ? round256((size_t)fp.nparts * fp.K * fp.C * sizeof(float)) : 0;
    }
    const BatchSlices bs = batch_slices(desc, P, Q);
    if (bs.images < desc->n && op == NGC_OP_BWD_FILTERS) {
        // one dw per group of images behind the workspace of a group's launch, added up in index order at the end
        const size_t groups = (size_t)(desc->n + bs.images - 1) / bs.images;
        const size_t row = ((size_t)desc->k * desc->c * desc->r * desc->s + 15) / 16 * 16;
        return round256(sliced_group_workspace(desc, op, bs, P, Q)) + round256(groups * row * sizeof(float));
    }
    if (bs.images < desc->n && (op == NGC_OP_FWD || op == NGC_OP_BWD_DATA || op == NGC_OP_BWD_DATA_DB)) {
        // the launches of the groups reuse one workspace; the channel sums come from a second pass over the whole dx
        const int gop = op == NGC_OP_FWD ? NGC_OP_FWD : NGC_OP_BWD_DATA;
        const size_t base = sliced_group_workspace(desc, gop, bs, P, Q);
        if (op != NGC_OP_BWD_DATA_DB) return base;
        const ngc_conv_desc t = dx_as_dy(desc);
        return base + round256((size_t)bias_grad_parts(t, desc->h, desc->w) * ((desc->c + 15) / 16 * 16) * sizeof(float));
    }
    return workspace_bytes(desc, op, pick(desc, op == NGC_OP_BWD_DATA_DB ? NGC_OP_BWD_DATA : op), P, Q);
}

const char *ngc_conv_variant(const ngc_conv_desc *desc, int op)
{
    if (op == NGC_OP_BWD_DATA_FILTERS) {
        int P, Q;
        if (validate(desc, &P, &Q) != NGC_OK) return "invalid";
        return bwd1x1_fused_plan(desc, P, Q, nullptr) ? "bwd1x1_fused_bf16" : "unsupported";
    }
    if (op == NGC_OP_BIAS_GRAD) {
        int P, Q;
        if (validate(desc, &P, &Q) != NGC_OK) return "invalid";
        return (desc->dtype == NGC_BF16 && desc->y_layout == NGC_NCHW16C) ? "bias_grad_blocked_bf16" : "bias_grad_generic";
    }
    {
        int P, Q;
        if (validate(desc, &P, &Q) == NGC_OK &&
            (op == NGC_OP_FWD || op == NGC_OP_BWD_DATA || op == NGC_OP_BWD_DATA_DB || op == NGC_OP_BWD_FILTERS)) {
            const BatchSlices bs = batch_slices(desc, P, Q);
            if (bs.images < desc->n) {                       // groups of images: the kernel of a group
                static thread_local char name[64];
                const ngc_conv_desc g = with_batch(desc, bs.images);
                snprintf(name, sizeof(name), "sliced:%s", ngc_conv_variant(&g, op));
                return name;
            }
        }
    }
    switch (pick(desc, op == NGC_OP_BWD_DATA_DB ? NGC_OP_BWD_DATA : op)) {
    case V_UNSUPPORTED: return "unsupported";
    case V_DIRECT: return "direct";
    case V_IGEMM_128: return "igemm_bf16_128x128";
    case V_IGEMM_64: return "igemm_bf16_256x64";
    case V_WGRAD_64: return "wgrad_bf16_64x64";
    case V_STRIP: return "strip_bf16";
    case V_ROWS: return "strip_rows_bf16";
    case V_WGRAD_STRIP: return "wgrad_strip_bf16";
    case V_STEM_FWD: return "stem_fwd_bf16";
    case V_WGRAD_STEM: return "wgrad_stem_bf16";
    case V_STEM_BWD: return "stem_bwd_strip_bf16";
    case V_WGRAD_GEMM: return "wgrad_gemm_bf16";
    case V_GEMM1X1: return "gemm1x1_bf16";
    case V_STAGED: {                                         // blocked copies in the workspace: the kernel that runs on them
        static thread_local char name[64];
        StagedPlan sp;
        if (!staged_plan(desc, op == NGC_OP_BWD_DATA_DB ? NGC_OP_BWD_DATA : op, &sp)) return "invalid";
        snprintf(name, sizeof(name), "staged:%s", ngc_conv_variant(&sp.inner, op));
        return name;
    }
    default: return "invalid";
    }
}

const char *ngc_status_string(int status)
{
    switch (status) {
    case NGC_OK: return "ok";
    case NGC_BAD_ARG: return "bad argument (null pointer, misaligned pointer, bad enum or flag)";
    case NGC_BAD_SHAPE: return "bad shape or attribute (non-positive dim, stride/dilation < 1, negative pad, empty output, tensor too large)";
    case NGC_UNSUPPORTED: return "no kernel for this element type / layout combination";
    case NGC_WORKSPACE_TOO_SMALL: return "workspace too small or missing";
    case NGC_LAUNCH_FAILED: return "HIP launch failed";
    case NGC_SCRATCH_EXCEEDED: return "the node needs more scratch memory than the library's static array holds (use the entry point with a workspace)";
    default: return "unknown status";
    }
}

int ngc_conv_fwd(const ngc_conv_desc *desc, const void *x, const void *w, const float *bias, void *y, void *ws,
                 size_t ws_bytes, void *hip_stream)
{
    int P, Q;
    const int vs = validate(desc, &P, &Q);
    if (vs != NGC_OK) return vs;
    if (!x || !w || !y) return NGC_BAD_ARG;
    if ((desc->epilogue & NGC_EPI_BIAS) && !bias) return NGC_BAD_ARG;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y) || !aligned16(bias) || !aligned16(ws)) return NGC_BAD_ARG;
    const BatchSlices bs = batch_slices(desc, P, Q);
    if (bs.images < desc->n) {                                // operands of 2 GiB or more: one launch per group of images
        for (int n0 = 0; n0 < desc->n; n0 += bs.images) {
            const ngc_conv_desc g = with_batch(desc, desc->n - n0 < bs.images ? desc->n - n0 : bs.images);
            const int rc = ngc_conv_fwd(&g, static_cast<const unsigned char *>(x) + (size_t)n0 * bs.x_bytes, w, bias,
                                        static_cast<unsigned char *>(y) + (size_t)n0 * bs.y_bytes, ws, ws_bytes, hip_stream);
            if (rc != NGC_OK) return rc;
        }
        return NGC_OK;
    }
    const Variant v = pick(desc, NGC_OP_FWD);
    if (v == V_UNSUPPORTED) return NGC_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (v == V_STAGED) {
        StagedPlan sp;
        if (!staged_plan(desc, NGC_OP_FWD, &sp)) return NGC_UNSUPPORTED;
        if (!ws || ws_bytes < workspace_bytes(desc, NGC_OP_FWD, v, P, Q)) return NGC_WORKSPACE_TOO_SMALL;
        unsigned char *base = static_cast<unsigned char *>(ws);
        const void *xin = x;
        void *yout = y;
        if (sp.cx) {
            const hipError_t e = launch_layout_convert(2, desc->n, desc->c, desc->h, desc->w, x, NGC_NCHW, base + sp.x_off, NGC_NCHW16C, st);
            if (e != hipSuccess) return launch_status(e);
            xin = base + sp.x_off;
        }
        if (sp.cy) yout = base + sp.y_off;
        const int rc = ngc_conv_fwd(&sp.inner, xin, w, bias, yout, base + sp.inner_off, ws_bytes - sp.inner_off, hip_stream);
        if (rc != NGC_OK || !sp.cy) return rc;
        return launch_status(launch_layout_convert(2, desc->n, desc->k, P, Q, yout, NGC_NCHW16C, y, NGC_NCHW, st));
    }
    if (v == V_DIRECT)
        return launch_status(launch_direct_fwd(*desc, P, Q, x, w, (desc->epilogue & NGC_EPI_BIAS) ? bias : nullptr, y, st));
    if (v == V_STEM_FWD) {
        StemFwdParams sp;
        size_t lds;
        if (!stem_fwd_plan(desc, P, Q, &sp, &lds)) return NGC_UNSUPPORTED;
        sp.x = static_cast<const uint16_t *>(x);
        sp.w = static_cast<const uint16_t *>(w);
        sp.bias = (desc->epilogue & NGC_EPI_BIAS) ? bias : nullptr;
        sp.y = static_cast<uint16_t *>(y);
        sp.relu = (desc->epilogue & NGC_EPI_RELU) ? 1 : 0;
        return launch_status(launch_stem_fwd(sp, lds, st));
    }

    const size_t need = workspace_bytes(desc, NGC_OP_FWD, v, P, Q);
    if (need > 0 && (!ws || ws_bytes < need)) return NGC_WORKSPACE_TOO_SMALL;
    const void *wt = w;
    if (desc->w_layout == NGC_KCRS) {
        const hipError_t e = launch_filter_convert(2, desc->k, desc->c, desc->r, desc->s, w, ws, NGC_BLOCKED_FWD, st);
        if (e != hipSuccess) return NGC_LAUNCH_FAILED;
        wt = ws;
    }
    if (v == V_ROWS) {
        RowsParams rp;
        size_t lds;
        if (!rows_plan(desc, NGC_OP_FWD, P, Q, &rp, &lds)) return NGC_UNSUPPORTED;
        rp.in = static_cast<const uint16_t *>(x);
        rp.wt = static_cast<const uint16_t *>(wt);
        rp.out = static_cast<uint16_t *>(y);
        rp.bias = (desc->epilogue & NGC_EPI_BIAS) ? bias : nullptr;
        rp.relu = (desc->epilogue & NGC_EPI_RELU) ? 1 : 0;
        return launch_status(launch_rows(rp, lds, st));
    }
    if (v == V_STRIP) {
        StripParams sp;
        int nf;
        size_t lds;
        if (!strip_plan_class(desc, NGC_OP_FWD, 0, 0, P, Q, &sp, &nf, &lds, nullptr)) return NGC_UNSUPPORTED;
        sp.in = static_cast<const uint16_t *>(x);
        sp.wt = static_cast<const uint16_t *>(wt);
        sp.out = static_cast<uint16_t *>(y);
        sp.bias = (desc->epilogue & NGC_EPI_BIAS) ? bias : nullptr;
        sp.relu = (desc->epilogue & NGC_EPI_RELU) ? 1 : 0;
        return launch_status(launch_strip(sp, nf, lds, st));
    }
    if (v == V_GEMM1X1) {
        Gemm1x1Params gp;
        if (!gemm1x1_plan(desc, NGC_OP_FWD, P, Q, &gp, nullptr)) return NGC_UNSUPPORTED;
        gp.in = static_cast<const uint16_t *>(x);
        gp.wt = static_cast<const uint16_t *>(wt);
        gp.out = static_cast<uint16_t *>(y);
        gp.bias = (desc->epilogue & NGC_EPI_BIAS) ? bias : nullptr;
        gp.relu = (desc->epilogue & NGC_EPI_RELU) ? 1 : 0;
        return launch_status(launch_gemm1x1(gp, st));
    }
    IgemmParams p;
    memset(&p, 0, sizeof(p));
    p.in = static_cast<const uint16_t *>(x);
    p.wt = static_cast<const uint16_t *>(wt);
    p.out = static_cast<uint16_t *>(y);
    p.bias = (desc->epilogue & NGC_EPI_BIAS) ? bias : nullptr;
    p.N = desc->n; p.Cin = desc->c; p.Hin = desc->h; p.Win = desc->w;
    p.Cout = desc->k; p.Hout = P; p.Wout = Q;
    p.os_h = p.os_w = 1;
    p.is_h = desc->stride_h; p.is_w = desc->stride_w;
    p.relu = (desc->epilogue & NGC_EPI_RELU) ? 1 : 0;
    p.ncls = 1;
    int t = 0;
    for (int r = 0; r < desc->r; ++r)
        for (int s = 0; s < desc->s; ++s) {
            p.taps[t].dh = r * desc->dil_h - desc->pad_below_h;
            p.taps[t].dw = s * desc->dil_w - desc->pad_below_w;
            p.taps[t].slab = r * desc->s + s;
            ++t;
        }
    fill_class(p.cls[0], 0, 0, P, Q, 0, t, desc->n);
    return launch_status(launch_igemm(p, v == V_IGEMM_128 ? 128 : 64, p.cls[0].M, st));
}

}  // extern "C"

namespace {

// Channel sums of dx (the bias gradient of the layer that produced the data input) from the backprop-data
// launches themselves: the strip and 1x1 GEMM kernels with blocked dx write one row of per-channel partial
// sums per workgroup; `rows` counts them.
struct DbFuse {
    float *partial;            // [rows][ld] fp32
    int ld;                    // C rounded up to 64
    int rows;                  // rows written by the launches (out)
};

// ConvolutionBackpropData; mask (may be null): same shape / layout / type as dx, dx = (mask > 0) ? dx : 0;
// fuse (may be null): also write the partial channel sums of dx
int bwd_data_core(const ngc_conv_desc *desc, const void *dy, const void *w, const void *mask, void *dx, void *ws,
                  size_t ws_bytes, void *hip_stream, DbFuse *fuse)
{
    int P, Q;
    const int vs = validate(desc, &P, &Q);
    if (vs != NGC_OK) return vs;
    if (!dy || !w || !dx) return NGC_BAD_ARG;
    if (!aligned16(dy) || !aligned16(w) || !aligned16(dx) || !aligned16(ws) || !aligned16(mask)) return NGC_BAD_ARG;
    Variant v = pick(desc, NGC_OP_BWD_DATA);
    if (v == V_UNSUPPORTED || v == V_STAGED) return NGC_UNSUPPORTED;    // blocked copies are the caller's part
    if (v == V_ROWS && fuse) v = V_STRIP;                  // the channel sums of dx come from the strip kernel
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (v == V_DIRECT) return launch_status(launch_direct_bwd_data(*desc, P, Q, dy, w, mask, dx, st));
    if (v == V_STEM_BWD) {
        StemBwdPlan pl;
        if (!stem_bwd_plan(desc, P, Q, &pl)) return NGC_UNSUPPORTED;
        if (!ws || ws_bytes < round256(pl.wu_bytes)) return NGC_WORKSPACE_TOO_SMALL;
        hipError_t e = launch_subpixel_filter(desc->k, desc->c, desc->r, desc->s, desc->pad_below_h, desc->pad_below_w,
                                              pl.dr_min, pl.ndr, pl.ds_min, pl.nds, pl.BH, pl.BW, 2, 2,
                                              static_cast<const uint16_t *>(w),
                                              static_cast<uint16_t *>(ws), st);
        if (e != hipSuccess) return launch_status(e);
        pl.sp.in = static_cast<const uint16_t *>(dy);
        pl.sp.wt = static_cast<const uint16_t *>(ws);
        pl.sp.out = static_cast<uint16_t *>(dx);
        pl.sp.mask = static_cast<const uint16_t *>(mask);
        pl.sp.bias = nullptr;
        pl.sp.relu = 0;
        return launch_status(launch_strip(pl.sp, pl.nf, pl.lds, st));
    }

    const size_t need = workspace_bytes(desc, NGC_OP_BWD_DATA, v, P, Q);
    if (need > 0 && (!ws || ws_bytes < need)) return NGC_WORKSPACE_TOO_SMALL;
    const void *wt = w;
    if (desc->w_layout == NGC_KCRS) {
        const hipError_t e = launch_filter_convert(2, desc->k, desc->c, desc->r, desc->s, w, ws, NGC_BLOCKED_BWD, st);
        if (e != hipSuccess) return NGC_LAUNCH_FAILED;
        wt = ws;
    }
    if (v == V_ROWS) {
        RowsParams rp;
        size_t lds;
        if (!rows_plan(desc, NGC_OP_BWD_DATA, P, Q, &rp, &lds)) return NGC_UNSUPPORTED;
        rp.in = static_cast<const uint16_t *>(dy);
        rp.wt = static_cast<const uint16_t *>(wt);
        rp.out = static_cast<uint16_t *>(dx);
        rp.mask = static_cast<const uint16_t *>(mask);
        return launch_status(launch_rows(rp, lds, st));
    }
    if (v == V_STRIP) {
        if (strip_zero_fill(desc)) {
            const hipError_t e = launch_zero_fill(dx, (size_t)desc->n * desc->c * desc->h * desc->w * 2, st);
            if (e != hipSuccess) return launch_status(e);
        }
        const int ncls = strip_classes(desc, NGC_OP_BWD_DATA);
        // the residue classes of the stride: one launch each, or (up to 4 classes, 8-wave kernels) all in one grid
        const bool merge = !(env_switch(SW_STRIP_MERGE) && atoi(env_switch(SW_STRIP_MERGE)) == 0);
        StripMulti mp;
        mp.n = 0;
        int nf_max = 0;
        size_t lds_max = 0;
        const bool col_tiles = strip_col_tiles(desc, NGC_OP_BWD_DATA, P, Q);    // then one launch per class
        for (int c = 0; c < ncls; ++c) {
            StripParams sp;
            int nf;
            size_t lds;
            bool empty;
            if (!strip_plan_class(desc, NGC_OP_BWD_DATA, c / desc->stride_w, c % desc->stride_w, P, Q, &sp, &nf, &lds, &empty))
                return NGC_UNSUPPORTED;
            if (empty) continue;
            sp.in = static_cast<const uint16_t *>(dy);
            sp.wt = static_cast<const uint16_t *>(wt);
            sp.out = static_cast<uint16_t *>(dx);
            sp.mask = static_cast<const uint16_t *>(mask);
            sp.bias = nullptr;
            sp.relu = 0;
            if (fuse) {
                sp.dbp = fuse->partial;
                sp.dbp_row0 = fuse->rows / 8;                            // the kernel writes rows (row0 + workgroup) * 8 + wave
                sp.dbp_ld = fuse->ld;
                fuse->rows += sp.groups * sp.strips * 8;
            }
            if (merge && ncls > 1 && ncls <= STRIP_MULTI_MAX && !col_tiles) {
                mp.c[mp.n] = sp;
                mp.wg_end[mp.n] = (mp.n ? mp.wg_end[mp.n - 1] : 0) + sp.groups * sp.strips;
                ++mp.n;
                if (nf > nf_max) nf_max = nf;
                if (lds > lds_max) lds_max = lds;
                continue;
            }
            const int rc = launch_status(launch_strip(sp, nf, lds, st));
            if (rc != NGC_OK) return rc;
        }
        if (mp.n == 1) return launch_status(launch_strip(mp.c[0], nf_max, lds_max, st));
        if (mp.n > 1) return launch_status(launch_strip_multi(mp, nf_max, lds_max, st));
        return NGC_OK;
    }
    if (v == V_GEMM1X1) {
        Gemm1x1Params gp;
        bool zero;
        if (!gemm1x1_plan(desc, NGC_OP_BWD_DATA, P, Q, &gp, &zero)) return NGC_UNSUPPORTED;
        if (zero) {
            const hipError_t e = launch_zero_fill(dx, (size_t)desc->n * desc->c * desc->h * desc->w * 2, st);
            if (e != hipSuccess) return launch_status(e);
        }
        if (gp.M == 0) return NGC_OK;
        gp.in = static_cast<const uint16_t *>(dy);
        gp.wt = static_cast<const uint16_t *>(wt);
        gp.out = static_cast<uint16_t *>(dx);
        gp.mask = static_cast<const uint16_t *>(mask);
        if (fuse) {
            gp.dbp = fuse->partial;
            gp.dbp_row0 = 0;
            gp.dbp_ld = fuse->ld;
            const int bm = gemm1x1_dbp_tile_m(gp);
            fuse->rows = (int)((gp.M + bm - 1) / bm) * (bm / 64);
        }
        return launch_status(launch_gemm1x1(gp, st));
    }
    IgemmParams p;
    memset(&p, 0, sizeof(p));
    p.in = static_cast<const uint16_t *>(dy);
    p.wt = static_cast<const uint16_t *>(wt);
    p.out = static_cast<uint16_t *>(dx);
    p.mask = static_cast<const uint16_t *>(mask);
    p.bias = nullptr;
    p.N = desc->n; p.Cin = desc->k; p.Hin = P; p.Win = Q;
    p.Cout = desc->c; p.Hout = desc->h; p.Wout = desc->w;
    p.os_h = desc->stride_h; p.os_w = desc->stride_w;
    p.is_h = p.is_w = 1;
    p.relu = 0;
    const int sh = desc->stride_h, sw = desc->stride_w;
    p.ncls = sh * sw;
    int t = 0;
    uint32_t max_m = 0;
    for (int a = 0; a < sh; ++a)
        for (int b = 0; b < sw; ++b) {
            const int begin = t;
            for (int r = 0; r < desc->r; ++r) {
                const int vh = a + desc->pad_below_h - r * desc->dil_h;
                if (((vh % sh) + sh) % sh != 0) continue;
                for (int s = 0; s < desc->s; ++s) {
                    const int vw = b + desc->pad_below_w - s * desc->dil_w;
                    if (((vw % sw) + sw) % sw != 0) continue;
                    p.taps[t].dh = vh / sh;              // exact
                    p.taps[t].dw = vw / sw;
                    p.taps[t].slab = r * desc->s + s;
                    ++t;
                }
            }
            const int OPc = a < desc->h ? (desc->h - a + sh - 1) / sh : 0;
            const int OQc = b < desc->w ? (desc->w - b + sw - 1) / sw : 0;
            IgemmClass &c = p.cls[a * sw + b];
            fill_class(c, a, b, OPc, OQc, begin, t - begin, desc->n);
            if (OPc == 0 || OQc == 0) c.M = 0;
            if (c.M > max_m) max_m = c.M;
        }
    return launch_status(launch_igemm(p, v == V_IGEMM_128 ? 128 : 64, max_m, st));
}

// db (may be null): [C] fp32 channel sums of the dx written; the workspace then holds the partial sums behind
// the backprop-data part
int bwd_data_impl(const ngc_conv_desc *desc, const void *dy, const void *w, const void *mask, void *dx, float *db, void *ws,
                  size_t ws_bytes, void *hip_stream)
{
    int P, Q;
    const int vs = validate(desc, &P, &Q);
    if (vs != NGC_OK) return vs;
    const BatchSlices bs = batch_slices(desc, P, Q);
    if (bs.images < desc->n) {                                // operands of 2 GiB or more: one launch per group of images
        if (!dy || !w || !dx) return NGC_BAD_ARG;
        if (!aligned16(db) || !aligned16(ws)) return NGC_BAD_ARG;
        if (db && (size_t)desc->n * desc->h * desc->w >= 0xFFFF0000ull) return NGC_BAD_SHAPE;
        const size_t base = ngc_conv_workspace_bytes(desc, NGC_OP_BWD_DATA);
        const size_t need = db ? ngc_conv_workspace_bytes(desc, NGC_OP_BWD_DATA_DB) : base;
        if (need > 0 && (!ws || ws_bytes < need)) return NGC_WORKSPACE_TOO_SMALL;
        for (int n0 = 0; n0 < desc->n; n0 += bs.images) {
            const ngc_conv_desc g = with_batch(desc, desc->n - n0 < bs.images ? desc->n - n0 : bs.images);
            const size_t xo = (size_t)n0 * bs.x_bytes, yo = (size_t)n0 * bs.y_bytes;
            const int rc = bwd_data_core(&g, static_cast<const unsigned char *>(dy) + yo, w,
                                         mask ? static_cast<const unsigned char *>(mask) + xo : nullptr,
                                         static_cast<unsigned char *>(dx) + xo, ws, base, hip_stream, nullptr);
            if (rc != NGC_OK) return rc;
        }
        if (!db) return NGC_OK;
        const ngc_conv_desc t = dx_as_dy(desc);               // channel sums: a pass over the whole dx
        float *partial = reinterpret_cast<float *>(static_cast<unsigned char *>(ws) + base);
        return launch_status(launch_bias_grad(t, desc->h, desc->w, dx, db, partial, bias_grad_parts(t, desc->h, desc->w),
                                              static_cast<hipStream_t>(hip_stream)));
    }
    if (pick(desc, NGC_OP_BWD_DATA) == V_STAGED) {
        if (!dy || !w || !dx) return NGC_BAD_ARG;
        if (!aligned16(dy) || !aligned16(w) || !aligned16(dx) || !aligned16(ws) || !aligned16(mask) || !aligned16(db)) return NGC_BAD_ARG;
        StagedPlan sp;
        if (!staged_plan(desc, NGC_OP_BWD_DATA, &sp)) return NGC_UNSUPPORTED;
        if (!ws || ws_bytes < workspace_bytes(desc, db ? NGC_OP_BWD_DATA_DB : NGC_OP_BWD_DATA, V_STAGED, P, Q)) return NGC_WORKSPACE_TOO_SMALL;
        hipStream_t st = static_cast<hipStream_t>(hip_stream);
        unsigned char *base = static_cast<unsigned char *>(ws);
        const void *dyin = dy, *min = mask;
        void *dxout = dx;
        if (sp.cy) {
            const hipError_t e = launch_layout_convert(2, desc->n, desc->k, P, Q, dy, NGC_NCHW, base + sp.y_off, NGC_NCHW16C, st);
            if (e != hipSuccess) return launch_status(e);
            dyin = base + sp.y_off;
        }
        if (sp.cx && mask) {
            const hipError_t e = launch_layout_convert(2, desc->n, desc->c, desc->h, desc->w, mask, NGC_NCHW, base + sp.m_off, NGC_NCHW16C, st);
            if (e != hipSuccess) return launch_status(e);
            min = base + sp.m_off;
        }
        if (sp.cx) dxout = base + sp.x_off;
        const int rc = bwd_data_impl(&sp.inner, dyin, w, min, dxout, db, base + sp.inner_off, ws_bytes - sp.inner_off, hip_stream);
        if (rc != NGC_OK || !sp.cx) return rc;
        return launch_status(launch_layout_convert(2, desc->n, desc->c, desc->h, desc->w, dxout, NGC_NCHW16C, dx, NGC_NCHW, st));
    }
    if (!db) return bwd_data_core(desc, dy, w, mask, dx, ws, ws_bytes, hip_stream, nullptr);
    if (!aligned16(db) || !aligned16(ws)) return NGC_BAD_ARG;
    if ((size_t)desc->n * desc->h * desc->w >= 0xFFFF0000ull) return NGC_BAD_SHAPE;
    const Variant v = pick(desc, NGC_OP_BWD_DATA);
    if (v == V_UNSUPPORTED) return NGC_UNSUPPORTED;
    const size_t base = workspace_bytes(desc, NGC_OP_BWD_DATA, v, P, Q);
    const size_t need = workspace_bytes(desc, NGC_OP_BWD_DATA_DB, v, P, Q);     // 0 if no class of a strided layer launches
    if (need > 0 && (!ws || ws_bytes < need)) return NGC_WORKSPACE_TOO_SMALL;
    float *partial = reinterpret_cast<float *>(static_cast<unsigned char *>(ws) + base);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (db_fusable(desc, v)) {
        DbFuse f{partial, (desc->c + 63) / 64 * 64, 0};
        const int rc = bwd_data_core(desc, dy, w, mask, dx, ws, base, hip_stream, &f);
        if (rc != NGC_OK) return rc;
        return launch_status(launch_bias_grad_reduce(partial, db, f.rows, desc->c, f.ld, st));
    }
    const int rc = bwd_data_core(desc, dy, w, mask, dx, ws, base, hip_stream, nullptr);
    if (rc != NGC_OK) return rc;
    const ngc_conv_desc t = dx_as_dy(desc);                 // second pass over dx
    return launch_status(launch_bias_grad(t, desc->h, desc->w, dx, db, partial, bias_grad_parts(t, desc->h, desc->w), st));
}

}  // namespace

extern "C" {

int ngc_conv_bwd_data(const ngc_conv_desc *desc, const void *dy, const void *w, void *dx, void *ws, size_t ws_bytes,
                      void *hip_stream)
{
    return bwd_data_impl(desc, dy, w, nullptr, dx, nullptr, ws, ws_bytes, hip_stream);
}

int ngc_conv_bwd_data_relu_db(const ngc_conv_desc *desc, const void *dy, const void *w, const void *x_in, void *dx, float *db,
                              void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!x_in || !db) return NGC_BAD_ARG;
    return bwd_data_impl(desc, dy, w, x_in, dx, db, ws, ws_bytes, hip_stream);
}

int ngc_conv_bwd_data_relu(const ngc_conv_desc *desc, const void *dy, const void *w, const void *x_in, void *dx, void *ws,
                           size_t ws_bytes, void *hip_stream)
{
    if (!x_in) return NGC_BAD_ARG;
    return bwd_data_impl(desc, dy, w, x_in, dx, nullptr, ws, ws_bytes, hip_stream);
}

int ngc_bias_grad(const ngc_conv_desc *desc, const void *dy, float *db, void *ws, size_t ws_bytes, void *hip_stream)
{
    int P, Q;
    const int vs = validate(desc, &P, &Q);
    if (vs != NGC_OK) return vs;
    if (!dy || !db || !ws) return dy && db ? NGC_WORKSPACE_TOO_SMALL : NGC_BAD_ARG;
    if (!aligned16(dy) || !aligned16(db) || !aligned16(ws)) return NGC_BAD_ARG;
    if ((size_t)desc->n * P * Q >= 0xFFFF0000ull) return NGC_BAD_SHAPE;
    const int nparts = bias_grad_parts(*desc, P, Q);
    if (ws_bytes < workspace_bytes(desc, NGC_OP_BIAS_GRAD, V_DIRECT, P, Q)) return NGC_WORKSPACE_TOO_SMALL;
    return launch_status(launch_bias_grad(*desc, P, Q, dy, db, static_cast<float *>(ws), nparts,
                                          static_cast<hipStream_t>(hip_stream)));
}

}  // extern "C"

namespace {

int softmax_impl(int32_t dtype, int64_t rows, int32_t cols, bool bwd, const void *a, const void *b, void *out, void *hip_stream)
{
    if (dtype != NGC_F32 && dtype != NGC_BF16) return NGC_BAD_ARG;
    if (rows < 1 || cols < 1 || rows > 0x7fffffffll || (unsigned long long)rows * (unsigned long long)cols >= (1ull << 40))
        return NGC_BAD_SHAPE;
    if (!a || !out || (bwd && !b)) return NGC_BAD_ARG;
    const uintptr_t esz = dtype == NGC_BF16 ? 2 : 4;
    const uintptr_t all = reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(out) | (bwd ? reinterpret_cast<uintptr_t>(b) : 0);
    if (all & (esz - 1)) return NGC_BAD_ARG;
    const int V = softmax_vectors(dtype, cols, bwd, (all & 15) == 0);
    return launch_status(launch_softmax(dtype, bwd, a, b, out, (uint32_t)rows, cols, V, static_cast<hipStream_t>(hip_stream)));
}

}  // namespace

extern "C" {

int ngc_softmax(int32_t dtype, int64_t rows, int32_t cols, const void *x, void *y, void *hip_stream)
{
    return softmax_impl(dtype, rows, cols, false, x, nullptr, y, hip_stream);
}

int ngc_softmax_bwd(int32_t dtype, int64_t rows, int32_t cols, const void *y, const void *dy, void *dx, void *hip_stream)
{
    return softmax_impl(dtype, rows, cols, true, y, dy, dx, hip_stream);
}

const char *ngc_softmax_variant(int32_t dtype, int32_t cols, int32_t bwd)
{
    if ((dtype != NGC_F32 && dtype != NGC_BF16) || cols < 1) return "invalid";
    const int v = softmax_vectors(dtype, cols, bwd != 0, true);
    return v == 0 ? "softmax_rows_block" : v > 256 ? "softmax_rows_wg" : "softmax_rows_wave";
}

static int bwd_data_filters_core(const ngc_conv_desc *desc, const void *x, const void *dy, const void *w, void *dx, float *dw,
                                 void *ws, size_t ws_bytes, void *hip_stream, int relu_mask)
{
    int P, Q;
    const int vs = validate(desc, &P, &Q);
    if (vs != NGC_OK) return vs;
    if (!x || !dy || !w || !dx || !dw) return NGC_BAD_ARG;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(w) || !aligned16(dx) || !aligned16(dw) || !aligned16(ws)) return NGC_BAD_ARG;
    Bwd1x1FusedParams fp;
    if (!bwd1x1_fused_plan(desc, P, Q, &fp)) return NGC_UNSUPPORTED;
    if (!ws || ws_bytes < round256((size_t)fp.nparts * fp.K * fp.C * sizeof(float))) return NGC_WORKSPACE_TOO_SMALL;
    fp.x = static_cast<const uint16_t *>(x);
    fp.dy = static_cast<const uint16_t *>(dy);
    fp.w = static_cast<const uint16_t *>(w);
    fp.dx = static_cast<uint16_t *>(dx);
    fp.partial = static_cast<float *>(ws);
    fp.dw = dw;
    fp.relu_mask = relu_mask;
    return launch_status(launch_bwd1x1_fused(fp, static_cast<hipStream_t>(hip_stream)));
}

int ngc_conv_bwd_data_filters(const ngc_conv_desc *desc, const void *x, const void *dy, const void *w, void *dx, float *dw,
                              void *ws, size_t ws_bytes, void *hip_stream)
{
    return bwd_data_filters_core(desc, x, dy, w, dx, dw, ws, ws_bytes, hip_stream, 0);
}

int ngc_conv_bwd_data_filters_relu(const ngc_conv_desc *desc, const void *x, const void *dy, const void *w, void *dx, float *dw,
                                   void *ws, size_t ws_bytes, void *hip_stream)
{
    return bwd_data_filters_core(desc, x, dy, w, dx, dw, ws, ws_bytes, hip_stream, 1);
}

int ngc_conv_bwd_filters(const ngc_conv_desc *desc, const void *x, const void *dy, float *dw, void *ws,
                         size_t ws_bytes, void *hip_stream)
{
    int P, Q;
    const int vs = validate(desc, &P, &Q);
    if (vs != NGC_OK) return vs;
    if (!x || !dy || !dw) return NGC_BAD_ARG;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(dw) || !aligned16(ws)) return NGC_BAD_ARG;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const BatchSlices bs = batch_slices(desc, P, Q);
    if (bs.images < desc->n) {
        // operands of 2 GiB or more: dw of each group of images into the workspace, then their sum in index order
        const size_t base = round256(sliced_group_workspace(desc, NGC_OP_BWD_FILTERS, bs, P, Q));
        if (!ws || ws_bytes < ngc_conv_workspace_bytes(desc, NGC_OP_BWD_FILTERS)) return NGC_WORKSPACE_TOO_SMALL;
        const int elems = desc->k * desc->c * desc->r * desc->s, row = (elems + 15) / 16 * 16;
        float *rows = reinterpret_cast<float *>(static_cast<unsigned char *>(ws) + base);
        int groups = 0;
        for (int n0 = 0; n0 < desc->n; n0 += bs.images, ++groups) {
            const ngc_conv_desc g = with_batch(desc, desc->n - n0 < bs.images ? desc->n - n0 : bs.images);
            const int rc = ngc_conv_bwd_filters(&g, static_cast<const unsigned char *>(x) + (size_t)n0 * bs.x_bytes,
                                                static_cast<const unsigned char *>(dy) + (size_t)n0 * bs.y_bytes,
                                                rows + (size_t)groups * row, ws, base, hip_stream);
            if (rc != NGC_OK) return rc;
        }
        return launch_status(launch_bias_grad_reduce(rows, dw, groups, elems, row, st));
    }
    const Variant v = pick(desc, NGC_OP_BWD_FILTERS);
    if (v == V_DIRECT) return launch_status(launch_direct_bwd_filters(*desc, P, Q, x, dy, dw, st));
    if (v == V_STAGED) {
        StagedPlan sp;
        if (!staged_plan(desc, NGC_OP_BWD_FILTERS, &sp)) return NGC_UNSUPPORTED;
        if (!ws || ws_bytes < workspace_bytes(desc, NGC_OP_BWD_FILTERS, v, P, Q)) return NGC_WORKSPACE_TOO_SMALL;
        unsigned char *base = static_cast<unsigned char *>(ws);
        const void *xin = x, *dyin = dy;
        if (sp.cx) {
            const hipError_t e = launch_layout_convert(2, desc->n, desc->c, desc->h, desc->w, x, NGC_NCHW, base + sp.x_off, NGC_NCHW16C, st);
            if (e != hipSuccess) return launch_status(e);
            xin = base + sp.x_off;
        }
        if (sp.cy) {
            const hipError_t e = launch_layout_convert(2, desc->n, desc->k, P, Q, dy, NGC_NCHW, base + sp.y_off, NGC_NCHW16C, st);
            if (e != hipSuccess) return launch_status(e);
            dyin = base + sp.y_off;
        }
        return ngc_conv_bwd_filters(&sp.inner, xin, dyin, dw, base + sp.inner_off, ws_bytes - sp.inner_off, hip_stream);
    }

    const size_t need = workspace_bytes(desc, NGC_OP_BWD_FILTERS, v, P, Q);
    if (!ws || ws_bytes < need) return NGC_WORKSPACE_TOO_SMALL;
    if (v == V_WGRAD_GEMM) {
        WgradGemmParams wp;
        if (!wgrad_gemm_plan(desc, P, Q, &wp)) return NGC_UNSUPPORTED;
        wp.x = static_cast<const uint16_t *>(x);
        wp.dy = static_cast<const uint16_t *>(dy);
        wp.partial = static_cast<float *>(ws);
        wp.dw = dw;
        return launch_status(launch_wgrad_gemm(wp, st));
    }
    if (v == V_WGRAD_STEM) {
        WgradStemParams wp;
        size_t lds;
        if (!wgrad_stem_plan(desc, P, Q, &wp, &lds)) return NGC_UNSUPPORTED;
        wp.x = static_cast<const uint16_t *>(x);
        wp.dy = static_cast<const uint16_t *>(dy);
        wp.partial = static_cast<float *>(ws);
        wp.dw = dw;
        return launch_status(launch_wgrad_stem(wp, lds, st));
    }
    if (v == V_WGRAD_STRIP) {
        WgradStripParams wp;
        size_t lds;
        if (!wgrad_strip_plan(desc, P, Q, &wp, &lds)) return NGC_UNSUPPORTED;
        wp.x = static_cast<const uint16_t *>(x);
        wp.dy = static_cast<const uint16_t *>(dy);
        wp.partial = static_cast<float *>(ws);
        wp.dw = dw;
        return launch_status(launch_wgrad_strip(wp, lds, st));
    }
    WgradParams p;
    memset(&p, 0, sizeof(p));
    p.x = static_cast<const uint16_t *>(x);
    p.dy = static_cast<const uint16_t *>(dy);
    p.partial = static_cast<float *>(ws);
    p.N = desc->n; p.C = desc->c; p.H = desc->h; p.W = desc->w;
    p.K = desc->k; p.P = P; p.Q = Q; p.R = desc->r; p.S = desc->s;
    p.sh = desc->stride_h; p.sw = desc->stride_w; p.dh = desc->dil_h; p.dw = desc->dil_w;
    p.pbh = desc->pad_below_h; p.pbw = desc->pad_below_w;
    p.M = (uint32_t)desc->n * P * Q;
    wgrad_split(desc, P, Q, &p.chunk, &p.splits);
    p.div_pq = make_fastdiv((uint32_t)(P * Q));
    p.div_q = make_fastdiv((uint32_t)Q);
    hipError_t e = launch_wgrad(p, st);
    if (e != hipSuccess) return NGC_LAUNCH_FAILED;
    return launch_status(launch_wgrad_reduce(p.partial, dw, p.splits, desc->k, desc->c, desc->r, desc->s, st));
}

int ngc_layout_convert(int32_t dtype, int32_t n, int32_t c, int32_t h, int32_t w, const void *src, int32_t src_layout,
                       void *dst, int32_t dst_layout, void *hip_stream)
{
    if (dtype != NGC_F32 && dtype != NGC_BF16) return NGC_BAD_ARG;
    if (!layout_ok(src_layout) || !layout_ok(dst_layout)) return NGC_BAD_ARG;
    if (!src || !dst) return NGC_BAD_ARG;
    if (n < 1 || c < 1 || h < 1 || w < 1) return NGC_BAD_SHAPE;
    if ((size_t)n * (((size_t)c + 15) / 16) * 16 * h * w >= MAX_ELEMS) return NGC_BAD_SHAPE;
    return launch_status(launch_layout_convert(dtype == NGC_F32 ? 4 : 2, n, c, h, w, src, src_layout, dst, dst_layout,
                                               static_cast<hipStream_t>(hip_stream)));
}

int ngc_filter_convert(const ngc_conv_desc *desc, const void *w_kcrs, void *w_blocked, int32_t dst_layout,
                       void *hip_stream)
{
    int P, Q;
    const int vs = validate(desc, &P, &Q);
    if (vs != NGC_OK) return vs;
    if (!w_kcrs || !w_blocked) return NGC_BAD_ARG;
    if (dst_layout != NGC_BLOCKED_FWD && dst_layout != NGC_BLOCKED_BWD) return NGC_BAD_ARG;
    return launch_status(launch_filter_convert(desc->dtype == NGC_F32 ? 4 : 2, desc->k, desc->c, desc->r, desc->s, w_kcrs,
                                               w_blocked, dst_layout, static_cast<hipStream_t>(hip_stream)));
}

}  // extern "C"
