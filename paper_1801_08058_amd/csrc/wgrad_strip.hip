// ConvolutionBackpropFilters for stride-1 3x3-class filters (9 taps) on bf16 MFMA (gfx950):
// every tap from one pass over the data.
//
//   dw[k,c,r,s] = sum_{m=(n,p,q)} dy[m][k] * X[m + tap(r,s)][c]
//
// A workgroup owns a strip of positions (TP rows of NI images) and the full 64(k) x 64(c) x
// 9(tap) block of dw for it, all accumulators resident in registers as MFMA 16x16 tiles:
// wave (cq, h) holds channels c in [16cq, 16cq+16) x all 64 k x all 9 taps = 36 tiles = 144
// registers.  NW = 8 waves: two waves per SIMD, h = parity of the 32-position step (a
// wave-level split of the reduction, summed through LDS at the end), so that one wave's LDS
// latency hides behind the other's MFMAs.  dy and x are read from HBM/L2 once per workgroup
// instead of once per tap.
//
// The strip is processed in stages of SR rows through a ring of 2 or 3 LDS buffers (3 when they
// fit: one stage of MFMAs is shorter than the latency of a load).  A stage brings into LDS, with direct
// global->LDS loads (16 bytes per lane; out-of-range lanes deliver zeros, which is the padding
// halo and the tail of the strip):
//     dy tile : [positions][64 k]   as 4 planes of [position][16 k]  (32-byte rows)
//     x patch : [(SR+2) x (Q+2) px][64 c] as 4 planes of [pixel][16 c]
// i.e. both in their natural channel-contiguous form.  The MFMA needs the reduction axis
// (positions) contiguous per lane; the LDS transpose load ds_read_b64_tr_b16 does exactly that:
// 16 lanes read a 4(position) x 16(channel) block and each lane receives one channel's 4
// positions.  Two such loads give a lane its 8 reduction elements of v_mfma_f32_16x16x32_bf16.
// Which 8 of the step's 32 positions a lane group holds is free as long as both operands agree:
// group g takes positions 4g..4g+3 and 16+4g..16+4g+3, so that the 64 lanes of one load cover
// 512 contiguous bytes (lane groups 256 bytes apart would hit the same banks).  Because rows of the transposed block are whole
// 32-byte pixels, a filter tap is just a pixel offset in the address (no alignment problem, no
// shifted copies).
//
// Per 32-position step a wave issues 8 (dy) + 18 (x, 9 taps) transpose loads for 36 MFMAs; x
// fragments run a whole step ahead of the MFMAs in a rolling 9-slot buffer (across step
// boundaries), the dy fragments of the wave's next step are fetched during the current one.
// The per-workgroup partial (in register order) goes to the workspace; wgrad_strip_reduce adds the
// workgroups in index order (deterministic) and writes dw as [K][C][R][S].
#include "common.h"

#include <type_traits>

namespace ngc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

#ifdef NGC_TIMELINE
// development builds only: time stamps (100 MHz counter) of lane 0 of every wave in 4 KB of LDS behind the stage ring
__device__ unsigned long long g_ws_timeline[1024 * 8 * 64];
#define WS_TL()                                                                                   \
    do {                                                                                          \
        if (lane == 0 && tl_n < 64) tl_lds[wave * 64 + tl_n] = wall_clock64();                    \
        ++tl_n;                                                                                   \
    } while (0)
#else
#define WS_TL() do { } while (0)
#endif

constexpr unsigned WS_OOB = 0x80000000u;
constexpr int WS_NT = 9;
constexpr int WS_NB = 9;                           // x operand slots of a wave: a divisor of WS_NT, so that the slot of a tap is the
                                                   // same in every step; 9 = every tap's operand is requested a whole step ahead
                                                   // (3: cfg2 27.5 -> 27.3 us, 256 -> 256 at 14x14 43.4 -> 42.4 us, others unchanged)
constexpr int WS_MAXDY = 4;                        // dy load slots per wave and stage: 4 planes x at most 7 blocks over 8 waves
constexpr int WS_MAXX = 7;                         // x load slots per wave and stage (the host plan keeps NCQ * blocks <= 56)

__device__ __forceinline__ bf16x8 tr_frag(const unsigned char *lo, const unsigned char *hi)
{
    // two 4x16 transposed blocks -> this lane's 8 reduction elements
    const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)lo);
    const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)hi);
    const s16x8 r = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

// NCQ = 16-channel groups of c per workgroup (4, 2 or 1); the 8 waves are NCQ channel groups x
// NH = 8/NCQ interleaved step streams.  Fewer channels per workgroup means fewer, longer position
// chunks for the same number of workgroups, i.e. fewer partial copies of dw to write and re-read.
// MULTI: stages of several whole images (p.G of them); a separate instantiation so that the
// one-image path carries none of the extra index arithmetic.
// U3: the nine taps are three rows of three with a column step of one pixel (a 3x3 window with dilation 1 along w):
// the taps of a row then differ by a constant 32 bytes, which rides in the offset field of the LDS read - two address
// additions per row and step instead of two per tap.
template <int NCQ, bool MULTI, bool U3>
__global__ __launch_bounds__(512) void wgrad_strip_bf16(const WgradStripParams p)
{
    constexpr int NW = 8;
    constexpr int NH = NW / NCQ;             // waves per channel group = step interleave
    extern __shared__ __align__(16) unsigned char smem[];
    preload_kernargs(p);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cq = wave % NCQ;               // 16-channel group inside the workgroup's c tile
    const int wh = wave / NCQ;               // which of the NH step streams
    const int L = lane & 15;                 // lane inside its 16-lane transpose group
    const int grp = lane >> 4;               // reduction group: positions 4*grp.. and 16+4*grp..

    const int igrp = blockIdx.x / p.strips;            // group of NI images
    const int strip = blockIdx.x - igrp * p.strips;
    const int n0 = igrp * p.NI;
    const int nimg = (p.N - n0 < p.NI) ? (p.N - n0) : p.NI;
    const int p0 = strip * p.TP;
    const int rows_strip = (p.P - p0 < p.TP) ? (p.P - p0) : p.TP;
    const int kt = blockIdx.y / p.ctiles;
    const int ct = blockIdx.y - kt * p.ctiles;

    const int PQ = p.P * p.Q;
    const int HW = p.H * p.W;
    const int KB = p.K >> 4, CB = p.C >> 4;
    const int stage_bytes = 4 * p.dyplane + NCQ * p.xplane;
#ifdef NGC_TIMELINE
    int tl_n = 0;
    unsigned long long *tl_lds = reinterpret_cast<unsigned long long *>(smem + p.nring * stage_bytes);
    WS_TL();
#endif

    const ngc_u32x4 rs_dy = make_rsrc_words(p.dy, p.dy_bytes);
    const ngc_u32x4 rs_x = make_rsrc_words(p.x, p.x_bytes);

    // G > 1: a stage holds G whole (small) images: positions and patch pixels are numbered image after
    // image (G = 1: one image, SR of its rows)
    const int G = MULTI ? p.G : 1;
    const int npatch1 = p.PRS * p.PC;                       // patch pixels of one image
    const int npatch = G * npatch1;
    const int nblk_x = (npatch + 31) >> 5;
    const int stage_pos = MULTI ? G * PQ : p.SR * p.Q;      // positions of a full stage
    const int steps_full = (stage_pos + 31) >> 5;           // 32-position steps of a full stage
    const int nblk_dy = steps_full;

    // load items of a stage: (plane, 32-position block) pairs, 4 dy planes and NCQ x planes, each kind dealt
    // round-robin to the 8 waves (slot i of a wave = item wave + 8 i of the kind).  What does not change from
    // stage to stage is computed once: per slot the LDS destination and the plane's byte offset (wave-uniform;
    // the latter goes into the load's scalar offset), per slot and lane the offset inside the stage and what
    // decides validity in a given stage.  A stage then costs a handful of instructions per load: the address
    // arithmetic would otherwise take more issue cycles than the MFMAs of the stage.
    const int items_dy = 4 * nblk_dy, items_x = NCQ * nblk_x;
    const int ndy = (items_dy - wave + NW - 1) / NW;                     // this wave's dy / x slots in use
    const int nx = (items_x - wave + NW - 1) / NW;
    const int lane_half = lane >> 1;
    int dy_lds[WS_MAXDY], dy_pos0[WS_MAXDY];
    unsigned dy_soff[WS_MAXDY], dy_voff[MULTI ? WS_MAXDY : 1];
#pragma unroll
    for (int i = 0; i < WS_MAXDY; ++i) {
        const int it = (i < ndy) ? wave + NW * i : 0;
        const int pln = it / nblk_dy, blk = it - pln * nblk_dy;
        dy_lds[i] = pln * p.dyplane + blk * 1024;
        dy_pos0[i] = blk * 32;                                           // the lane's position is dy_pos0 + lane / 2
        // G = 1: positions of a stage are contiguous in a plane; G > 1: image g of the stage is KB planes further on
        dy_soff[i] = (unsigned)(pln * PQ * 32) + (MULTI ? 0u : (unsigned)(blk * 1024));
        if constexpr (MULTI) {
            const int pos = blk * 32 + lane_half;
            const uint32_t g = fd_div((uint32_t)pos, p.div_pq);
            dy_voff[i] = (unsigned)(((int)g * (KB - 1) * PQ + pos) * 32 + (lane & 1) * 16);
        }
    }
    // x: x_row = the patch row (G = 1) or the image inside the stage (G > 1, rows are then always the whole
    // image); lanes that never load (beyond the patch, or a column outside the image) get a row no stage accepts
    int x_lds[WS_MAXX], x_row[WS_MAXX];
    unsigned x_soff[WS_MAXX], x_off[WS_MAXX];
#pragma unroll
    for (int j = 0; j < WS_MAXX; ++j) {
        const int it = (j < nx) ? wave + NW * j : 0;
        const int pln = it / nblk_x, blk = it - pln * nblk_x;
        x_lds[j] = 4 * p.dyplane + pln * p.xplane + blk * 1024;
        x_soff[j] = (unsigned)(pln * HW * 32);
        const uint32_t px = (uint32_t)(blk * 32 + lane_half);
        const uint32_t g = MULTI ? fd_div(px, p.div_patch) : 0;
        const uint32_t px1 = px - g * (uint32_t)npatch1;
        const uint32_t pr = fd_div(px1, p.div_pc);
        const uint32_t pc = px1 - pr * p.div_pc.d;
        const int w = p.min_dw + (int)pc;
        bool ok = px < (uint32_t)npatch && (unsigned)w < (unsigned)p.W;
        if (MULTI) ok = ok && (unsigned)(p.min_dh + (int)pr) < (unsigned)p.H;   // stage = whole images: rows fixed
        x_off[j] = (unsigned)((((int)g * CB * p.H + (int)pr) * p.W + (int)pc) * 32 + (lane & 1) * 16);
        x_row[j] = ok ? (MULTI ? (int)g : (int)pr) : 0x40000000;
    }
    // Stages are issued in order, one call each: the (image, row block) of the next one is carried along.
    int is_img = n0, is_stage = 0;
    auto issue_loads = [&](int buf) {
        unsigned char *base = smem + buf * stage_bytes;
        const int r0 = is_stage * p.SR;                                  // first strip row of the stage (G = 1)
        int rows = rows_strip - r0;
        if (rows > p.SR) rows = p.SR;
        int gvalid = nimg - (is_img - n0);                               // images of the stage that exist (G > 1)
        if (gvalid > G) gvalid = G;
        const int nvalid = MULTI ? gvalid * PQ : rows * p.Q;             // positions of the stage that exist
        const int h0 = p0 + r0 + p.min_dh;
        // stage origins (x: pixel (h0, min_dw), possibly outside the image; valid lanes end up in range)
        const unsigned dy_org = (unsigned)((((is_img * KB + kt * 4) * PQ) + (p0 + r0) * p.Q) * 32);
        const unsigned x_org = (unsigned)(((is_img * CB + ct * NCQ) * HW + h0 * p.W + p.min_dw) * 32);
        const unsigned dy_lane = dy_org + (unsigned)(lane * 16);
        const int radd = MULTI ? 0 : h0;                                 // x lane valid: (unsigned)(x_row + radd) < rlim
        const unsigned rlim = MULTI ? (unsigned)gvalid : (unsigned)p.H;
#pragma unroll
        for (int i = 0; i < WS_MAXDY; ++i)
            if (i < ndy) {                                               // wave-uniform
                const bool ok = lane_half < nvalid - dy_pos0[i];
                const unsigned off = ok ? (MULTI ? dy_org + dy_voff[MULTI ? i : 0] : dy_lane) : WS_OOB;
                dma_load_lds16(rs_dy, base + dy_lds[i], off, dy_soff[i]);
            }
#pragma unroll
        for (int j = 0; j < WS_MAXX; ++j)
            if (j < nx) {
                const bool ok = (unsigned)(x_row[j] + radd) < rlim;
                const unsigned off = ok ? x_org + x_off[j] : WS_OOB;
                dma_load_lds16(rs_x, base + x_lds[j], off, x_soff[j]);
            }
        if (MULTI) is_img += G;
        else if (++is_stage == p.nstages) { is_stage = 0; ++is_img; }
    };

    // Accumulator block i of this wave holds k block i ^ kbm: the streams number their blocks differently so that the
    // exchange at the end moves the same registers in every wave (sends blocks 2-3, then block 1; keeps block 0)
    const int kbm = NH == 4 ? (((wh & 1) << 1) | (wh >> 1)) : NH == 2 ? ((wh & 1) << 1) : 0;
    f32x4 acc[4][WS_NT];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int t = 0; t < WS_NT; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[a][t][v] = 0.f;

    const int last_pos = stage_pos - 1;
    // byte offset of this lane inside a transposed 4x16 block: row L/4 (32 B each), 8-byte column group L%4
    const int lane_col = (L & 3) * 8;

    // LDS byte offsets of this lane's two 4-position groups of a 32-position step
    auto step_offsets = [&](int step, int (&dyoff)[2], int (&xoff)[2]) {
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            int pos = step * 32 + e * 16 + grp * 4 + (L >> 2);
            dyoff[e] = pos * 32 + lane_col;
            if (pos > last_pos) pos = last_pos;                          // dy is zero there; keep x in range
            const uint32_t g = MULTI ? fd_div((uint32_t)pos, p.div_pq) : 0;
            const uint32_t pos1 = (uint32_t)pos - g * (uint32_t)PQ;
            const uint32_t row = fd_div(pos1, p.div_q);
            const uint32_t col = pos1 - row * p.div_q.d;
            xoff[e] = (int)((g * p.PRS + row) * p.PC + col) * 32 + lane_col;
        }
    };

    // Ring of p.nring (2 or 3) stage buffers.  Every stage costs this wave the same number of
    // loads (lpw), so "stage s has landed" is vmcnt <= lpw * (stages issued after s).
    const int total_stages = MULTI ? (nimg + G - 1) / G : nimg * p.nstages;
    const int lpw = ndy + nx;
    const int ahead = p.nring - 1;
    // Waves of the late group issue the loads of stage s + ahead after their MFMAs of stage s instead of
    // before: a wave is held at issue while the memory system takes its loads, and with one wave of each
    // SIMD in either group the other one's MFMAs run meanwhile.  Counting is unchanged (per wave, in order).
    const bool late = (p.late_mask >> wave) & 1;
    WS_TL();
    for (int s = 0; s < ahead && s < total_stages; ++s) issue_loads(s);
    WS_TL();
    int buf = 0;                                            // s % nring
    for (int s = 0; s < total_stages; ++s) {
        const int later = (total_stages - 1 - s < ahead - 1) ? total_stages - 1 - s : ahead - 1;
        wait_vmcnt(later * lpw);
        wg_barrier_nofence();                                 // stage s complete for everybody; buffer of s-1 is free
        WS_TL();
        const int nbuf = (buf + ahead) % p.nring;
        if (!late && s + ahead < total_stages) issue_loads(nbuf);
        WS_TL();
        int rows = rows_strip - (s % p.nstages) * p.SR;
        if (rows > p.SR) rows = p.SR;
        int gv = nimg - s * G;
        if (gv > G) gv = G;
        const int nsteps = ((MULTI ? gv * PQ : rows * p.Q) + 31) >> 5;      // steps that contain at least one position
        const unsigned char *dys = smem + buf * stage_bytes;
        const unsigned char *xs = smem + buf * stage_bytes + 4 * p.dyplane + cq * p.xplane;
        buf = (buf + 1 == p.nring) ? 0 : buf + 1;
        auto load_a = [&](const int (&dyoff)[2], bf16x8 (&a)[4]) {
#pragma unroll
            for (int kb = 0; kb < 4; ++kb)
                a[kb] = tr_frag(dys + (kb ^ kbm) * p.dyplane + dyoff[0], dys + (kb ^ kbm) * p.dyplane + dyoff[1]);
        };
        auto load_b = [&](const int (&xoff)[2], int t) {
            if constexpr (U3) {
                const int row = p.tap_off[(t / 3) * 3] * 32;
                return tr_frag(xs + xoff[0] + row + (t % 3) * 32, xs + xoff[1] + row + (t % 3) * 32);
            }
            return tr_frag(xs + xoff[0] + p.tap_off[t] * 32, xs + xoff[1] + p.tap_off[t] * 32);
        };

        // step streams continue across stages so that the remainders even out
        int j = (wh - (s * steps_full) % NH + NH) % NH;
        if (j < nsteps) {
            int dyo[2], xo[2];
            bf16x8 acur[4], b[WS_NB];
            step_offsets(j, dyo, xo);
            load_a(dyo, acur);
#pragma unroll
            for (int t = 0; t < WS_NB; ++t) b[t] = load_b(xo, t);
            // One step = 9 taps x 4 MFMAs.  The body exists in two straight-line versions (with and
            // without the fetches of the wave's next step) so that every LDS wait is an exact count.
            auto step_body = [&](auto has_next_tag) {
                constexpr bool HAS_NEXT = decltype(has_next_tag)::value;
                int dyn[2], xn[2];
                bf16x8 anext[4];
                if (HAS_NEXT) step_offsets(j + NH, dyn, xn);
#pragma unroll
                for (int t = 0; t < WS_NT; ++t) {
#pragma unroll
                    for (int kb = 0; kb < 4; ++kb)
                        acc[kb][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(acur[kb], b[t % WS_NB], acc[kb][t], 0, 0, 0);
                    // refill the slot just consumed: tap t + WS_NB of this step, or tap t + WS_NB - 9 of the next
                    if (t + WS_NB < WS_NT) b[t % WS_NB] = load_b(xo, t + WS_NB);
                    else if (HAS_NEXT) b[t % WS_NB] = load_b(xn, t + WS_NB - WS_NT);
                    if (t == 2 && HAS_NEXT) load_a(dyn, anext);
                }
                if (HAS_NEXT) {
#pragma unroll
                    for (int kb = 0; kb < 4; ++kb) acur[kb] = anext[kb];
#pragma unroll
                    for (int e = 0; e < 2; ++e) { dyo[e] = dyn[e]; xo[e] = xn[e]; }
                }
            };
            while (j + NH < nsteps) {
                step_body(std::true_type{});
                j += NH;
            }
            step_body(std::false_type{});
        }
        WS_TL();
        if (late && s + ahead < total_stages) issue_loads(nbuf);
    }
    WS_TL();
    __syncthreads();                                        // all stage buffers are free
    WS_TL();

    // ---- sum the NH step-stream copies of the tile and write the partial.
    // Accumulator register v of tile (kb, t): k = 16 kb + 4*(lane/16) + v, c = 16 cq + lane%16.
    // The partial is stored in register order, [tile][cq][kb][tap][lane][v] (16 bytes per lane,
    // 1 KB per store instruction); wgrad_strip_reduce maps it back to [K][C][R][S].
    f32x4 *red = reinterpret_cast<f32x4 *>(smem);
    f32x4 *out = reinterpret_cast<f32x4 *>(p.partial) +
                 (((size_t)blockIdx.x * gridDim.y + blockIdx.y) * NCQ + cq) * (4 * WS_NT * 64);
    // Partials are streamed out (non-temporal stores) when there are few enough of them for the reduce kernel to find
    // them in the memory-side cache anyway; with more, ordinary stores are faster (the host decides, p.stream_partials).
    const bool stream_part = p.stream_partials != 0;
    auto put = [&](int idx, const f32x4 &v) {
        const ngc_u32x4 w = __builtin_bit_cast(ngc_u32x4, v);
        store16_result(out + idx, make_uint4(w[0], w[1], w[2], w[3]), stream_part);
    };
    if constexpr (NH == 2 || NH == 4) {
        // Butterfly over the streams: in every round each wave hands half of the k blocks it still owns to the
        // partner stream and adds the partner's copy of the half it keeps, so all eight waves move data in every
        // round and each ends up owning 4 / NH k blocks of the sum (k block kbm, and kbm + 1 for NH = 2), which it
        // stores itself.  The block numbering per stream (kbm) makes a wave's kept blocks its partner's sent ones.
        // Outbox of wave w: 18 tiles of 1 KB at red + w * 18 * 64.
        f32x4 *outbox = red + wave * (18 * 64);
        const f32x4 *inbox1 = red + (cq + NCQ * (wh ^ 1)) * (18 * 64);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int t = 0; t < WS_NT; ++t) outbox[(i * WS_NT + t) * 64 + lane] = acc[2 + i][t];
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int t = 0; t < WS_NT; ++t) acc[i][t] += inbox1[(i * WS_NT + t) * 64 + lane];
        if constexpr (NH == 4) {
            __syncthreads();                                        // outboxes are free again
            const f32x4 *inbox2 = red + (cq + NCQ * (wh ^ 2)) * (18 * 64);
#pragma unroll
            for (int t = 0; t < WS_NT; ++t) outbox[t * 64 + lane] = acc[1][t];
            __syncthreads();
#pragma unroll
            for (int t = 0; t < WS_NT; ++t) acc[0][t] += inbox2[t * 64 + lane];
#pragma unroll
            for (int t = 0; t < WS_NT; ++t) put((kbm * WS_NT + t) * 64 + lane, acc[0][t]);
        } else {
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int t = 0; t < WS_NT; ++t) put(((kbm + i) * WS_NT + t) * 64 + lane, acc[i][t]);
        }
        WS_TL();
    } else {
        // eight streams (NCQ = 1): plain tree, waves of the upper half publish, the lower half adds
#pragma unroll
        for (int stride = NH / 2; stride >= 1; stride >>= 1) {
            if (wh >= stride && wh < 2 * stride) {
                f32x4 *dst = red + ((wh - stride) * NCQ + cq) * (4 * WS_NT * 64);
#pragma unroll
                for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                    for (int t = 0; t < WS_NT; ++t) dst[(kb * WS_NT + t) * 64 + lane] = acc[kb][t];
            }
            __syncthreads();
            if (wh < stride) {
                const f32x4 *src = red + (wh * NCQ + cq) * (4 * WS_NT * 64);
#pragma unroll
                for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                    for (int t = 0; t < WS_NT; ++t) acc[kb][t] += src[(kb * WS_NT + t) * 64 + lane];
            }
            __syncthreads();
        }
        WS_TL();
        if (wh == 0) {
#pragma unroll
            for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                for (int t = 0; t < WS_NT; ++t) put((kb * WS_NT + t) * 64 + lane, acc[kb][t]);
        }
    }
#ifdef NGC_TIMELINE
    WS_TL();
    __builtin_amdgcn_s_waitcnt(0x0F70);
    WS_TL();
    if (lane == 0 && blockIdx.x < 512 && blockIdx.y < 2)
        for (int i = 0; i < 64; ++i) g_ws_timeline[((blockIdx.y * 512 + blockIdx.x) * 8 + wave) * 64 + i] = i < tl_n ? tl_lds[wave * 64 + i] : 0;
#endif
}

// dw[k][c][tap] = sum over workgroup partials (index order) of partial[part][tile][cq][kb][tap][lane][v].
// 256 threads = 256 / SL float4 outputs x SL interleaved partial streams (two chains each), joined in a fixed order.
// SL = 16 when there are many parts (few (k, c) tiles: more loads in flight per output), 8 otherwise.
template <int SL>
__global__ __launch_bounds__(256) void wgrad_strip_reduce(const f32x4 *__restrict__ partial, float *__restrict__ dw,
                                                         int nparts, int K, int C, int ctiles, int ncq)
{
    constexpr int NO = 256 / SL;
    __shared__ f32x4 sm[SL == 1 ? 1 : SL][SL == 1 ? 1 : NO];
    const size_t per4 = (size_t)WS_NT * K * C / 4;          // float4 elements of one partial
    const int o = threadIdx.x % NO;
    const int sl = threadIdx.x / NO;
    const size_t i = (size_t)blockIdx.x * NO + o;           // per4 is a multiple of 32
    f32x4 t0 = {0.f, 0.f, 0.f, 0.f}, t1 = t0;
    int sp = sl;
    for (; sp + SL < nparts; sp += 2 * SL) {
        t0 += partial[(size_t)sp * per4 + i];
        t1 += partial[(size_t)(sp + SL) * per4 + i];
    }
    if (sp < nparts) t0 += partial[(size_t)sp * per4 + i];
    if constexpr (SL > 1) {
        sm[sl][o] = t0 + t1;
        __syncthreads();
    }
    if (sl == 0) {
        f32x4 r = t0 + t1;                                  // SL == 1: one thread per output, no exchange
        if constexpr (SL > 1) {
            f32x4 q[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) q[j] = SL == 16 ? sm[2 * j][o] + sm[(2 * j + 1) % SL][o] : sm[j % SL][o];
            r = ((q[0] + q[1]) + (q[2] + q[3])) + ((q[4] + q[5]) + (q[6] + q[7]));
        }
        // decode register order: i = (((tile*ncq + cq)*4 + kb)*9 + t)*64 + lane
        const int lane = (int)(i & 63);
        size_t u = i >> 6;
        const int t = (int)(u % WS_NT); u /= WS_NT;
        const int kb = (int)(u & 3); u >>= 2;
        const int cq = (int)(u % ncq); u /= ncq;
        const int tile = (int)u;
        const int kt = tile / ctiles, ct = tile - kt * ctiles;
        const int c = (ct * ncq + cq) * 16 + (lane & 15);
        const int k = kt * 64 + kb * 16 + 4 * (lane >> 4);
#pragma unroll
        for (int v = 0; v < 4; ++v) dw[((size_t)(k + v) * C + c) * WS_NT + t] = r[v];
    }
}

template <int NCQ, bool MULTI, bool U3>
static hipError_t launch_wgrad_strip_t(const WgradStripParams &p, size_t lds_bytes, hipStream_t st)
{
    static LdsLimitOnce lds_limit;                  // per template instantiation
    {
        const hipError_t e = lds_limit.raise(reinterpret_cast<const void *>(&wgrad_strip_bf16<NCQ, MULTI, U3>));
        if (e != hipSuccess) return e;
    }
    dim3 grid(p.nparts, (p.K / 64) * p.ctiles);
#ifdef NGC_TIMELINE
    lds_bytes += 4096;
#endif
    NGC_LAUNCH((wgrad_strip_bf16<NCQ, MULTI, U3>), grid, dim3(512), lds_bytes, st, p);
    return ngc::launch_result();
}

template <int NCQ, bool MULTI>
static hipError_t launch_wgrad_strip_ncq(const WgradStripParams &p, size_t lds_bytes, hipStream_t st)
{
    bool u3 = true;
    for (int t = 0; t < WS_NT; ++t) u3 = u3 && p.tap_off[t] == p.tap_off[(t / 3) * 3] + t % 3;
    return u3 ? launch_wgrad_strip_t<NCQ, MULTI, true>(p, lds_bytes, st) : launch_wgrad_strip_t<NCQ, MULTI, false>(p, lds_bytes, st);
}

#ifdef NGC_TIMELINE
extern "C" int ngc_debug_ws_timeline(unsigned long long *host_dst, size_t count)
{
    return (int)hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(g_ws_timeline), count * sizeof(unsigned long long));
}
#endif

hipError_t launch_wgrad_strip(const WgradStripParams &p, size_t lds_bytes, hipStream_t st)
{
    hipError_t e = hipErrorInvalidValue;
    if (p.G > 1) {
        e = p.ncq == 4 ? launch_wgrad_strip_ncq<4, true>(p, lds_bytes, st)
            : p.ncq == 2 ? launch_wgrad_strip_ncq<2, true>(p, lds_bytes, st)
            : p.ncq == 1 ? launch_wgrad_strip_ncq<1, true>(p, lds_bytes, st)
                         : hipErrorInvalidValue;
    } else {
        e = p.ncq == 4 ? launch_wgrad_strip_ncq<4, false>(p, lds_bytes, st)
            : p.ncq == 2 ? launch_wgrad_strip_ncq<2, false>(p, lds_bytes, st)
            : p.ncq == 1 ? launch_wgrad_strip_ncq<1, false>(p, lds_bytes, st)
                         : hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    const size_t per4 = (size_t)WS_NT * p.K * p.C / 4;
    if (p.nparts >= 16)
        NGC_LAUNCH(wgrad_strip_reduce<16>, dim3((unsigned)(per4 / 16)), dim3(256), 0, st,
                   reinterpret_cast<const f32x4 *>(p.partial), p.dw, p.nparts, p.K, p.C, p.ctiles, p.ncq);
    else if (p.nparts > 8)
        NGC_LAUNCH(wgrad_strip_reduce<8>, dim3((unsigned)(per4 / 32)), dim3(256), 0, st,
                   reinterpret_cast<const f32x4 *>(p.partial), p.dw, p.nparts, p.K, p.C, p.ctiles, p.ncq);
    else                                                // a handful of parts: one thread per output adds them itself
        NGC_LAUNCH(wgrad_strip_reduce<1>, dim3((unsigned)(per4 / 256)), dim3(256), 0, st,
                   reinterpret_cast<const f32x4 *>(p.partial), p.dw, p.nparts, p.K, p.C, p.ctiles, p.ncq);
    return ngc::launch_result();
}

}  // namespace ngc
