// Kernel templates of the strip convolution, shared by the translation units that instantiate them (rank 2 in
// conv_strip.hip, rank 3 in conv_strip3.hip: two code objects, so that work on one leaves the other byte-identical).
//
// Multi-tap convolution (forward with any stride, backprop-data per residue class of the stride)
// as an output-stationary "strip" kernel on bf16 MFMA (gfx950), fp32 accumulate.
//
// A workgroup (256 threads, 4 waves, one per SIMD) owns a strip of up to 4*NF*32 output
// positions (TN images x TP output rows x full width) for 64 output channels and keeps ALL
// of its accumulators in registers: wave w owns position fragments w, w+4, ... (NF of them,
// 32 positions each) x 2 channel fragments = 2*NF MFMA 32x32 tiles.  The reduction runs over
// 16-input-channel chunks.  For each chunk the workgroup brings into LDS, with direct
// global->LDS loads (buffer_load_dwordx4 ... lds, 16 bytes per lane, out-of-range lanes
// return zeros = the padding halo):
//     X patch : the input footprint of the strip (TN x PR x PC pixels) x 16 channels, once,
//               and uses it for every filter tap (an input pixel is read from L2/HBM once per
//               strip instead of once per tap),
//     W slab  : all taps x 16 channels x 64 output channels,
// as 16-byte-unit planes (g = which 8 of the 16 channels) so that every MFMA operand fetch is
// one conflict-free ds_read_b128.  Two LDS stages: the loads of chunk c+1 are issued right
// after the barrier that opens chunk c and are in flight during its MFMAs (one chunk = taps *
// 2 * NF MFMAs per wave, about 4000 cycles for 3x3), so one barrier per chunk suffices.
//
// MFMA roles as in the gather kernel: A = filters (rows = output channels), B = activations
// (columns = positions), v_mfma_f32_32x32x16_bf16.  Epilogue: the accumulators start from the bias, one RNE
// rounding, ReLU on the rounded pairs, lane-pair exchange, 16-byte stores; for blocked rank-2 results below 2 GiB it
// runs inside the last chunk, fragment after fragment (strip_chunk_mfma_last).  The kernels here also come with two
// waves per SIMD (NW = 8: wave w owns fragments w, w + 8, ...), a fragment shared between two waves where that evens
// out the SIMDs, and two chunks per LDS stage for small strips (StripParams::cps).
#pragma once
#include "common.h"

#include <stdlib.h>

#include <type_traits>

namespace ngc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void lds_void;

#ifdef NGC_TIMELINE
// development builds only: time stamps (100 MHz counter, low 32 bits) of every wave, 16 slots, kept in registers
static __device__ unsigned g_strip_timeline[1024 * 8 * 16];   // one copy per translation unit
#define STRIP_TL(k) tl[k] = (unsigned)wall_clock64()
#else
#define STRIP_TL(k) do { } while (0)
#endif

constexpr int STRIP_WPITCH = 64 * 16 + 128;     // bytes per (tap, g) filter plane
constexpr int STRIP_MAXBLOCKS = 24;             // 64-pixel patch blocks per plane (whole workgroup)
constexpr unsigned STRIP_OOB = 0x80000000u;     // byte offset beyond any buffer -> load returns 0

__device__ __forceinline__ void load_lds16(__amdgpu_buffer_rsrc_t rsrc, unsigned char *lds_dst_uniform, unsigned voff,
                                           unsigned soff)
{
    // each lane: 16 bytes from (base + voff + soff) -> lds_dst_uniform + lane*16
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void *)lds_dst_uniform, 16, (int)voff, (int)soff, 0, 0);
}

// MFMAs of one 16-channel chunk for a wave that holds NFR position fragments.  The LDS reads run one tap ahead of the
// MFMAs: the two filter operands of tap t+1 are requested before the MFMAs of tap t, and the activation operand of a
// fragment is requested for tap t+1 right after the MFMAs of tap t that read it, into the same registers - so the
// wave never waits for a read it has just issued, at the price of 8 more registers.  No branch inside the loop: the
// counted waits the compiler derives stay exact.  tapv holds the patch byte offset of tap l in lane l
// (STRIP_MAX_TAPS <= 64): a lane read brings it into a scalar register without a memory operation in the loop.
// HS: the wave also holds one channel half of a fragment it shares with another wave (slot NFR of acc / pbase, tile 0;
// wsh = ws moved to that channel half's filter rows): one MFMA per tap.
template <int NF, int NFR, bool HS, bool UPPER, int WSTRIDE_T>
__device__ __forceinline__ void strip_chunk_mfma(f32x16 (&acc)[NF][2], const unsigned char *xs, const unsigned char *ws,
                                                 const unsigned char *wsh, const int (&pbase)[NF], const int tapv,
                                                 const int ntaps)
{
    static_assert(NFR >= 1 && NFR + (HS ? 1 : 0) <= NF, "fragments held by the wave");
    constexpr int SH = HS ? NFR : 0;                     // slot of the shared fragment
    bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(ws);
    bf16x8 a1 = a0;
    if (UPPER) a1 = *reinterpret_cast<const bf16x8 *>(ws + 32 * 16);
    bf16x8 ah = a0, bh = a0;
    if (HS) ah = *reinterpret_cast<const bf16x8 *>(wsh);
    bf16x8 b[NFR];
    {
        const int toff = __builtin_amdgcn_readlane(tapv, 0);
#pragma unroll
        for (int i = 0; i < NFR; ++i) b[i] = *reinterpret_cast<const bf16x8 *>(xs + pbase[i] + toff);
        if (HS) bh = *reinterpret_cast<const bf16x8 *>(xs + pbase[SH] + toff);
    }
    for (int t = 1; t < ntaps; ++t) {
        const int toff = __builtin_amdgcn_readlane(tapv, t);
        const bf16x8 a0n = *reinterpret_cast<const bf16x8 *>(ws + t * WSTRIDE_T);
        bf16x8 a1n = a0n;
        if (UPPER) a1n = *reinterpret_cast<const bf16x8 *>(ws + t * WSTRIDE_T + 32 * 16);
        bf16x8 ahn = a0n;
        if (HS) ahn = *reinterpret_cast<const bf16x8 *>(wsh + t * WSTRIDE_T);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < NFR; ++i) {
            acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b[i], acc[i][0], 0, 0, 0);
            if (UPPER) acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b[i], acc[i][1], 0, 0, 0);
            b[i] = *reinterpret_cast<const bf16x8 *>(xs + pbase[i] + toff);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (HS) {
            acc[SH][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc[SH][0], 0, 0, 0);
            bh = *reinterpret_cast<const bf16x8 *>(xs + pbase[SH] + toff);
            __builtin_amdgcn_sched_barrier(0);
        }
        a0 = a0n;
        a1 = a1n;
        ah = ahn;
    }
#pragma unroll
    for (int i = 0; i < NFR; ++i) {
        acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b[i], acc[i][0], 0, 0, 0);
        if (UPPER) acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b[i], acc[i][1], 0, 0, 0);
    }
    if (HS) acc[SH][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc[SH][0], 0, 0, 0);
}

// The last chunk of a workgroup, fragment after fragment instead of tap after tap: a fragment's accumulators are
// final after its own taps, so its epilogue (epi(i): ReLU, rounding, stores; epih() for the shared fragment) runs
// while the wave's other fragments - and the other wave of the SIMD - still have MFMAs to issue, and the results leave
// the chip during the chunk instead of all at once behind it.  Costs the two filter operands once per fragment and tap
// instead of once per tap (LDS is far from busy).  Same MFMAs per accumulator in the same order as strip_chunk_mfma:
// same bits.
template <int NF, int NFR, bool HS, bool UPPER, int WSTRIDE_T, class Epi, class EpiH>
__device__ __forceinline__ void strip_chunk_mfma_last(f32x16 (&acc)[NF][2], const unsigned char *xs, const unsigned char *ws,
                                                      const unsigned char *wsh, const int (&pbase)[NF], const int tapv,
                                                      const int ntaps, Epi &&epi, EpiH &&epih)
{
    static_assert(NFR >= 1 && NFR + (HS ? 1 : 0) <= NF, "fragments held by the wave");
#pragma unroll
    for (int i = 0; i < NFR; ++i) {
        bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(ws);
        bf16x8 a1 = a0;
        if (UPPER) a1 = *reinterpret_cast<const bf16x8 *>(ws + 32 * 16);
        bf16x8 b = *reinterpret_cast<const bf16x8 *>(xs + pbase[i] + __builtin_amdgcn_readlane(tapv, 0));
        for (int t = 1; t < ntaps; ++t) {
            const int toff = __builtin_amdgcn_readlane(tapv, t);
            const bf16x8 a0n = *reinterpret_cast<const bf16x8 *>(ws + t * WSTRIDE_T);
            bf16x8 a1n = a0n;
            if (UPPER) a1n = *reinterpret_cast<const bf16x8 *>(ws + t * WSTRIDE_T + 32 * 16);
            const bf16x8 bn = *reinterpret_cast<const bf16x8 *>(xs + pbase[i] + toff);
            __builtin_amdgcn_sched_barrier(0);
            acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b, acc[i][0], 0, 0, 0);
            if (UPPER) acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b, acc[i][1], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            a0 = a0n;
            a1 = a1n;
            b = bn;
        }
        acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b, acc[i][0], 0, 0, 0);
        if (UPPER) acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b, acc[i][1], 0, 0, 0);
        epi(i);
    }
    if constexpr (HS) {
        constexpr int SH = NFR;
        bf16x8 a = *reinterpret_cast<const bf16x8 *>(wsh);
        bf16x8 b = *reinterpret_cast<const bf16x8 *>(xs + pbase[SH] + __builtin_amdgcn_readlane(tapv, 0));
        for (int t = 1; t < ntaps; ++t) {
            const int toff = __builtin_amdgcn_readlane(tapv, t);
            const bf16x8 an = *reinterpret_cast<const bf16x8 *>(wsh + t * WSTRIDE_T);
            const bf16x8 bn = *reinterpret_cast<const bf16x8 *>(xs + pbase[SH] + toff);
            __builtin_amdgcn_sched_barrier(0);
            acc[SH][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[SH][0], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            a = an;
            b = bn;
        }
        acc[SH][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[SH][0], 0, 0, 0);
        epih();
    }
}

// SUB = 0: blocked output (p.out_mode 0).  SUB = 1 / 2: sub-pixel NCHW output (p.out_mode 1); with
// SUB = 1 only the lower 32 of the tile's 64 output columns are in use: one filter plane per tap (32
// rows of g = 0, then 32 rows of g = 1) and no upper MFMA.  The store modes are separate
// instantiations so that the blocked-output kernel carries none of the sub-pixel code.
// DB (blocked output only): every wave also writes the sums over its positions of the values it
// stored, per output channel (fp32, fixed order), to row (p.dbp_row0 + blockIdx.x) * NW + wave of
// p.dbp - the partials of a bias gradient of the stored tensor.  A separate instantiation.
// R3 (blocked output, no DB): rank-3 spatial tensors; images are (batch element, depth slice) pairs and the
// chunk loop runs over (depth tap, 16-channel chunk) pairs, the patch of a chunk coming from the depth slice
// the tap reads (zeros outside the volume).
// bx = workgroup index inside the launch's (group, strip) grid
// CT (blocked output, no DB): column tiles - a strip covers p.BW of the p.Wout lattice columns (rows wider than a
// strip holds); a separate instantiation so that the full-width kernels carry none of it.
template <int NF, int NW, int SUB, bool DB, bool R3 = false, bool CT = false>
__device__ __forceinline__ void conv_strip_body(const StripParams &p, const int bx, const int by)
{
    static_assert(!R3 || (SUB == 0 && !DB), "rank-3 launches store blocked tensors and no channel sums");
    static_assert(!CT || (SUB == 0 && !DB), "column tiles exist for blocked tensors without channel sums");
    constexpr bool HALF = SUB == 1;
    constexpr int MAXXB = STRIP_MAXBLOCKS / NW;         // patch blocks per wave
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31;
    const int lg = lane >> 5;
#ifdef NGC_TIMELINE
    unsigned tl[16] = {};
    STRIP_TL(0);
    auto tl_flush = [&]() {
        __builtin_amdgcn_s_waitcnt(0x0F70);
        STRIP_TL(15);
        if (lane < 16 && bx < 1024 && by == 0) {
            unsigned v = 0;
#pragma unroll
            for (int k = 0; k < 16; ++k) v = lane == k ? tl[k] : v;
            g_strip_timeline[(bx * 8 + wave) * 16 + lane] = v;
        }
    };
#endif

    const int grp = bx / p.strips;
    int strip = bx - grp * p.strips;
    int q0 = 0;                                          // first lattice column of the strip's column tile
    if constexpr (CT) {
        const int rs = (int)fd_div((uint32_t)strip, p.div_ncolt);
        q0 = (strip - rs * p.ncolt) * p.BW;
        strip = rs;
    }
    const int n0 = grp * p.TN;
    const int p0 = strip * p.TP;
    const int k0 = by * 64;

    const int CB = p.Cin >> 4;
    const int HWin = p.Hin * p.Win;
    const int xplane = p.xpitch;
    // filter planes of a stage: (tap, g) planes of 64 output channels, or one plane per tap (HALF)
    constexpr int wstride_t = HALF ? STRIP_WPITCH : 2 * STRIP_WPITCH;
    constexpr int wstride_g = HALF ? 512 : STRIP_WPITCH;
    // A stage of the LDS ring holds cps chunks (1, or 2 for small strips: half as many barriers where a chunk is only a
    // few hundred MFMA cycles per wave); sub_bytes = one chunk's patch planes and filter planes.
    const int cps = (!R3 && p.cps == 2) ? 2 : 1;
    const int sub_bytes = 2 * xplane + p.ntaps * wstride_t;
    const int stage_bytes = cps * sub_bytes;

    __amdgpu_buffer_rsrc_t rs_in = __builtin_amdgcn_make_buffer_rsrc((void *)p.in, 0, (int)p.in_bytes, 0x00020000);
    __amdgpu_buffer_rsrc_t rs_wt = __builtin_amdgcn_make_buffer_rsrc((void *)p.wt, 0, (int)p.wt_bytes, 0x00020000);

    // bias values of this lane's channels
    float4 bv[2][2][2];                                   // [a][h][which quad]
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            bv[a][h][0] = bv[a][h][1] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (p.bias && k0 + a * 32 + 16 * h < p.Cout) {       // the last 64-channel tile may be partial (Cout % 16 == 0)
                bv[a][h][0] = *reinterpret_cast<const float4 *>(p.bias + k0 + a * 32 + 16 * h + 4 * lg);
                bv[a][h][1] = *reinterpret_cast<const float4 *>(p.bias + k0 + a * 32 + 16 * h + 8 + 4 * lg);
            }
        }

    // ---- loader bookkeeping: wave w loads patch blocks b = w, w+4, ... of both planes
    const int nblocks = (p.npatch + 63) >> 6;
    unsigned xoff[MAXXB];
    int xz[R3 ? MAXXB : 1];                              // R3: input slice of the pixel's image at depth offset 0
#pragma unroll
    for (int i = 0; i < MAXXB; ++i) {
        const int b = wave + NW * i;
        const uint32_t pi = (uint32_t)(b * 64 + lane);
        unsigned off = STRIP_OOB;
        if (R3) xz[R3 ? i : 0] = 0;
        if (b < nblocks && pi < (uint32_t)p.npatch) {
            const uint32_t ti = fd_div(pi, p.div_prpc);
            const uint32_t rem = pi - ti * p.div_prpc.d;
            const uint32_t pr = fd_div(rem, p.div_pc);
            const uint32_t pc = rem - pr * p.div_pc.d;
            const int n = n0 + (int)ti;
            const int h = p0 * p.sh + p.min_dh + (int)pr;
            const int w = (CT ? q0 * p.sw : 0) + p.min_dw + (int)pc;
            if (n < p.N && (unsigned)h < (unsigned)p.Hin && (unsigned)w < (unsigned)p.Win) {
                if constexpr (R3) {
                    const int nb = (int)fd_div((uint32_t)n, p.div_od);
                    xz[i] = (n - nb * p.OD) * p.is_d;
                    off = (unsigned)((nb * CB * p.Din * HWin + h * p.Win + w) * 32);      // without the depth slice
                } else {
                    off = (unsigned)((n * CB * HWin + h * p.Win + w) * 32);
                }
            }
        }
        xoff[i] = off;
    }
    // Row of the filter slab.  Rows past Cout (partial last tile) get the out-of-range constant and read as zeros:
    // only this per-lane offset takes part in the range check of a buffer load, the scalar slab / chunk offset is
    // added to the base unchecked, so a row index past the slab would read the next slab or past the tensor.
    const unsigned woff_lane = (k0 + lane < p.Cout) ? (unsigned)((k0 + lane) * 32) : STRIP_OOB;
    // fragments of this wave that hold at least one position of the strip (wave-uniform)
    int nfrag = 0;
#pragma unroll
    for (int i = 0; i < NF; ++i) nfrag += ((wave + NW * i) * 32 < p.npix) ? 1 : 0;
    // blocked rank-2 output below 2 GiB: the epilogue that stores through a buffer descriptor
    const bool store32 = !R3 && SUB == 0 && p.out_bytes != 0;
    // Shared last fragment.  The fragments are dealt round-robin, so with NW (NF - 1) + r of them waves 0 .. r - 1 hold
    // NF and the others NF - 1.  When r is 1 or 5 exactly one SIMD carries one fragment more than every other (the 784
    // positions of 14 rows of 56 are 24.5 fragments: 7 against 6, 6, 6).  The two 32-channel halves of the last fragment
    // then go to its owner, wave r - 1, and to wave r on the next SIMD (6.5 / 6.5 / 6 / 6): slot NF - 1 of both waves is
    // fragment nfrag_all - 1, tile 0 of the slot holds channel half hsel = wave - owner.
    const int nfrag_all = (p.npix + 31) >> 5;
    const int r_extra = nfrag_all - NW * (NF - 1);
    const bool split = SUB == 0 && !DB && !R3 && NF > 1 && store32 && p.frag_split != 0 && r_extra >= 1 && r_extra < NW &&
                       (r_extra & 3) == 1;
    const int owner = r_extra - 1;
    const bool half_slot = split && (wave == owner || wave == owner + 1);
    const int hsel = half_slot ? wave - owner : 0;

    // R3: the loads are issued chunk after chunk; (ld_td, ld_cb) is the (depth tap, channel chunk) pair of the next call
    int ld_td = 0, ld_cb = 0;
    auto issue_loads = [&](int chunk, int stage, int sub) {
        unsigned char *xs = smem + stage * stage_bytes + sub * sub_bytes;
        unsigned char *ws = xs + 2 * xplane;
        if constexpr (R3) chunk = ld_cb;
        const unsigned soff_x = (unsigned)(chunk * (R3 ? p.Din * HWin : HWin) * 32);
        int dz = 0, slab0 = 0;
        if constexpr (R3) {
            dz = p.dt_off[ld_td];
            slab0 = p.dt_slab[ld_td];
        }
#pragma unroll
        for (int i = 0; i < MAXXB; ++i) {
            const int b = wave + NW * i;
            if (b < nblocks) {                                           // wave-uniform
                unsigned base = xoff[i];
                if constexpr (R3) {
                    const int z = xz[i] + dz;
                    base = (base == STRIP_OOB || (unsigned)z >= (unsigned)p.Din) ? STRIP_OOB : base + (unsigned)(z * HWin * 32);
                }
#pragma unroll
                for (int g = 0; g < 2; ++g) {
                    const unsigned v = (base == STRIP_OOB) ? STRIP_OOB : base + 16 * g;
                    load_lds16(rs_in, xs + g * xplane + b * 1024, v, soff_x);
                }
            }
        }
        if (HALF) {
            for (int t = wave; t < p.ntaps; t += NW) {                   // lanes 0-31: g = 0, lanes 32-63: g = 1
                const unsigned soff_w = (unsigned)(((p.tap_slab[t] * CB + chunk) * p.Cout) * 32);
                load_lds16(rs_wt, ws + t * STRIP_WPITCH, (k0 + l32 < p.Cout) ? (unsigned)((k0 + l32) * 32 + lg * 16) : STRIP_OOB,
                           soff_w);
            }
        } else {
            for (int j = wave; j < 2 * p.ntaps; j += NW) {                // plane j = tap*2 + g
                const int t = j >> 1, g = j & 1;
                const unsigned soff_w = (unsigned)((((slab0 + p.tap_slab[t]) * CB + chunk) * p.Cout) * 32 + 16 * g);
                load_lds16(rs_wt, ws + j * STRIP_WPITCH, woff_lane, soff_w);
            }
        }
        if constexpr (R3) {
            if (++ld_cb == CB) { ld_cb = 0; ++ld_td; }
        }
    };

    // The first chunk is requested before anything else is set up: position tables and initial accumulators cost a
    // few hundred vector instructions per wave, which run while the loads are in flight.
    const int nchunks = R3 ? p.ndt * CB : CB;
    const int nstages = (nchunks + cps - 1) / cps;
    auto issue_stage = [&](int s) {
        issue_loads(s * cps, s & 1, 0);
        if (cps == 2 && s * 2 + 1 < nchunks) issue_loads(s * 2 + 1, s & 1, 1);
    };
    STRIP_TL(1);
    issue_stage(0);
    STRIP_TL(2);

    // ---- positions owned by this lane: fragment f = wave + 4 i, position m = 32 f + l32
    int pbase[NF];          // patch pixel index of the position at tap offset 0 (clamped to 0 if invalid)
#pragma unroll
    for (int i = 0; i < NF; ++i) {
        const int frag = (half_slot && i == NF - 1) ? nfrag_all - 1 : wave + NW * i;
        const uint32_t m = (uint32_t)(frag * 32 + l32);
        int pb = 0;
        if (m < (uint32_t)p.npix) {
            const uint32_t ti = fd_div(m, p.div_tpq);
            const uint32_t rem = m - ti * p.div_tpq.d;
            const uint32_t tp = fd_div(rem, p.div_q);
            const uint32_t q = rem - tp * p.div_q.d;
            pb = (int)((ti * p.PR + tp * p.sh) * p.PC + q * p.sw);
        }
        pbase[i] = pb * 16;
    }

    // Blocked output: the accumulators start from the bias (register 8 h + e of channel half a holds the channel of
    // bv[a][h][e / 4], component e % 4), so the epilogue has no additions and the bias registers are free during the
    // chunk loop.  The sub-pixel store modes take no bias.
    f32x16 acc[NF][2];
#pragma unroll
    for (int i = 0; i < NF; ++i)
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float4 b0 = bv[a][h][0], b1 = bv[a][h][1];
                if (NF > 1 && i == NF - 1 && a == 0 && hsel) {           // wave-uniform
                    b0 = bv[1][h][0];
                    b1 = bv[1][h][1];
                }
                const float bias8[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[i][a][8 * h + e] = SUB == 0 ? bias8[e] : 0.f;
            }

    // Blocked rank-2 output below 2 GiB: 16-byte stores with 32-bit offsets into a buffer descriptor, lanes that
    // must not store get an out-of-range offset (no 64-bit address arithmetic, no divergent branch per store).
    const int CBout = p.Cout >> 4;
    const int HWout = p.Hfull * p.Wfull;
    const int plane_out = R3 ? p.Dfull * HWout : HWout;  // pixel blocks per 16-channel plane of a batch element
    const bool dense_out = p.os_h == 1 && p.os_w == 1;     // every pixel written: whole cache lines, streaming stores
    __amdgpu_buffer_rsrc_t rs_out = __builtin_amdgcn_make_buffer_rsrc((void *)p.out, 0, (int)p.out_bytes, 0x00020000);
    const int relu_on = p.relu;
    const bool has_mask = p.mask != nullptr;
    __amdgpu_buffer_rsrc_t rs_mask = __builtin_amdgcn_make_buffer_rsrc((void *)p.mask, 0, has_mask ? (int)p.out_bytes : 0, 0x00020000);
    // ReLU on the rounded values, two at a time (relu_bf16x2)
    const bool relu_b = relu_on != 0;
    // Epilogue of fragment i on that path (the bias is in the accumulators): one rounding, ReLU, lane-pair exchange,
    // stores.  STREAM: every pixel of the tensor is written by this launch, the stores are streaming stores.
    // SHARED: slot i is the shared fragment; its tile 0 goes to channel half hsel, there is no tile 1.
    auto store_frag32 = [&](const int i, auto stream_tag, auto shared_tag) {
        constexpr bool STREAM = decltype(stream_tag)::value;
        constexpr bool SHARED = decltype(shared_tag)::value;
        const uint32_t m = (uint32_t)((SHARED ? nfrag_all - 1 : wave + NW * i) * 32 + l32);
        bool ok = m < (uint32_t)p.npix;
        const uint32_t mm = ok ? m : 0;
        const uint32_t ti = fd_div(mm, p.div_tpq);
        const uint32_t rem = mm - ti * p.div_tpq.d;
        const uint32_t tp = fd_div(rem, p.div_q);
        const uint32_t q = rem - tp * p.div_q.d;
        const int n = n0 + (int)ti;
        const int oh = p0 + (int)tp;
        ok = ok && n < p.N && oh < p.Hout;
        if constexpr (CT) ok = ok && q0 + (int)q < p.Wout;
        const unsigned pix = (unsigned)((oh * p.os_h + p.oa_h) * p.Wfull + ((CT ? q0 : 0) + (int)q) * p.os_w + p.oa_w) +
                             (unsigned)(n * CBout * HWout);
        const unsigned off0 = ok ? (pix + (unsigned)((k0 >> 4) * plane_out)) * 32u + (unsigned)(lg * 16) : STRIP_OOB;
#pragma unroll
        for (int a = 0; a < (SHARED ? 1 : 2); ++a) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const f32x16 &t = acc[i][a];
                const uint32_t w0 = relu_bf16x2(pack_bf16x2_hw(t[8 * h], t[8 * h + 1]), relu_b);
                const uint32_t w1 = relu_bf16x2(pack_bf16x2_hw(t[8 * h + 2], t[8 * h + 3]), relu_b);
                const uint32_t w2 = relu_bf16x2(pack_bf16x2_hw(t[8 * h + 4], t[8 * h + 5]), relu_b);
                const uint32_t w3 = relu_bf16x2(pack_bf16x2_hw(t[8 * h + 6], t[8 * h + 7]), relu_b);
                uint4 o = lane_pair_exchange(w0, w1, w2, w3);
                const int cb = 2 * (SHARED ? hsel : a) + h;              // 16-channel block inside the tile
                const bool st = off0 != STRIP_OOB && (k0 >> 4) + cb < CBout;
                const unsigned off = st ? off0 + (unsigned)(cb * plane_out) * 32u : STRIP_OOB;
                if (has_mask) {                                          // same shape and layout as the stored tensor
                    const ngc_u32x4 mk = __builtin_amdgcn_raw_buffer_load_b128(rs_mask, (int)off, 0, 0);
                    o = relu_keep8(o, make_uint4(mk[0], mk[1], mk[2], mk[3]));
                }
                ngc_u32x4 ov = {o.x, o.y, o.z, o.w};
                if constexpr (STREAM) __builtin_amdgcn_raw_buffer_store_b128(ov, rs_out, (int)off, 0, NGC_ST_AUX);
                else __builtin_amdgcn_raw_buffer_store_b128(ov, rs_out, (int)off, 0, 0);
            }
        }
    };
    // the last chunk runs fragment-outer with the epilogues inside it (strip_chunk_mfma_last)
    const bool tail_fuse = SUB == 0 && !DB && !R3 && store32 && dense_out && p.tail_fuse != 0;

    // the sub-pixel store mode may use no more than 32 of the 64 output columns: skip the upper MFMA
    constexpr bool upper = !HALF;
    // Waves that hold every fragment, or all but the last, run chunk loops with the software-pipelined MFMA
    // sequence; the others (ragged strips) the loop that tests every fragment.  NFR = 0 selects the latter.
    static_assert(STRIP_MAX_TAPS <= 64, "one lane per tap");
    const int tapv = p.tap_off[lane < p.ntaps ? lane : 0] * 16;
    auto chunk_loop = [&](auto nfr_tag, auto hs_tag) -> bool {
        constexpr int NFR = decltype(nfr_tag)::value;
        constexpr bool HS = decltype(hs_tag)::value;
        const bool tail = NFR > 0 && tail_fuse;
        const int last = nchunks - 1;
        for (int sg = 0; sg < nstages; ++sg) {
            const int c0 = sg * cps;
            if (tail && c0 == last) break;                  // this stage holds nothing but the tail chunk: below
            __builtin_amdgcn_s_waitcnt(0x0F70);             // vmcnt(0): this wave's loads of stage sg have landed
            __syncthreads();                                // ... and everybody else's; stage (sg+1)&1 is free
#ifdef NGC_TIMELINE
            if (sg < 5) { if (sg == 0) STRIP_TL(3); else if (sg == 1) STRIP_TL(4); else if (sg == 2) STRIP_TL(5); else if (sg == 3) STRIP_TL(6); else STRIP_TL(7); }
#endif
            if (sg + 1 < nstages) issue_stage(sg + 1);
            for (int u = 0; u < cps; ++u) {
                const int c = c0 + u;
                if (c > last || (tail && c == last)) break;
                const unsigned char *xs = smem + (sg & 1) * stage_bytes + u * sub_bytes + lg * xplane;
                const unsigned char *ws = smem + (sg & 1) * stage_bytes + u * sub_bytes + 2 * xplane + lg * wstride_g + l32 * 16;
                if constexpr (NFR > 0) {
                    strip_chunk_mfma<NF, NFR, HS, upper, wstride_t>(acc, xs, ws, ws + hsel * (32 * 16), pbase, tapv, p.ntaps);
                } else {
                    for (int t = 0; t < p.ntaps; ++t) {
                        const bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(ws + t * wstride_t);
                        bf16x8 a1 = a0;
                        if (upper) a1 = *reinterpret_cast<const bf16x8 *>(ws + t * wstride_t + 32 * 16);
                        const int toff = p.tap_off[t] * 16;
#pragma unroll
                        for (int i = 0; i < NF; ++i) {
                            if (i < nfrag) {
                                const bf16x8 b = *reinterpret_cast<const bf16x8 *>(xs + pbase[i] + toff);
                                acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b, acc[i][0], 0, 0, 0);
                                if (upper) acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b, acc[i][1], 0, 0, 0);
                            }
                        }
                    }
                }
            }
        }
        if constexpr (NFR > 0 && SUB == 0 && !DB && !R3) {
            if (tail) {                                     // last chunk, with the epilogues inside it
                const int sg = last / cps, u = last - sg * cps;
                if (u == 0) {                               // its stage has not been opened yet
                    __builtin_amdgcn_s_waitcnt(0x0F70);
                    __syncthreads();
                }
                STRIP_TL(8);
                const unsigned char *xs = smem + (sg & 1) * stage_bytes + u * sub_bytes + lg * xplane;
                const unsigned char *ws = smem + (sg & 1) * stage_bytes + u * sub_bytes + 2 * xplane + lg * wstride_g + l32 * 16;
                strip_chunk_mfma_last<NF, NFR, HS, upper, wstride_t>(
                    acc, xs, ws, ws + hsel * (32 * 16), pbase, tapv, p.ntaps,
                    [&](const int i) { store_frag32(i, std::true_type{}, std::false_type{}); },
                    [&]() { store_frag32(NF - 1, std::true_type{}, std::true_type{}); });
                STRIP_TL(10);
#ifdef NGC_TIMELINE
                tl_flush();
#endif
                return true;
            }
        }
        return false;
    };
    constexpr bool CAN_SPLIT = SUB == 0 && !DB && !R3 && NF > 1;
    if (CAN_SPLIT && half_slot) {
        if (chunk_loop(std::integral_constant<int, (NF > 1 ? NF - 1 : 1)>{}, std::integral_constant<bool, CAN_SPLIT>{})) return;
    } else if (nfrag == NF) {
        if (chunk_loop(std::integral_constant<int, NF>{}, std::false_type{})) return;
    } else if (NF > 1 && nfrag == NF - 1) {
        if (chunk_loop(std::integral_constant<int, (NF > 1 ? NF - 1 : 0)>{}, std::false_type{})) return;
    } else {
        chunk_loop(std::integral_constant<int, 0>{}, std::false_type{});
    }

    // ---- epilogue
    float csum[DB ? 2 : 1][2][8];                         // DB: channel sums of this lane's stored values
#pragma unroll
    for (int a = 0; a < (DB ? 2 : 1); ++a)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int e = 0; e < 8; ++e) csum[a][h][e] = 0.f;
    if (SUB != 0 && p.sub_stage) {
        // Sub-pixel NCHW store through LDS: column col = (a*BW+b)*C + c of position (tp, q) of image ti is
        // pixel (BH tp + a, BW q + b) of channel c; the strip's pixels are assembled as [ti][c][row][WP]
        // in LDS (the stage buffers are free now) and written out as whole rows with 16-byte stores
        // (scattered 2-byte stores cost a wave hundreds of cycles each).
        __syncthreads();
        uint16_t *ob = reinterpret_cast<uint16_t *>(smem);
        const int ROWS = p.sub_BH * p.TP, WP = p.sub_BW * p.Wout;
        // element offsets of this lane's 16 (32) columns inside a position's block: the column of
        // accumulator register v is a*32 + 8*(v/4) + 4*lg + v%4 (table from the host, -1 = padding)
        constexpr int NA = HALF ? 1 : 2;
        int coff[NA][16];
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int c0 = a * 32 + 8 * (v >> 2) + (v & 3);
                coff[a][v] = lg ? p.sub_off[c0 + 4] : p.sub_off[c0];
            }
#pragma unroll
        for (int i = 0; i < NF; ++i) {
            if (i >= nfrag) break;
            const uint32_t m = (uint32_t)((wave + NW * i) * 32 + l32);
            const bool ok = m < (uint32_t)p.npix;
            const uint32_t mm = ok ? m : 0;
            const uint32_t ti = fd_div(mm, p.div_tpq);
            const uint32_t rem = mm - ti * p.div_tpq.d;
            const uint32_t tp = fd_div(rem, p.div_q);
            const uint32_t q = rem - tp * p.div_q.d;
            const int base = ((int)ti * p.sub_C * ROWS + p.sub_BH * (int)tp) * WP + p.sub_BW * (int)q;
#pragma unroll
            for (int a = 0; a < NA; ++a)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (ok && coff[a][v] >= 0)
                        ob[base + coff[a][v]] = (uint16_t)(pack_bf16x2_hw(acc[i][a][v], 0.f) & 0xFFFFu);
        }
        __syncthreads();
        // rows of the strip: (ti, c, lrow) -> global row ((n0+ti)*C + c, BH*p0 + lrow); sub_W % 8 == 0
        const int chunks = p.sub_W >> 3;                                 // 16-byte pieces per row
        const int nrows = p.TN * p.sub_C * ROWS;
        const int vrows = p.sub_BH * (p.Hout - p0 < p.TP ? p.Hout - p0 : p.TP);
        for (int e = tid; e < nrows * chunks; e += NW * 64) {
            const int row = (int)fd_div((uint32_t)e, p.div_chunks), ch = e - row * chunks;
            const int tc = (int)fd_div((uint32_t)row, p.div_rows), lrow = row - tc * ROWS;
            const int ti = (int)fd_div((uint32_t)tc, p.div_subc), c = tc - ti * p.sub_C;
            const int n = n0 + ti, y = p.sub_BH * p0 + lrow;
            if (n < p.N && y < p.sub_H && lrow < vrows) {
                uint4 val = *reinterpret_cast<const uint4 *>(ob + (size_t)row * WP + ch * 8);
                const size_t off = (((size_t)n * p.sub_C + c) * p.sub_H + y) * p.sub_W + ch * 8;
                if (p.mask) val = relu_keep8(val, *reinterpret_cast<const uint4 *>(p.mask + off));
                store16_result(p.out + off, val, true);
            }
        }
        return;
    }
    if (store32 && !DB) {
        STRIP_TL(9);
        const int nfull = half_slot ? NF - 1 : nfrag;
        if (dense_out) {
#pragma unroll
            for (int i = 0; i < NF; ++i)
                if (i < nfull) store_frag32(i, std::true_type{}, std::false_type{});
            if (NF > 1 && half_slot) store_frag32(NF - 1, std::true_type{}, std::true_type{});
        } else {
#pragma unroll
            for (int i = 0; i < NF; ++i)
                if (i < nfull) store_frag32(i, std::false_type{}, std::false_type{});
            if (NF > 1 && half_slot) store_frag32(NF - 1, std::false_type{}, std::true_type{});
        }
        STRIP_TL(10);
#ifdef NGC_TIMELINE
        tl_flush();
#endif
        return;
    }
#pragma unroll
    for (int i = 0; i < NF; ++i) {
        if (i >= nfrag) break;
        const uint32_t m = (uint32_t)((wave + NW * i) * 32 + l32);
        bool ok = m < (uint32_t)p.npix;
        const uint32_t mm = ok ? m : 0;
        const uint32_t ti = fd_div(mm, p.div_tpq);
        const uint32_t rem = mm - ti * p.div_tpq.d;
        const uint32_t tp = fd_div(rem, p.div_q);
        const uint32_t q = rem - tp * p.div_q.d;
        const int n = n0 + (int)ti;
        const int oh = p0 + (int)tp;
        ok = ok && n < p.N && oh < p.Hout;
        size_t pix;
        if constexpr (CT) {
            ok = ok && q0 + (int)q < p.Wout;
            pix = (size_t)(oh * p.os_h + p.oa_h) * p.Wfull + ((q0 + (int)q) * p.os_w + p.oa_w);
        } else {
            pix = (size_t)(oh * p.os_h + p.oa_h) * p.Wfull + (q * p.os_w + p.oa_w);
        }
        if constexpr (R3) {
            const int nb = (int)fd_div((uint32_t)(ok ? n : 0), p.div_od);
            const int o = (ok ? n : 0) - nb * p.OD;
            pix += (size_t)nb * CBout * plane_out + (size_t)(o * p.os_d + p.oa_d) * HWout;
        } else {
            pix += (size_t)n * CBout * HWout;
        }
        if (SUB != 0) {
            // sub-pixel NCHW store: column col = (a*BW+b)*C + c -> pixel (BH oh + a, BW q + b) of channel c
            const int ncol = p.sub_BH * p.sub_BW * p.sub_C;
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int col = k0 + a * 32 + 8 * (v >> 2) + 4 * lg + (v & 3);
                    if (ok && col < ncol) {
                        const int ab = col / p.sub_C, c = col - ab * p.sub_C;
                        const int a2 = ab / p.sub_BW;
                        const int hh = p.sub_BH * oh + a2, ww = p.sub_BW * (int)q + (ab - a2 * p.sub_BW);
                        if (hh < p.sub_H && ww < p.sub_W) {
                            const size_t off = (((size_t)n * p.sub_C + c) * p.sub_H + hh) * p.sub_W + ww;
                            uint32_t bits = pack_bf16x2_hw(acc[i][a][v], 0.f) & 0xFFFFu;
                            if (p.mask) bits = relu_keep2(bits, p.mask[off]);
                            p.out[off] = (uint16_t)bits;
                        }
                    }
                }
            continue;
        }
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            const int co_base = k0 + a * 32;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = acc[i][a][8 * h + e];      // bias included
                const uint32_t q0 = relu_bf16x2(pack_bf16x2_hw(v[0], v[1]), relu_on != 0), q1 = relu_bf16x2(pack_bf16x2_hw(v[2], v[3]), relu_on != 0);
                const uint32_t q2 = relu_bf16x2(pack_bf16x2_hw(v[4], v[5]), relu_on != 0), q3 = relu_bf16x2(pack_bf16x2_hw(v[6], v[7]), relu_on != 0);
                uint4 o = lane_pair_exchange(q0, q1, q2, q3);
                if (ok && (co_base >> 4) + h < CBout) {
                    const size_t blk = pix + (size_t)((co_base >> 4) + h) * plane_out;
                    if (p.mask) o = relu_keep8(o, *reinterpret_cast<const uint4 *>(p.mask + blk * 16 + lg * 8));
                    store16_result(p.out + blk * 16 + lg * 8, o, dense_out);
                    if (DB) {                                            // the rounded, masked values as stored
                        const uint32_t w4[4] = {o.x, o.y, o.z, o.w};
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            csum[DB ? a : 0][h][2 * j] += __uint_as_float(w4[j] << 16);
                            csum[DB ? a : 0][h][2 * j + 1] += __uint_as_float(w4[j] & 0xFFFF0000u);
                        }
                    }
                }
            }
        }
    }
    if (DB) {
        // lanes of a 32-lane half hold different positions of the same 8 channels: transpose-sum over the
        // half (no LDS, no barrier: a wave that is done leaves), one row of 64 channel sums per wave;
        // value index j = a*16 + h*8 + e is channel k0 + a*32 + 16 h + 8 lg + e
        float flat[32];
#pragma unroll
        for (int j = 0; j < 32; ++j) flat[j] = csum[DB ? (j >> 4) : 0][(j >> 3) & 1][j & 7];
        const float mine = half_wave_transpose_sum32(flat, l32);
        const int j = ((l32 & 15) << 1) | (l32 >> 4);
        const int ch = k0 + (j >> 4) * 32 + ((j >> 3) & 1) * 16 + 8 * lg + (j & 7);
        if (ch < p.Cout) p.dbp[((size_t)(p.dbp_row0 + bx) * NW + wave) * p.dbp_ld + ch] = mine;
    }
}


template <int NF, int NW, int SUB = 0, bool DB = false, bool R3 = false, bool CT = false>
__global__ __launch_bounds__(NW * 64) void conv_strip_bf16(const StripParams p)
{
    preload_kernargs(p);
    if (p.xcd_order) {
        // one-dimensional grid: workgroup ids go round-robin to the 8 XCDs (one L2 each); strip bx lives on XCD
        // bx % 8 and its output-channel tiles are consecutive there, so they share the strip's input through that L2
        const int nk = (p.Cout + 63) >> 6;
        const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
        const int sl = j / nk;
        const int bx = sl * 8 + xcd;
        if (bx >= p.groups * p.strips) return;           // uniform per workgroup
        conv_strip_body<NF, NW, SUB, DB, R3, CT>(p, bx, j - sl * nk);
        return;
    }
    conv_strip_body<NF, NW, SUB, DB, R3, CT>(p, blockIdx.x, blockIdx.y);
}

// Several launches of the kernel above in one grid (the residue classes of a strided backprop-data: each has
// its own tap list and geometry): workgroups [wg_end[i-1], wg_end[i]) run launch i.  Small classes then share
// the chip with large ones instead of leaving it half empty, and three launch gaps go away.
template <int NF, int NW, bool DB, bool R3 = false>
__global__ __launch_bounds__(NW * 64) void conv_strip_multi_bf16(const StripMulti mp)
{
    int cls = 0;
    while (cls + 1 < mp.n && (int)blockIdx.x >= mp.wg_end[cls]) ++cls;   // uniform per workgroup
    const int bx = (int)blockIdx.x - (cls ? mp.wg_end[cls - 1] : 0);
    preload_kernargs(mp.c[cls]);
    conv_strip_body<NF, NW, 0, DB, R3>(mp.c[cls], bx, blockIdx.y);
}

template <int NF, int NW, int SUB, bool DB, bool R3 = false, bool CT = false>
static hipError_t launch_strip_d(const StripParams &p, size_t lds_bytes, hipStream_t st)
{
    static LdsLimitOnce lds_limit;                  // per template instantiation
    {
        const hipError_t e = lds_limit.raise(reinterpret_cast<const void *>(&conv_strip_bf16<NF, NW, SUB, DB, R3, CT>));
        if (e != hipSuccess) return e;
    }
    dim3 grid(p.groups * p.strips, (p.Cout + 63) / 64);
    if (p.xcd_order) grid = dim3(8 * ((p.groups * p.strips + 7) / 8) * ((p.Cout + 63) / 64));
    NGC_LAUNCH((conv_strip_bf16<NF, NW, SUB, DB, R3, CT>), grid, dim3(NW * 64), lds_bytes, st, p);
    return ngc::launch_result();
}

template <int NF, bool DB, bool R3 = false>
static hipError_t launch_strip_multi_t(const StripMulti &mp, size_t lds_bytes, hipStream_t st)
{
    static LdsLimitOnce lds_limit;
    {
        const hipError_t e = lds_limit.raise(reinterpret_cast<const void *>(&conv_strip_multi_bf16<NF, 8, DB, R3>));
        if (e != hipSuccess) return e;
    }
    dim3 grid(mp.wg_end[mp.n - 1], (mp.c[0].Cout + 63) / 64);
    NGC_LAUNCH((conv_strip_multi_bf16<NF, 8, DB, R3>), grid, dim3(8 * 64), lds_bytes, st, mp);
    return ngc::launch_result();
}

// rank-3 launches: defined in conv_strip3.hip
hipError_t launch_strip_r3(const StripParams &p, int nf, size_t lds_bytes, hipStream_t st);
hipError_t launch_strip_multi_r3(const StripMulti &mp, int nf, size_t lds_bytes, hipStream_t st);

}  // namespace ngc
