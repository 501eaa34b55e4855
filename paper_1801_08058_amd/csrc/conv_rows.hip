// Stride-1 multi-tap convolution (forward, or backprop-data of a stride-1 node) for filters that fit the LDS:
// the filter-resident form of the strip kernel (conv_strip_kernels.h), bf16 MFMA, fp32 accumulate (gfx950).
//
// A workgroup (512 threads, two waves per SIMD) owns TP output rows of one image for 64 output channels.  All
// taps x all input channels x 64 output channels of the filter are brought into LDS once and stay there.  The
// strip is worked off in sub-strips of SRB rows (at most 512 positions); a sub-strip runs over the 16-input-
// channel chunks, and the (sub-strip, chunk) pairs of the whole strip form one flat sequence of stages whose
// input patches stream through a ring of three LDS buffers with direct global->LDS loads, two stages ahead.
// So the loads of the next sub-strip are in flight during the last chunks of the current one, and the stores
// of a finished sub-strip drain while the next one's MFMAs run: only the first stage's loads and the last
// sub-strip's stores are not covered by MFMA work.
//
// MFMA roles, LDS plane layouts and the epilogue (bias, ReLU, one RNE rounding, lane-pair exchange, 16-byte
// stores) are those of the strip kernel.  The 32-position fragments of a sub-strip are dealt to the SIMDs so
// that their tile counts differ by at most one: whole fragments (both 32-channel halves, sharing the
// activation operand) first, the left-over fragments split into their two halves.
#include "conv_strip_kernels.h"

namespace ngc {

namespace {

#ifdef NGC_TIMELINE
// development builds only: time stamps (100 MHz counter) of lane 0 of every wave, 64 slots per wave, kept in the
// 4 KB of LDS behind the kernel's own buffers while the kernel runs (no global stores that the counted waits
// would see) and written out at the end
__device__ unsigned long long g_rows_timeline[1024 * 8 * 64];
#define ROWS_TL()                                                                                          \
    do {                                                                                                   \
        if (lane == 0 && tl_n < 64) tl_lds[wave * 64 + tl_n] = wall_clock64();                             \
        ++tl_n;                                                                                            \
    } while (0)
#else
#define ROWS_TL() do { } while (0)
#endif

constexpr int ROWS_NW = 8;
constexpr int ROWS_MAXXB = STRIP_MAXBLOCKS / ROWS_NW;      // patch blocks per wave

// MFMAs of one stage (one 16-channel chunk, NT taps) for a wave that holds NFULL whole fragments (both channel
// halves) and, if HALF, one half fragment (channel half ha).  The tap loop is unrolled and the LDS reads of tap
// t + 2 are issued before the MFMAs of tap t, through a ring of three operand sets (a wave with one or two
// fragments has only 64-128 MFMA cycles per tap to cover an LDS read, less than its latency under load; two taps
// are enough).  toff[t] = patch byte offset of tap t.
template <int NFULL, bool HALF, int NT>
__device__ __forceinline__ void rows_stage_mfma_nt(f32x16 (&acc)[2][2], f32x16 &acch, const unsigned char *xs, const unsigned char *ws,
                                                   const int (&pb)[2], const int pbh, const int ha, const int (&toff)[NT])
{
    constexpr int WT = 2 * STRIP_WPITCH;
    constexpr int NB = NFULL > 0 ? NFULL : 1;
    bf16x8 a0[3], a1[3], ah[3], b[3][NB], bh[3];
    auto fetch = [&](int t, int r) {
        if (NFULL > 0) {
            a0[r] = *reinterpret_cast<const bf16x8 *>(ws + t * WT);
            a1[r] = *reinterpret_cast<const bf16x8 *>(ws + t * WT + 32 * 16);
        }
        if (HALF) ah[r] = *reinterpret_cast<const bf16x8 *>(ws + t * WT + ha * (32 * 16));
#pragma unroll
        for (int i = 0; i < NFULL; ++i) b[r][i] = *reinterpret_cast<const bf16x8 *>(xs + pb[i] + toff[t]);
        if (HALF) bh[r] = *reinterpret_cast<const bf16x8 *>(xs + pbh + toff[t]);
    };
    fetch(0, 0);
    if (NT > 1) fetch(1, 1);
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int r = t % 3;
        if (t + 2 < NT) fetch(t + 2, (t + 2) % 3);
#pragma unroll
        for (int i = 0; i < NFULL; ++i) {
            acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[r], b[r][i], acc[i][0], 0, 0, 0);
            acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[r], b[r][i], acc[i][1], 0, 0, 0);
        }
        if (HALF) acch = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[r], bh[r], acch, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
}

__global__ __launch_bounds__(ROWS_NW * 64) void conv_rows_bf16(const RowsParams p)
{
    constexpr int NW = ROWS_NW;
    extern __shared__ __align__(16) unsigned char smem[];

    // All kernel arguments are fetched at once: left to itself the compiler loads them where they are first used,
    // and every such group costs a wave a round trip to memory at a point where nothing else can hide it (the start
    // of the kernel, the set-up of a sub-strip).
#define ROWS_PRELOAD(x) asm volatile("" ::"s"(x))
    {
        ROWS_PRELOAD(p.N); ROWS_PRELOAD(p.Cin); ROWS_PRELOAD(p.Hin); ROWS_PRELOAD(p.Win); ROWS_PRELOAD(p.Cout);
        ROWS_PRELOAD(p.Hout); ROWS_PRELOAD(p.Wout); ROWS_PRELOAD(p.TP); ROWS_PRELOAD(p.strips); ROWS_PRELOAD(p.SRB);
        ROWS_PRELOAD(p.PC); ROWS_PRELOAD(p.min_dh); ROWS_PRELOAD(p.min_dw); ROWS_PRELOAD(p.span_h); ROWS_PRELOAD(p.nblocks);
        ROWS_PRELOAD(p.xpitch); ROWS_PRELOAD(p.relu); ROWS_PRELOAD(p.ntaps); ROWS_PRELOAD(p.in_bytes); ROWS_PRELOAD(p.wt_bytes);
        ROWS_PRELOAD(p.out_bytes); ROWS_PRELOAD(p.late_mask);
        ROWS_PRELOAD(p.div_q.mul); ROWS_PRELOAD(p.div_q.sh1); ROWS_PRELOAD(p.div_q.sh2); ROWS_PRELOAD(p.div_q.d);
        ROWS_PRELOAD(p.div_pc.mul); ROWS_PRELOAD(p.div_pc.sh1); ROWS_PRELOAD(p.div_pc.sh2); ROWS_PRELOAD(p.div_pc.d);
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            ROWS_PRELOAD(p.tap_off[t]);
            ROWS_PRELOAD(p.tap_slab[t]);
        }
    }
#undef ROWS_PRELOAD
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31;
    const int lg = lane >> 5;
#ifdef NGC_TIMELINE
    int tl_n = 0;
    unsigned long long *tl_lds = nullptr;                 // set below, once the LDS sizes are known
#endif

    const int n = blockIdx.x / p.strips;
    const int strip = blockIdx.x - n * p.strips;
    const int p0 = strip * p.TP;
    const int rows_strip = (p.Hout - p0 < p.TP) ? (p.Hout - p0) : p.TP;
    const int k0 = blockIdx.y * 64;

    const int CB = p.Cin >> 4;
    const int HWin = p.Hin * p.Win;
    const int wchunk = p.ntaps * 2 * STRIP_WPITCH;        // filter planes of one 16-channel chunk
    unsigned char *const wbase = smem;
    unsigned char *const xbase = smem + CB * wchunk;
    const int stage_bytes = 2 * p.xpitch;
    const int nsub = (rows_strip + p.SRB - 1) / p.SRB;
    const int nstages = nsub * CB;
#ifdef NGC_TIMELINE
    tl_lds = reinterpret_cast<unsigned long long *>(xbase + ROWS_NBUF * stage_bytes + 256);
    ROWS_TL();
#endif
    // rows of sub-strip js: full sub-strips first, the remainder of the strip last (the stores of the last sub-strip
    // are the only ones no MFMA work covers)
    auto sub_rows = [&](int js, int &r0, int &rows) {
        r0 = js * p.SRB;
        rows = rows_strip - r0 < p.SRB ? rows_strip - r0 : p.SRB;
    };

    // The 64 bias values of the tile go to LDS behind the stage buffers, with a direct global->LDS load of wave 0
    // that belongs to stage 0 (zeros without a bias and for channels past Cout).  The accumulators start from them, so
    // the epilogue is ReLU, rounding and the store.  (An ordinary LDS write after direct loads have been issued
    // would make the compiler wait for every one of them.)
    const int CBout = p.Cout >> 4;
    const int HWout = p.Hout * p.Wout;
    float *const bias_lds = reinterpret_cast<float *>(xbase + ROWS_NBUF * stage_bytes);

    __amdgpu_buffer_rsrc_t rs_in = __builtin_amdgcn_make_buffer_rsrc((void *)p.in, 0, (int)p.in_bytes, 0x00020000);
    __amdgpu_buffer_rsrc_t rs_wt = __builtin_amdgcn_make_buffer_rsrc((void *)p.wt, 0, (int)p.wt_bytes, 0x00020000);
    __amdgpu_buffer_rsrc_t rs_out = __builtin_amdgcn_make_buffer_rsrc((void *)p.out, 0, (int)p.out_bytes, 0x00020000);

    // ---- loader bookkeeping: wave w loads patch blocks b = w, w + 8, ... of both planes.  Per lane and block: the
    // pixel's patch row and its byte offset inside the image at patch row 0 (fixed), and the offset of the load for
    // the sub-strip the load stream is in (xv, recomputed when the stream enters a new sub-strip).
    int xrow[ROWS_MAXXB];
    unsigned xrel[ROWS_MAXXB], xv[ROWS_MAXXB];
    int lx = 0;                                           // x load instructions of this wave per stage (wave-uniform)
#pragma unroll
    for (int i = 0; i < ROWS_MAXXB; ++i) {
        const int b = wave + NW * i;
        const uint32_t pi = (uint32_t)(b * 64 + lane);
        const uint32_t pr = fd_div(pi, p.div_pc);
        const uint32_t pc = pi - pr * p.div_pc.d;
        const int w = p.min_dw + (int)pc;
        xrow[i] = (int)pr;
        xrel[i] = ((unsigned)w < (unsigned)p.Win) ? (unsigned)((n * CB * HWin + (int)pr * p.Win + w) * 32) : STRIP_OOB;
        xv[i] = STRIP_OOB;
        if (b < p.nblocks) lx += 2;
    }
    const unsigned woff_lane = (k0 + lane < p.Cout) ? (unsigned)((k0 + lane) * 32) : STRIP_OOB;
    int lw = 0;                                           // filter load instructions of this wave per chunk
    for (int j = wave; j < 2 * p.ntaps; j += NW) ++lw;

    // loads of the next stage of the load stream, (sub-strip ld_js, chunk ld_c); the first CB stages also bring in
    // their chunk of the filter
    int ld_sg = 0, ld_js = 0, ld_c = 0;
    auto issue_next_stage = [&]() {
        if (ld_sg == 0 && wave == 0) {
            __amdgpu_buffer_rsrc_t rs_b = __builtin_amdgcn_make_buffer_rsrc((void *)p.bias, 0, p.bias ? p.Cout * 4 : 0, 0x00020000);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_b, (lds_void *)bias_lds, 4, (k0 + lane) * 4, 0, 0, 0);
        }
        if (ld_sg < CB) {
            for (int j = wave; j < 2 * p.ntaps; j += NW) {               // plane j = tap * 2 + g
                const int t = j >> 1, g = j & 1;
                const unsigned soff_w = (unsigned)(((p.tap_slab[t] * CB + ld_c) * p.Cout) * 32 + 16 * g);
                load_lds16(rs_wt, wbase + ld_c * wchunk + j * STRIP_WPITCH, woff_lane, soff_w);
            }
        }
        if (ld_c == 0) {
            int r0, rows;
            sub_rows(ld_js, r0, rows);
            const int prows = rows + p.span_h;                           // patch rows this sub-strip reads
            const int h0 = p0 + r0 + p.min_dh;                           // input row of patch row 0
#pragma unroll
            for (int i = 0; i < ROWS_MAXXB; ++i) {
                const int h = h0 + xrow[i];
                const bool ok = xrel[i] != STRIP_OOB && xrow[i] < prows && (unsigned)h < (unsigned)p.Hin;
                xv[i] = ok ? xrel[i] + (unsigned)(h0 * p.Win * 32) : STRIP_OOB;
            }
        }
        unsigned char *xs = xbase + (ld_sg % ROWS_NBUF) * stage_bytes;
        const unsigned soff_x = (unsigned)(ld_c * HWin * 32);
#pragma unroll
        for (int i = 0; i < ROWS_MAXXB; ++i) {
            const int b = wave + NW * i;
            if (b < p.nblocks) {                                         // wave-uniform; same count for every stage
                load_lds16(rs_in, xs + b * 1024, xv[i], soff_x);
                load_lds16(rs_in, xs + p.xpitch + b * 1024, xv[i] == STRIP_OOB ? STRIP_OOB : xv[i] + 16, soff_x);
            }
        }
        ++ld_sg;
        if (++ld_c == CB) { ld_c = 0; ++ld_js; }
    };
    auto stage_loads = [&](int sg) {
        return lx + (sg < CB ? lw : 0) + ((sg == 0 && wave == 0) ? 1 : 0);
    };

    // accumulator register v of channel half a holds channel a * 32 + 8 * (v / 4) + 4 * lg + v % 4
    auto init_tile = [&](f32x16 &t, int a) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float4 b4 = *reinterpret_cast<const float4 *>(bias_lds + a * 32 + 8 * j + 4 * lg);
            t[4 * j] = b4.x; t[4 * j + 1] = b4.y; t[4 * j + 2] = b4.z; t[4 * j + 3] = b4.w;
        }
    };

    // Finished tiles wait in registers as packed bf16 and leave during the stages of the next sub-strip, a tile or
    // two per stage: the memory system then sees a steady trickle of stores under the MFMAs instead of every
    // workgroup of the chip storing a whole sub-strip at the same moment.  Slot i: 2 x 16 bytes per lane (the two
    // 16-channel blocks of channel half pend_a[i]) for the pixel at byte offset pend_pix[i] (out of range: no store).
    constexpr int NPEND = 5;
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    u32x4 pend[NPEND][2];
    unsigned pend_pix[NPEND];
    int pend_a[NPEND];
    int npend = 0;
    // ReLU, rounding, lane-pair exchange of one 32x32 tile (channel half a) into slot i
    auto finish_tile = [&](const f32x16 &t, unsigned pixoff, int a, int i) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = p.relu ? fmaxf(t[8 * h + e], 0.f) : t[8 * h + e];
            const uint32_t q0 = pack_bf16x2_hw(v[0], v[1]), q1 = pack_bf16x2_hw(v[2], v[3]);
            const uint32_t q2 = pack_bf16x2_hw(v[4], v[5]), q3 = pack_bf16x2_hw(v[6], v[7]);
            const uint4 o = lane_pair_exchange(q0, q1, q2, q3);
            pend[i][h] = u32x4{o.x, o.y, o.z, o.w};
        }
        pend_pix[i] = pixoff;
        pend_a[i] = a;
    };
    // The two stores of slot i.  Always two store instructions (lanes without an element get the out-of-range
    // offset): the counted waits of the stage loop need the exact number of memory operations in flight.
    auto store_slot = [&](int i) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int cb = ((k0 + pend_a[i] * 32) >> 4) + h;
            const bool st = pend_pix[i] != STRIP_OOB && cb < CBout;
            const uint32_t off = st ? pend_pix[i] + (uint32_t)(cb * HWout * 32) : STRIP_OOB;
            u32x4 ov = pend[i][h];
            if (p.mask) {
                uint4 mk = make_uint4(0, 0, 0, 0);
                if (st) mk = *reinterpret_cast<const uint4 *>(reinterpret_cast<const unsigned char *>(p.mask) + off);
                const uint4 o = relu_keep8(make_uint4(ov[0], ov[1], ov[2], ov[3]), mk);
                ov = u32x4{o.x, o.y, o.z, o.w};
            }
            __builtin_amdgcn_raw_buffer_store_b128(ov, rs_out, (int)off, 0, NGC_ST_AUX);
        }
    };

    // ---- prologue: the first two stages
    issue_next_stage();
    if (nstages > 1) issue_next_stage();

    const int s = wave & 3, second = wave >> 2;
    const bool late = (p.late_mask >> wave) & 1;          // issue the loads of a stage after this stage's MFMAs
    int toff9[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) toff9[t] = p.tap_off[t] * 16;

    // Counted waits.  This wave's memory operations complete in issue order; n1 = operations issued after the loads
    // of the stage that is waited for next, n2 = after those of the stage behind it (whose loads are in flight if
    // have2).  "Stage sg has landed" is then vmcnt <= n1.
    int n1 = (nstages > 1) ? stage_loads(1) : 0, n2 = 0;
    bool have2 = false;
    int sg = 0;

    for (int js = 0; js < nsub; ++js) {
        // Which fragments this wave holds in sub-strip js.  F fragments = 2 F tiles over 4 SIMDs: SIMD s takes the
        // whole fragments s, s + 4, ... below 4 (F / 4); of the F % 4 left over, whole ones go to the first SIMDs
        // while two SIMDs remain for the halves of the last.  The two waves of a SIMD share its whole fragments
        // (at most two each); the half goes to the second wave.
        int r0, rows;
        sub_rows(js, r0, rows);
        const int npix = rows * p.Wout;
        const int F = (npix + 31) >> 5, q4 = F >> 2, rem = F & 3;
        const int nfs = q4 + ((rem == 3 && s < 2) ? 1 : 0);
        int hf = -1, hk = 0;
        if (rem == 1 && s < 2) { hf = 4 * q4; hk = s; }
        if (rem == 2) { hf = 4 * q4 + (s >> 1); hk = s & 1; }
        if (rem == 3 && s >= 2) { hf = 4 * q4 + 2; hk = s - 2; }
        const int nf1 = (nfs + 1) >> 1;                                   // at most 2 (nfs <= 4)
        const int first = second ? nf1 : 0;
        const int nfull = second ? nfs - nf1 : nf1;
        const int half = (second && hf >= 0) ? 1 : 0;
        const int ha = hk;
        // per fragment: LDS byte offset of the lane's position inside the patch at tap offset 0, and the byte offset
        // of its output pixel (16-channel block 0, this lane's 8-channel half) or out of range
        int pb[2], pbh;
        unsigned opix[2], opixh;
        auto frag_setup = [&](int f, int &pbase, unsigned &pixoff) {
            const uint32_t m = (uint32_t)(f * 32 + l32);
            pbase = 0;
            pixoff = STRIP_OOB;
            if (m < (uint32_t)npix) {
                const uint32_t tp = fd_div(m, p.div_q);
                const uint32_t q = m - tp * p.div_q.d;
                pbase = (int)(tp * p.PC + q) * 16;
                pixoff = (uint32_t)(n * CBout * HWout + (p0 + r0 + (int)tp) * p.Wout + (int)q) * 32 + lg * 16;
            }
        };
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int idx = first + i;
            frag_setup(idx < q4 ? s + 4 * idx : 4 * q4 + s, pb[i], opix[i]);
        }
        frag_setup(hf < 0 ? 0 : hf, pbh, opixh);

        // The CB stages of the sub-strip and its stores, one instantiation per shape of the wave's work: the
        // accumulators are local to it.
        auto substrip = [&](auto nfull_tag, auto half_tag) {
            constexpr int NFULL = decltype(nfull_tag)::value;
            constexpr bool HALF = decltype(half_tag)::value;
            f32x16 acc[2][2], acch;
            for (int c = 0; c < CB; ++c, ++sg) {
                wait_vmcnt(n1);                            // this wave's loads of stage sg have landed
                wg_barrier_nofence();                      // ... and everybody's; the buffer of stage sg - 1 is free
                ROWS_TL();
                n1 = have2 ? n2 : 0;
                n2 = 0;
                have2 = false;
                const bool more = sg + 2 < nstages;
                if (more && !late) {
                    n1 += stage_loads(sg + 2);
                    issue_next_stage();
                    have2 = true;
                }
                if (c == 0) {                              // behind the barrier: the bias values have landed
#pragma unroll
                    for (int i = 0; i < NFULL; ++i) {
                        init_tile(acc[i][0], 0);
                        init_tile(acc[i][1], 1);
                    }
                    if (HALF) init_tile(acch, ha);
                }
                const unsigned char *xs = xbase + (sg % ROWS_NBUF) * stage_bytes + lg * p.xpitch;
                const unsigned char *ws = wbase + c * wchunk + lg * STRIP_WPITCH + l32 * 16;
                if constexpr (NFULL > 0 || HALF) {
                    rows_stage_mfma_nt<NFULL, HALF, 9>(acc, acch, xs, ws, pb, pbh, ha, toff9);
                }
                ROWS_TL();
                if (more && late) {
                    n1 += stage_loads(sg + 2);
                    issue_next_stage();
                    have2 = true;
                }
                // the previous sub-strip's tiles: slots c, c + CB, ... leave in this stage
#pragma unroll
                for (int i = 0; i < NPEND; ++i) {
                    if (i < npend && i % CB == c) {
                        store_slot(i);
                        n1 += 2;
                        if (have2) n2 += 2;
                    }
                }
            }
            npend = 0;
#pragma unroll
            for (int i = 0; i < NFULL; ++i) {
                finish_tile(acc[i][0], opix[i], 0, 2 * i);
                finish_tile(acc[i][1], opix[i], 1, 2 * i + 1);
            }
            if (HALF) finish_tile(acch, opixh, ha, 2 * NFULL);
            npend = 2 * NFULL + (HALF ? 1 : 0);
        };
        typedef std::integral_constant<int, 0> I0;
        typedef std::integral_constant<int, 1> I1;
        typedef std::integral_constant<int, 2> I2;
        if (nfull == 2) substrip(I2{}, std::false_type{});
        else if (nfull == 1 && half) substrip(I1{}, std::true_type{});
        else if (nfull == 1) substrip(I1{}, std::false_type{});
        else if (half) substrip(I0{}, std::true_type{});
        else substrip(I0{}, std::false_type{});
        ROWS_TL();
    }
#pragma unroll
    for (int i = 0; i < NPEND; ++i)
        if (i < npend) store_slot(i);
#ifdef NGC_TIMELINE
    __builtin_amdgcn_s_waitcnt(0x0F70);
    ROWS_TL();
    if (lane == 0 && blockIdx.x < 1024 && blockIdx.y == 0)
        for (int i = 0; i < 64; ++i) g_rows_timeline[(blockIdx.x * 8 + wave) * 64 + i] = i < tl_n ? tl_lds[wave * 64 + i] : 0;
#endif
}

}  // namespace

#ifdef NGC_TIMELINE
extern "C" int ngc_debug_rows_timeline(unsigned long long *host_dst, size_t count)
{
    return (int)hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(g_rows_timeline), count * sizeof(unsigned long long));
}
#endif

hipError_t launch_rows(const RowsParams &p, size_t lds_bytes, hipStream_t st)
{
    static LdsLimitOnce lds_limit;
    {
        const hipError_t e = lds_limit.raise(reinterpret_cast<const void *>(&conv_rows_bf16));
        if (e != hipSuccess) return e;
    }
    const dim3 grid(p.N * p.strips, (p.Cout + 63) / 64);
    lds_bytes += 256;                                     // bias values of the tile
#ifdef NGC_TIMELINE
    lds_bytes += 4096;
#endif
    NGC_LAUNCH(conv_rows_bf16, grid, dim3(ROWS_NW * 64), lds_bytes, st, p);
    return launch_result();
}

}  // namespace ngc
