// 1x1 convolution (forward and backprop-data) as a pipelined GEMM on bf16 MFMA (gfx950).
//
//   out[pos][co] = sum_ci in[pos'][ci] * wt[ci/16][co][ci%16]        (one tap, any stride)
//
// Workgroup = 8 MFMA waves + 2 loader waves, tile BM = 64*WM positions x BN = 64*WN output
// channels (WM*WN = 8), MFMA wave tile 64 x 64 = 2x2 v_mfma_f32_32x32x16_bf16 (A = filters, B =
// activations, as in the other forward kernels).  The reduction runs over 16*KB-input-channel stages
// through an NS-deep LDS ring filled by direct global->LDS loads (buffer_load_dwordx4 ... lds)
// that only the loader waves issue: a loader issues the same number of loads per stage, so
// "stage s has landed" is a counted s_waitcnt vmcnt(N) and the loads of the next NS-1 stages stay
// in flight during the MFMAs of stage s.  One barrier per stage, shared by all 10 waves.
// LDS planes of 16-byte units (8 channels of one row) as in the strip kernel: conflict-free
// ds_read_b128 operand fetches.
//
// Workgroups that share an activation tile (different output-channel tiles) are given ids that
// land on the same XCD (id % 8), so the tile is fetched into one L2 only.
//
// Layout propagation (stride 1, no padding, H*W % 8 == 0): with XN the activations are read from an
// NCHW tensor, with YN the result is written to one, so a layer at the edge of the blocked part of a
// graph needs no conversion pass.  XN: a load instruction brings 4 channels x 128 positions to LDS
// as [16 positions][4 channels][16 positions] blocks and the MFMA operand (8 channels of one position
// per lane) comes from two ds_read_b64_tr_b16 of a 4 x 16 block each (conflict-free: a block is 128
// contiguous bytes).  YN: the wave tile goes through LDS ([channel][64 positions], rows padded to
// 144 bytes) and leaves as 16-byte pieces of 8 consecutive positions.
#include "common.h"

#include <stdlib.h>

namespace ngc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4_q __attribute__((ext_vector_type(4)));
typedef short s16x8_q __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void lds_void_q;
typedef __attribute__((address_space(3))) s16x4_q lds_s16x4_q;

// rows lo: channels c..c+3, rows hi: channels c+4..c+7 of 16 positions -> this lane's 8 channels of its position
__device__ __forceinline__ bf16x8 tr_frag_q(const unsigned char *lo, const unsigned char *hi)
{
    const s16x4_q a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_q *)lo);
    const s16x4_q b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_q *)hi);
    const s16x8_q r = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

constexpr unsigned G1_OOB = 0x80000000u;

// NS = ring depth; KB = 16-channel blocks per stage (4 or 2): a stage holds 2 KB planes (8-channel halves) per operand.
// NL = loader waves (1 or 2); WM x WN MFMA waves; FA = 32-channel output fragments per MFMA wave
// (2: 64 x 64 wave tiles; 4: 64 positions x 128 channels, 6 instead of 8 LDS operand fetches per 8 MFMAs).
// XN / YN: activations read from / result written to an NCHW tensor (else 16-channel blocked).
// DB (blocked result only): every MFMA wave also writes the per-channel sums over its positions of the values
// it stored (fp32, fixed order) to row (p.dbp_row0 + m-tile) * WM + wm of p.dbp: partials of a bias gradient
// of the result.
template <int WM, int WN, int NS, int KB, int NL, int FA, bool XN, bool YN, bool DB = false>
__global__ __launch_bounds__(64 * (WM * WN + NL)) void conv_gemm1x1_bf16(const Gemm1x1Params p)
{
    preload_kernargs(p);
    constexpr int BM = 64 * WM, BN = 32 * FA * WN;
    constexpr int WB = BN / 64;                       // 64-row blocks of a filter plane
    constexpr int XPLANE = BM * 16 + 128, WPLANE = BN * 16 + 128;
    constexpr int NPL = 2 * KB;                       // planes per operand and stage
    constexpr int STAGE = NPL * XPLANE + NPL * WPLANE;
    constexpr int NCW = WM * WN;                      // MFMA waves
    constexpr int PPL = NPL / NL;                     // planes per loader wave
    constexpr int LPL = PPL * (WM + WB);              // loads per loader wave per stage (same count with XN)
    constexpr int NH128 = BM / 128;                   // XN: 128-position pieces of the tile
    constexpr int QPL = 4 * KB / NL;                  // XN: 4-channel groups per loader wave and stage
    constexpr int YROW = 144;                         // YN: bytes per channel row of a wave's staging tile
    static_assert(QPL * NH128 == PPL * WM, "XN load count");
    static_assert((NCW == 8 || NCW == 4) && (NL == 1 || NL == 2), "wave roles");
    static_assert(NS >= 2 && NS <= 4 && (KB == 2 || KB == 4), "ring depth / stage size");
    static_assert(LPL * (NS - 2) < 64, "vmcnt range");
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // XCD-aware tile order: id = xcd + 8 * (mgroup * NT + ntile), m-tile = mgroup * 8 + xcd
    const int NT = (p.Cout + BN - 1) / BN;             // the last tile may be partial (Cout % 16 == 0)
    const int xcd = blockIdx.x & 7;
    const int slot = blockIdx.x >> 3;
    const int ntile = slot % NT;
    const int mtile = (slot / NT) * 8 + xcd;
    const uint32_t m0 = (uint32_t)mtile * BM;
    if (m0 >= p.M) return;                             // uniform per workgroup
    const int n0 = ntile * BN;
    const int nsteps = (p.Cin + 16 * KB - 1) / (16 * KB);   // channel blocks past Cin (% 16 == 0) are loaded as zeros

    if (wave >= NCW) {
        // ---- loader waves (the last NL): all global->LDS traffic of the workgroup.  A wave whose loads are
        // held back by the memory system stalls at issue; keeping the loads out of the MFMA waves
        // lets the matrix pipes run meanwhile.  Loader l fills planes PPL*l .. PPL*l+PPL-1 (plane = 16-channel
        // block * 2 + 8-channel half) of both operands, KB planes each: LPL loads per stage.
        const int lw = wave - NCW;
        const int CBin = p.Cin >> 4;
        const int HWin = p.Hin * p.Win;
        __amdgpu_buffer_rsrc_t rs_in = __builtin_amdgcn_make_buffer_rsrc((void *)p.in, 0, (int)p.in_bytes, 0x00020000);
        __amdgpu_buffer_rsrc_t rs_wt = __builtin_amdgcn_make_buffer_rsrc((void *)p.wt, 0, (int)p.wt_bytes, 0x00020000);
        unsigned xvoff[WM];
        if constexpr (XN) {
            // lane = 16-byte unit: channel (lane / 2) % 4 of the group, positions (lane / 8) * 16 + (lane % 2) * 8 + 0..7
            const int chq = (lane >> 1) & 3;
            const int poff = (lane >> 3) * 16 + (lane & 1) * 8;
#pragma unroll
            for (int h = 0; h < NH128; ++h) {
                const uint32_t m = m0 + (uint32_t)(h * 128 + poff);
                xvoff[h] = G1_OOB;
                if (m < p.M) {
                    const uint32_t n = fd_div(m, p.div_pq);
                    const uint32_t pp = m - n * p.div_pq.d;
                    xvoff[h] = (unsigned)((((size_t)n * p.Cin + chq) * HWin + pp) * 2);
                }
            }
        }
#pragma unroll
        for (int b = 0; b < WM; ++b) {
            if constexpr (XN) break;
            const uint32_t m = m0 + (uint32_t)(b * 64 + lane);
            xvoff[b] = G1_OOB;
            if (m < p.M) {
                const uint32_t n = fd_div(m, p.div_pq);
                const uint32_t rem = m - n * p.div_pq.d;
                const uint32_t i = fd_div(rem, p.div_q);
                const uint32_t j = rem - i * p.div_q.d;
                const int ih = (int)i * p.is_h + p.dh;
                const int iw = (int)j * p.is_w + p.dw;
                if ((unsigned)ih < (unsigned)p.Hin && (unsigned)iw < (unsigned)p.Win)
                    xvoff[b] = (unsigned)(((int)n * CBin * HWin + ih * p.Win + iw) * 32);
            }
        }
        const unsigned wvoff = (unsigned)((n0 + lane) * 32);

        auto issue_loads = [&](int s, int buf) {
            unsigned char *xs = smem + buf * STAGE;
            unsigned char *ws = xs + NPL * XPLANE;
            if constexpr (XN) {
#pragma unroll
                for (int q = 0; q < QPL; ++q) {
                    const int quad = lw * QPL + q;                     // 4-channel group of the stage
                    const bool live = s * 16 * KB + 4 * quad < p.Cin;
                    const unsigned soff_x = live ? (unsigned)((s * 16 * KB + 4 * quad) * HWin * 2) : 0u;
#pragma unroll
                    for (int h = 0; h < NH128; ++h)
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_in, (lds_void_q *)(xs + quad * (BM * 8) + h * 1024), 16,
                                                                 (int)(live ? xvoff[h] : G1_OOB), (int)soff_x, 0, 0);
                }
            }
#pragma unroll
            for (int q = 0; q < PPL; ++q) {
                const int pl = lw * PPL + q;
                const int cb = s * KB + (pl >> 1);
                const bool live = cb < CBin;                          // wave-uniform
                const unsigned soff_x = live ? (unsigned)(cb * HWin * 32) : 0u;
                // Filter rows past Cout and channel blocks past Cin must read as zeros.  Only the per-lane offset
                // takes part in the range check of a buffer load (the scalar offset is added to the base unchecked), so
                // those lanes get the out-of-range constant rather than an address behind the caller's filter tensor.
                const unsigned soff_w = live ? (unsigned)(cb * p.Cout * 32 + (pl & 1) * 16) : 0u;
#pragma unroll
                for (int b = 0; b < WM; ++b) {
                    if constexpr (XN) break;
                    const unsigned v = (xvoff[b] == G1_OOB || !live) ? G1_OOB : xvoff[b] + (pl & 1) * 16;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_in, (lds_void_q *)(xs + pl * XPLANE + b * 1024), 16, (int)v,
                                                             (int)soff_x, 0, 0);
                }
#pragma unroll
                for (int b = 0; b < WB; ++b)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_wt, (lds_void_q *)(ws + pl * WPLANE + b * 1024), 16,
                                                             (int)((live && n0 + lane + b * 64 < p.Cout) ? wvoff + b * 64 * 32 : G1_OOB),
                                                             (int)soff_w, 0, 0);
            }
        };
#pragma unroll
        for (int s = 0; s < NS - 1; ++s)
            if (s < nsteps) issue_loads(s, s);
        for (int s = 0; s < nsteps; ++s) {
            // stage s has landed when at most the loads of the NS-2 later stages are outstanding
            constexpr int W2 = LPL * 2, W1 = LPL;
            if (NS == 4 && s + 2 < nsteps) __builtin_amdgcn_s_waitcnt(0x0F70 | (W2 & 15) | ((W2 >> 4) << 14));
            else if (NS >= 3 && s + 1 < nsteps) __builtin_amdgcn_s_waitcnt(0x0F70 | (W1 & 15) | ((W1 >> 4) << 14));
            else __builtin_amdgcn_s_waitcnt(0x0F70);
            wg_barrier_nofence();                      // stage s visible to all; buffer of stage s-1 is free
            if (s + NS - 1 < nsteps) issue_loads(s + NS - 1, (s + NS - 1) % NS);
        }
        if constexpr (YN) wg_barrier_nofence();        // the ring becomes the staging area of the stores
        return;
    }

    // ---- MFMA waves 0 .. NCW-1
    const int wm = wave % WM;
    const int wn = wave / WM;
    const int l32 = lane & 31;
    const int lg = lane >> 5;

    // The accumulators start from the bias (register v of fragment a holds channel n0 + 32 FA wn + 32 a + 8 (v / 4) +
    // 4 lg + v % 4): the loads are under the ring's start-up and the epilogue has no additions.
    f32x16 acc[FA][2];
#pragma unroll
    for (int a = 0; a < FA; ++a)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int ch = n0 + wn * 32 * FA + a * 32 + 8 * j + 4 * lg;
            float4 b4 = make_float4(0.f, 0.f, 0.f, 0.f);
            if (p.bias && ch < p.Cout) b4 = *reinterpret_cast<const float4 *>(p.bias + ch);      // Cout % 16 == 0
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                acc[a][b][4 * j] = b4.x; acc[a][b][4 * j + 1] = b4.y; acc[a][b][4 * j + 2] = b4.z; acc[a][b][4 * j + 3] = b4.w;
            }
        }

    for (int s = 0; s < nsteps; ++s) {
        wg_barrier_nofence();
        const unsigned char *xs = XN
            ? smem + (s % NS) * STAGE + (wm * 4 + ((lane >> 4) & 1)) * 128 + ((lane & 15) >> 2) * 32 + (lane & 3) * 8
            : smem + (s % NS) * STAGE + lg * XPLANE + (wm * 64 + l32) * 16;
        const unsigned char *ws = smem + (s % NS) * STAGE + NPL * XPLANE + lg * WPLANE + (wn * 32 * FA + l32) * 16;
#pragma unroll
        for (int ks = 0; ks < KB; ++ks) {
            bf16x8 fa[FA], fb[2];
#pragma unroll
            for (int a = 0; a < FA; ++a) fa[a] = *reinterpret_cast<const bf16x8 *>(ws + (2 * ks) * WPLANE + a * 512);
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                if constexpr (XN) {
                    const unsigned char *q0 = xs + (ks * 4 + 2 * lg) * (BM * 8) + b * 256;
                    fb[b] = tr_frag_q(q0, q0 + BM * 8);
                } else {
                    fb[b] = *reinterpret_cast<const bf16x8 *>(xs + (2 * ks) * XPLANE + b * 512);
                }
            }
#pragma unroll
            for (int a = 0; a < FA; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
        }
    }

    const int HWout = p.Hout * p.Wout;
    if constexpr (YN) {
        // ---- NCHW epilogue: ReLU (bias is in the accumulators), one RNE rounding, wave tile -> LDS [channel][64 positions] -> 16-byte stores
        wg_barrier_nofence();                          // every wave is done with the ring
        unsigned char *st = smem + wave * (32 * FA * YROW);
#pragma unroll
        for (int a = 0; a < FA; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int ch = a * 32 + 8 * (v >> 2) + 4 * lg + (v & 3);
                    float val = acc[a][b][v];                          // bias included
                    if (p.relu) val = fmaxf(val, 0.f);
                    *reinterpret_cast<uint16_t *>(st + ch * YROW + (b * 32 + l32) * 2) =
                        (uint16_t)(pack_bf16x2_hw(val, 0.f) & 0xFFFFu);
                }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // own writes only: no other wave touches this region
        const int piece = lane & 7;
        const uint32_t m = m0 + (uint32_t)(wm * 64 + piece * 8);
        if (m < p.M) {                                 // M % 8 == 0: a piece is valid as a whole
            const uint32_t n = fd_div(m, p.div_pq);
            const uint32_t pp = m - n * p.div_pq.d;
#pragma unroll
            for (int it = 0; it < 4 * FA; ++it) {
                const int ch = it * 8 + (lane >> 3);
                if (n0 + wn * 32 * FA + ch >= p.Cout) continue;
                uint4 o = *reinterpret_cast<const uint4 *>(st + ch * YROW + piece * 16);
                const size_t off = ((size_t)n * p.Cout + (n0 + wn * 32 * FA + ch)) * HWout + pp;
                if (p.mask) o = relu_keep8(o, *reinterpret_cast<const uint4 *>(p.mask + off));
                store16_result(p.out + off, o, true);
            }
        }
        return;
    }
    // ---- epilogue: ReLU (bias is in the accumulators), one RNE rounding, lane-pair exchange, 16-byte stores
    const int CBout = p.Cout >> 4;
    const bool dense_out = p.os_h == 1 && p.os_w == 1;     // every pixel written: whole cache lines
    const bool fast = !DB && p.out_bytes != 0 && p.mask == nullptr && !p.zero_sib;
    const bool relu_b = p.relu != 0;
    const __amdgpu_buffer_rsrc_t rs_out = __builtin_amdgcn_make_buffer_rsrc((void *)p.out, 0, (int)p.out_bytes, 0x00020000);
    float csum[DB ? FA : 1][2][8];                        // DB: channel sums of this lane's stored values
#pragma unroll
    for (int a = 0; a < (DB ? FA : 1); ++a)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int e = 0; e < 8; ++e) csum[a][h][e] = 0.f;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const uint32_t m = m0 + (uint32_t)(wm * 64 + b * 32 + l32);
        const bool ok = m < p.M;
        const uint32_t mm = ok ? m : 0;
        const uint32_t n = fd_div(mm, p.div_pq);
        const uint32_t rem = mm - n * p.div_pq.d;
        const uint32_t i = fd_div(rem, p.div_q);
        const uint32_t j = rem - i * p.div_q.d;
        const int oh = (int)i * p.os_h + p.oa_h;
        const int ow = (int)j * p.os_w + p.oa_w;
        const size_t pix = (size_t)n * CBout * HWout + (size_t)oh * p.Wout + ow;
        if (fast) {
            // plain blocked stores below 2 GiB: 32-bit offsets into a buffer descriptor, lanes that must not store get an
            // out-of-range offset (no 64-bit address arithmetic, no divergent branch per store)
#pragma unroll
            for (int a = 0; a < FA; ++a)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const f32x16 &t = acc[a][b];
                    const uint32_t q0 = relu_bf16x2(pack_bf16x2_hw(t[8 * h], t[8 * h + 1]), relu_b);
                    const uint32_t q1 = relu_bf16x2(pack_bf16x2_hw(t[8 * h + 2], t[8 * h + 3]), relu_b);
                    const uint32_t q2 = relu_bf16x2(pack_bf16x2_hw(t[8 * h + 4], t[8 * h + 5]), relu_b);
                    const uint32_t q3 = relu_bf16x2(pack_bf16x2_hw(t[8 * h + 6], t[8 * h + 7]), relu_b);
                    const uint4 o = lane_pair_exchange(q0, q1, q2, q3);
                    const int cb = ((n0 + wn * 32 * FA + a * 32) >> 4) + h;
                    const unsigned off = (ok && cb < CBout) ? ((unsigned)pix + (unsigned)(cb * HWout)) * 32u + (unsigned)(lg * 16) : 0x80000000u;
                    const ngc_u32x4 ov = {o.x, o.y, o.z, o.w};
                    if (dense_out) __builtin_amdgcn_raw_buffer_store_b128(ov, rs_out, (int)off, 0, NGC_ST_AUX);
                    else __builtin_amdgcn_raw_buffer_store_b128(ov, rs_out, (int)off, 0, 0);
                }
            continue;
        }
#pragma unroll
        for (int a = 0; a < FA; ++a) {
            const int co_base = n0 + wn * 32 * FA + a * 32;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = acc[a][b][8 * h + e];      // bias included
                const bool relu_on = p.relu != 0;                        // ReLU on the rounded pairs: see relu_bf16x2
                const uint32_t q0 = relu_bf16x2(pack_bf16x2_hw(v[0], v[1]), relu_on), q1 = relu_bf16x2(pack_bf16x2_hw(v[2], v[3]), relu_on);
                const uint32_t q2 = relu_bf16x2(pack_bf16x2_hw(v[4], v[5]), relu_on), q3 = relu_bf16x2(pack_bf16x2_hw(v[6], v[7]), relu_on);
                uint4 o = lane_pair_exchange(q0, q1, q2, q3);
                if (ok && (co_base >> 4) + h < CBout) {
                    const size_t blk = pix + (size_t)((co_base >> 4) + h) * HWout;
                    if (p.mask) o = relu_keep8(o, *reinterpret_cast<const uint4 *>(p.mask + blk * 16 + lg * 8));
                    store16_result(p.out + blk * 16 + lg * 8, o, dense_out);
                    if (p.zero_sib) {
                        // strided backprop-data whose one class of pixels starts at (0, 0): the pixels of the block
                        // that no tap reaches are zero, written here instead of by a fill pass over the whole dx
                        for (int zh = 0; zh < p.os_h; ++zh)
                            for (int zw = 0; zw < p.os_w; ++zw)
                                if ((zh | zw) != 0 && oh + zh < p.Hout && ow + zw < p.Wout)
                                    store16_result(p.out + (blk + (size_t)(zh * p.Wout + zw)) * 16 + lg * 8, make_uint4(0, 0, 0, 0), false);
                    }
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
        // half (no LDS, no barrier: a wave that is done leaves), one row of 64 channel sums per MFMA wave row
        // wm; value index j = a*16 + h*8 + e is channel n0 + wn*64 + a*32 + 16 h + 8 lg + e
        static_assert(!DB || FA == 2, "channel sums: 64-channel wave tiles");
        float flat[32];
#pragma unroll
        for (int j = 0; j < 32; ++j) flat[j] = csum[DB ? (j >> 4) : 0][(j >> 3) & 1][j & 7];
        const float mine = half_wave_transpose_sum32(flat, l32);
        const int j = ((l32 & 15) << 1) | (l32 >> 4);
        const int ch = n0 + wn * 64 + (j >> 4) * 32 + ((j >> 3) & 1) * 16 + 8 * lg + (j & 7);
        if (ch < p.Cout) p.dbp[((size_t)(p.dbp_row0 + mtile) * WM + wm) * p.dbp_ld + ch] = mine;
    }
}

// 16-byte zero fill (pixels of a strided backprop-data that no tap reaches)
__global__ __launch_bounds__(256) void zero_fill16(uint4 *__restrict__ dst, size_t n16)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n16; i += stride) dst[i] = make_uint4(0, 0, 0, 0);
}

hipError_t launch_zero_fill(void *dst, size_t bytes, hipStream_t st)
{
    const size_t n16 = bytes / 16;                     // blocked tensors are multiples of 32 bytes
    unsigned blocks = (unsigned)((n16 + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    NGC_LAUNCH(zero_fill16, dim3(blocks), dim3(256), 0, st, static_cast<uint4 *>(dst), n16);
    return ngc::launch_result();
}

template <int WM, int WN, int NS, int KB, int NL, int FA, bool XN, bool YN, bool DB = false>
static hipError_t launch_gemm1x1_l(const Gemm1x1Params &p, hipStream_t st)
{
    static LdsLimitOnce lds_limit;                  // per template instantiation
    {
        const hipError_t e = lds_limit.raise(reinterpret_cast<const void *>(&conv_gemm1x1_bf16<WM, WN, NS, KB, NL, FA, XN, YN, DB>));
        if (e != hipSuccess) return e;
    }
    constexpr int BM = 64 * WM, BN = 32 * FA * WN;
    constexpr size_t stage = (size_t)2 * KB * ((BM * 16 + 128) + (BN * 16 + 128));
    // short reductions use fewer ring buffers than NS: less LDS, more workgroups per compute unit
    const int nsteps = (p.Cin + 16 * KB - 1) / (16 * KB);
    size_t lds = (size_t)(nsteps < NS ? nsteps : NS) * stage;
    constexpr size_t staging = (size_t)WM * WN * 32 * FA * 144;        // YN: one [channel][64 positions] tile per MFMA wave
    if (YN && lds < staging) lds = staging;
    const unsigned mtiles = (p.M + BM - 1) / BM;
    const unsigned grid = ((mtiles + 7) / 8) * 8 * ((p.Cout + BN - 1) / BN);
    NGC_LAUNCH((conv_gemm1x1_bf16<WM, WN, NS, KB, NL, FA, XN, YN, DB>), dim3(grid), dim3(64 * (WM * WN + NL)), lds, st, p);
    return ngc::launch_result();
}

// the NCHW modes exist for the dispatcher's own tile choices (FA = 2)
template <int WM, int WN, int NS, int KB, int NL, int FA = 2>
static hipError_t launch_gemm1x1_t(const Gemm1x1Params &p, hipStream_t st)
{
    constexpr bool dispatcher_tile = FA == 2 && KB == 2 &&
        ((WM == 4 && WN == 2 && NS == 3 && NL == 2) || (WM == 2 && WN == 2 && NS == 3 && NL == 1) ||
         (WM == 8 && WN == 1 && NS == 2 && NL == 2) || (WM == 4 && WN == 1 && NS == 3 && NL == 1));
    if constexpr (dispatcher_tile) {
        if (p.dbp) {
            if (p.in_nchw || p.out_nchw) return hipErrorInvalidValue;
            return launch_gemm1x1_l<WM, WN, NS, KB, NL, FA, false, false, true>(p, st);
        }
        if (p.in_nchw && p.out_nchw) return launch_gemm1x1_l<WM, WN, NS, KB, NL, FA, true, true>(p, st);
        if (p.in_nchw) return launch_gemm1x1_l<WM, WN, NS, KB, NL, FA, true, false>(p, st);
        if (p.out_nchw) return launch_gemm1x1_l<WM, WN, NS, KB, NL, FA, false, true>(p, st);
    }
    if (p.in_nchw || p.out_nchw || p.dbp) return hipErrorInvalidValue;
    return launch_gemm1x1_l<WM, WN, NS, KB, NL, FA, false, false>(p, st);
}

// 32-channel stages in a ring of 3 (75 KB of LDS): two workgroups per compute unit, so one's
// epilogue and ring start-up overlap the other's MFMAs.  Few-tile launches (fewer 256x128 tiles
// than the 512 workgroup slots of the chip) and strided forward gathers take 128x128 tiles (4 MFMA
// waves + 1 loader, three workgroups per compute unit).  NGC_G1_VARIANT (experiments only) forces
// 64-channel stages (1), a ring of 4 (2), the 128x128 tile with a ring of 3 (3) / 4 (4), or the
// 256x128 tile whatever the size (5), or the 256x256 tile with 64x128 wave tiles (6; needs Cout % 256 == 0).
// 128-channel tiles when they waste no more of a partial last tile than 64-channel tiles would (Cout % 16 == 0)
static bool wide_tiles(const Gemm1x1Params &p)
{
    const int c128 = (p.Cout + 127) / 128, c64 = (p.Cout + 63) / 64;
    return p.Cout > 64 && c128 * 128 <= c64 * 64;
}

// tile choice of the NCHW / channel-sum modes (they exist for the dispatcher's own tiles): 0 = large, 3 = small
static int special_mode_variant(const Gemm1x1Params &p)
{
    const char *ev = env_switch(SW_G1_VARIANT);
    if (ev && atoi(ev) == 3) return 3;
    if (ev && atoi(ev) == 5) return 0;
    if (!wide_tiles(p)) return 3;                      // same rules as the plain launches
    const int c128 = (p.Cout + 127) / 128;
    const unsigned tiles = ((p.M + 255) / 256) * (unsigned)c128;
    return ((tiles < 2 * 256 && c128 >= 3) || p.Cin <= 64) ? 3 : 0;
}

// positions per row of p.dbp (64: one row per MFMA wave row of a tile) of the launch launch_gemm1x1 makes when
// p.dbp is set, and positions per tile: rows written = ceil(M / tile) * (tile / 64)
int gemm1x1_dbp_tile_m(const Gemm1x1Params &p)
{
    const int variant = special_mode_variant(p);
    if (wide_tiles(p)) return variant == 3 ? 128 : 256;
    return variant == 3 ? 256 : 512;
}

hipError_t launch_gemm1x1(const Gemm1x1Params &p, hipStream_t st)
{
    const char *ev = env_switch(SW_G1_VARIANT);
    int variant = ev ? atoi(ev) : 0;
    const int c128 = (p.Cout + 127) / 128;
    const bool wide = wide_tiles(p);
    if (p.in_nchw || p.out_nchw || p.dbp) {
        variant = special_mode_variant(p);
        if (wide) return variant == 3 ? launch_gemm1x1_t<2, 2, 3, 2, 1>(p, st) : launch_gemm1x1_t<4, 2, 3, 2, 2>(p, st);
        return variant == 3 ? launch_gemm1x1_t<4, 1, 3, 2, 1>(p, st) : launch_gemm1x1_t<8, 1, 2, 2, 2>(p, st);
    }
    if (wide) {
        if (variant == 0) {
            const unsigned tiles = ((p.M + 255) / 256) * (unsigned)c128;
            // long reductions over enough 256 x 256 tiles: 64 x 128 wave tiles (fewer LDS operand fetches
            // per MFMA; one workgroup per compute unit, which short reductions do not amortise)
            // measured on the ResNet-50 layers: with few tiles the 128 x 128 tile pays only from three channel tiles
            // on (the same activations feed that many workgroups); a one- or two-stage reduction (Cin <= 64) has
            // too little work per 256 x 128 tile to hide its start-up and stores behind
            if (p.Cout % 256 == 0 && p.Cin >= 512 && tiles / 2 >= 192) variant = 6;
            else if ((tiles < 2 * 256 && c128 >= 3) || p.is_h > 1 || p.is_w > 1 || p.Cin <= 64) variant = 3;
        }
        if (variant == 1) return launch_gemm1x1_t<4, 2, 3, 4, 2>(p, st);
        if (variant == 2) return launch_gemm1x1_t<4, 2, 4, 2, 2>(p, st);
        if (variant == 3) return launch_gemm1x1_t<2, 2, 3, 2, 1>(p, st);
        if (variant == 4) return launch_gemm1x1_t<2, 2, 4, 2, 1>(p, st);
        if (variant == 6 && p.Cout % 256 == 0) return launch_gemm1x1_t<4, 2, 3, 2, 2, 4>(p, st);
        return launch_gemm1x1_t<4, 2, 3, 2, 2>(p, st);
    }
    // 64 output channels: 256 x 64 tiles (4 MFMA waves + 1 loader, ring of 3) beat 512 x 64 on every layer measured
    if (variant == 1) return launch_gemm1x1_t<8, 1, 2, 4, 2>(p, st);
    if (variant == 2) return launch_gemm1x1_t<8, 1, 3, 2, 2>(p, st);
    if (variant == 5) return launch_gemm1x1_t<8, 1, 2, 2, 2>(p, st);
    return launch_gemm1x1_t<4, 1, 3, 2, 1>(p, st);
}

}  // namespace ngc
