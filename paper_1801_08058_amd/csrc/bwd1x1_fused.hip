// ConvolutionBackpropData and ConvolutionBackpropFilters of a 1x1 stride-1 node in one pass over dy
// (bf16 MFMA, gfx950).  Both derivative ops of a node read dy (paper Sec. 3: the derivative graph
// holds one op per input of the forward op, each fed by the same adjoint); for an expanding 1x1
// layer dy is the largest tensor of the node and the two ops are bound by reading it, so one kernel
// that brings a tile of dy into LDS once and runs both contractions on it moves 0.6 of the bytes.
//
//   dx[m][c]  = sum_k dy[m][k] * w[k][c]                 (m = (n, h, w); reduction over channels)
//   dw[k][c]  = sum_m dy[m][k] * x[m][c]                 (reduction over positions)
//
// Workgroup = 8 waves, a chunk of positions x one tile of 64 input channels x all K = 64 KT output
// channels.  A stage = 64 positions: dy [64][K] and x [64][64] go to LDS in their natural
// channel-contiguous form (direct global->LDS loads, ring of three stages, counted waits, bare
// barriers).  dx: wave (c32, pos16) owns a 32 c x 16 position tile of the stage; its filter operands
// (all K for its 32 channels, 16 KT registers) stay in registers for the whole kernel, the dy
// operand is a plain 16-byte LDS read (8 consecutive k of one position); the result is rounded once
// and stored 4 channels (8 bytes) per lane.  dw: wave w owns KT/2 (or 1) 16-channel blocks of k x
// 4 (or 2) blocks of c as 16x16 tiles that live in registers for the whole kernel; operands come
// through the LDS transpose load (8 positions per lane).  Partial sums of dw go to the workspace as
// [part][K][C] fp32; bwd1x1_fused_reduce adds the parts in index order (deterministic).
// p.relu_mask: dx is masked with x > 0 (the backprop of the ReLU that produced the node's data input, compounded
// into the store: x is in LDS anyway).
#include "common.h"

namespace ngc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4_f;

constexpr unsigned BF_OOB = 0x80000000u;
constexpr int BF_SP = 64;                         // positions per stage
constexpr int BF_PLANE = BF_SP * 32 + 128;        // bytes per 16-channel plane of a stage

__device__ __forceinline__ bf16x8 tr_frag_f(const unsigned char *lo)
{
    // two 4x16 transposed blocks (positions +0..3 and +16..19) -> this lane's 8 reduction elements
    const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_f *)lo);
    const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_f *)(lo + 512));
    const s16x8 r = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

// NBUF = stage buffers of the ring (3; 2 for K = 512, whose stages are 78 KB)
template <int KT, int NBUF>
__global__ __launch_bounds__(512) void bwd1x1_fused_bf16(const Bwd1x1FusedParams p)
{
    preload_kernargs(p);
    constexpr int NW = 8;
    constexpr int BF_NBUF = NBUF;
    constexpr int KB = 4 * KT;                    // 16-channel planes of dy
    constexpr int NPL = KB + 4;                   // planes per stage: dy, then the 4 planes of the x tile
    constexpr int STAGE = NPL * BF_PLANE;
    constexpr int KSTEPS = 2 * KT;                // 32-channel reduction steps of the dx contraction
    constexpr int KBW = KT >= 2 ? KT / 2 : 1;     // dw tiles of a wave: KBW blocks of k x CBW blocks of c
    constexpr int CBW = KT >= 2 ? 4 : 2;
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int L = lane & 15;
    const int grp = lane >> 4;
    const int part = blockIdx.x, ct = blockIdx.y;
    const int CBt = p.C >> 4;                     // 16-channel planes of x / dx
    const int HW = p.HW;

    const ngc_u32x4 rs_dy = make_rsrc_words(p.dy, p.dy_bytes);
    const ngc_u32x4 rs_x = make_rsrc_words(p.x, p.x_bytes);
    __amdgpu_buffer_rsrc_t rs_dx = __builtin_amdgcn_make_buffer_rsrc((void *)p.dx, 0, (int)p.x_bytes, 0x00020000);

    // stages [s_begin, s_end) of 64 positions each
    const int s_begin = part * p.stages_per_part;
    const int s_end = (s_begin + p.stages_per_part < p.nstages) ? s_begin + p.stages_per_part : p.nstages;
    const int nst = s_end > s_begin ? s_end - s_begin : 0;

    // ---- dx: two 16 c x 16 position tiles of a stage per wave.  K <= 256: wave (c32, pos16) holds channel blocks
    // 2 c32, 2 c32 + 1 of the tile for position block pos16 (two filter operand sets, one dy operand per step);
    // K = 512 (WIDE): wave (c16, pos32) holds channel block c16 for position blocks 2 pos32, 2 pos32 + 1 (one
    // filter operand set of 64 registers instead of two, two dy operands per step).
    constexpr bool WIDE = KT == 8;
    constexpr int NWA = WIDE ? 1 : 2;
    const int cblk0 = WIDE ? (wave & 3) : 2 * (wave & 1);               // first 16-channel block (inside the tile)
    const int pblk0 = WIDE ? 2 * (wave >> 2) : (wave >> 1);             // first 16-position block
    // filter operands: rows = channels c (lane L of 16), 8 consecutive k per lane group (w is [k/16][c][k%16])
    bf16x8 wa[NWA][KSTEPS];
#pragma unroll
    for (int a = 0; a < NWA; ++a)
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const int kb = 2 * ks + (grp >> 1);
            const int c = ct * 64 + (cblk0 + a) * 16 + L;
            wa[a][ks] = *reinterpret_cast<const bf16x8 *>(p.w + ((size_t)kb * p.C + c) * 16 + (grp & 1) * 8);
        }

    // ---- dw tiles of this wave
    const int kb_w0 = KT >= 2 ? wave * KBW : (wave & 3);
    const int cb_w0 = KT >= 2 ? 0 : (wave >> 2) * 2;
    f32x4 acc[KBW][CBW];
#pragma unroll
    for (int i = 0; i < KBW; ++i)
#pragma unroll
        for (int j = 0; j < CBW; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;

    // ---- loads: plane item j = wave + 8 i (i < KT: dy plane j >> 1, else x plane wave >> 1), always block wave & 1
    const int my_blk = wave & 1;
    const int my_pos = my_blk * 32 + (lane >> 1);                        // position inside the stage this lane loads
    auto issue_loads = [&](int s, int buf) {
        unsigned char *base = smem + buf * STAGE;
        const uint32_t m = (uint32_t)((s_begin + s) * BF_SP + my_pos);
        const bool in = m < p.M;
        const uint32_t n = fd_div(in ? m : 0, p.div_hw);
        const uint32_t pq = (in ? m : 0) - n * p.div_hw.d;
        const unsigned half = (unsigned)(lane & 1) * 16;
        const unsigned dy_off = in ? (unsigned)((n * KB * HW + pq) * 32) + half : BF_OOB;
        const unsigned x_off = in ? (unsigned)((n * CBt * HW + pq) * 32) + half : BF_OOB;
#pragma unroll
        for (int i = 0; i < KT; ++i) {
            const int pl = (wave + NW * i) >> 1;
            dma_load_lds16(rs_dy, base + pl * BF_PLANE + my_blk * 1024, dy_off, (unsigned)(pl * HW * 32));
        }
        const int plx = wave >> 1;
        dma_load_lds16(rs_x, base + (KB + plx) * BF_PLANE + my_blk * 1024, x_off, (unsigned)((ct * 4 + plx) * HW * 32));
    };
    constexpr int LPW = KT + 1;                                          // loads per wave and stage

    // byte offset of this lane inside a plane for the transposed reads of a 32-position step
    const int lane_off = (grp * 4 + (L >> 2)) * 32 + (L & 3) * 8;
    // ... and for the dy operand of the dx contraction: position 16 pblk0 + L, 8 channels (grp & 1) of block (grp >> 1)
    const int dxb_off = (grp >> 1) * BF_PLANE + (pblk0 * 16 + L) * 32 + (grp & 1) * 16;

    for (int s = 0; s < BF_NBUF - 1 && s < nst; ++s) issue_loads(s, s);
    int buf = 0;
    for (int s = 0; s < nst; ++s) {
        // This wave's vector-memory operations complete in the order they were issued, loads and stores alike.  After
        // the loads of stage s it has issued the loads of the `later` stages that follow (NBUF - 2 of them, fewer at
        // the end) and the 2 stores of each of the stages s - NBUF + 1 .. s - 1 that exist.
        const int later = (nst - 1 - s < BF_NBUF - 2) ? nst - 1 - s : BF_NBUF - 2;
        wait_vmcnt(later * LPW + 2 * (s < BF_NBUF - 1 ? s : BF_NBUF - 1));
        wg_barrier_nofence();                                            // stage s complete; buffer of stage s - 1 is free
        {
            const int nb = buf + BF_NBUF - 1 >= BF_NBUF ? buf - 1 : buf + BF_NBUF - 1;
            if (s + BF_NBUF - 1 < nst) issue_loads(s + BF_NBUF - 1, nb);
        }
        const unsigned char *dys = smem + buf * STAGE;
        const unsigned char *xs = dys + KB * BF_PLANE;
        buf = (buf + 1 == BF_NBUF) ? 0 : buf + 1;

        // dx tiles of the stage
        f32x4 d0 = {0.f, 0.f, 0.f, 0.f}, d1 = d0;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const bf16x8 b = *reinterpret_cast<const bf16x8 *>(dys + 2 * ks * BF_PLANE + dxb_off);
            d0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[0][ks], b, d0, 0, 0, 0);
            if constexpr (WIDE) {
                const bf16x8 b1 = *reinterpret_cast<const bf16x8 *>(dys + 2 * ks * BF_PLANE + dxb_off + 16 * 32);
                d1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[0][ks], b1, d1, 0, 0, 0);
            } else {
                d1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[NWA - 1][ks], b, d1, 0, 0, 0);
            }
        }
        // dw: two 32-position steps
#pragma unroll
        for (int j = 0; j < BF_SP / 32; ++j) {
            bf16x8 a[KBW], b[CBW];
#pragma unroll
            for (int i = 0; i < KBW; ++i) a[i] = tr_frag_f(dys + (kb_w0 + i) * BF_PLANE + j * 1024 + lane_off);
#pragma unroll
            for (int i = 0; i < CBW; ++i) b[i] = tr_frag_f(xs + (cb_w0 + i) * BF_PLANE + j * 1024 + lane_off);
#pragma unroll
            for (int i = 0; i < KBW; ++i)
#pragma unroll
                for (int k = 0; k < CBW; ++k) acc[i][k] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[k], acc[i][k], 0, 0, 0);
        }
        // store dx: this lane holds channels 4 grp .. +3 of a 16-channel block for position 16 (position block) + L;
        // d1 is the next channel block at the same position, or (WIDE) the same block 16 positions on
        {
            typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
            u32x2 v0 = {pack_bf16x2_hw(d0[0], d0[1]), pack_bf16x2_hw(d0[2], d0[3])};
            u32x2 v1 = {pack_bf16x2_hw(d1[0], d1[1]), pack_bf16x2_hw(d1[2], d1[3])};
            if (p.relu_mask) {
                // ReLU backprop of the node's data input: x sits in the stage buffer, the same 4 channels of the same
                // position are 8 bytes of its plane
                const unsigned char *xm = xs + cblk0 * BF_PLANE + (pblk0 * 16 + L) * 32 + grp * 8;
                const u32x2 m0 = *reinterpret_cast<const u32x2 *>(xm);
                const u32x2 m1 = *reinterpret_cast<const u32x2 *>(xm + (WIDE ? 16 * 32 : BF_PLANE));
                v0[0] = relu_keep2(v0[0], m0[0]); v0[1] = relu_keep2(v0[1], m0[1]);
                v1[0] = relu_keep2(v1[0], m1[0]); v1[1] = relu_keep2(v1[1], m1[1]);
            }
            const uint32_t m = (uint32_t)((s_begin + s) * BF_SP + pblk0 * 16 + L);
            const bool in = m < p.M;
            const uint32_t n = fd_div(in ? m : 0, p.div_hw);
            const uint32_t pq = (in ? m : 0) - n * p.div_hw.d;
            const unsigned o0 = in ? (unsigned)(((n * CBt + ct * 4 + cblk0) * HW + pq) * 32 + grp * 8) : BF_OOB;
            unsigned o1 = in ? o0 + (unsigned)(HW * 32) : BF_OOB;
            if constexpr (WIDE) {
                const uint32_t m1 = m + 16;
                const bool in1 = m1 < p.M;
                const uint32_t n1 = fd_div(in1 ? m1 : 0, p.div_hw);
                const uint32_t pq1 = (in1 ? m1 : 0) - n1 * p.div_hw.d;
                o1 = in1 ? (unsigned)(((n1 * CBt + ct * 4 + cblk0) * HW + pq1) * 32 + grp * 8) : BF_OOB;
            }
            __builtin_amdgcn_raw_buffer_store_b64(v0, rs_dx, (int)o0, 0, NGC_ST_AUX);
            __builtin_amdgcn_raw_buffer_store_b64(v1, rs_dx, (int)o1, 0, NGC_ST_AUX);
        }
    }

    // ---- partial sums of dw: [part][K][C] fp32; register v of tile (i, j): k = 16 (kb_w0 + i) + 4 grp + v, c = 16 (cb_w0 + j) + L
    float *out = p.partial + (size_t)part * p.K * p.C + ct * 64;
#pragma unroll
    for (int i = 0; i < KBW; ++i)
#pragma unroll
        for (int j = 0; j < CBW; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                out[(size_t)(16 * (kb_w0 + i) + 4 * grp + v) * p.C + 16 * (cb_w0 + j) + L] = acc[i][j][v];
}

// dw[i] = sum over parts of partial[part][i], i over K*C (float4 units), in a fixed order.  256 threads = 16 outputs
// x 16 part slices (slice s adds parts s, s + 16, ... in two interleaved chains); the slices are summed through LDS
// in a fixed tree.
__global__ __launch_bounds__(256) void bwd1x1_fused_reduce(const f32x4 *__restrict__ partial, f32x4 *__restrict__ dw, int nparts, int n4)
{
    __shared__ f32x4 sm[16][16];
    const int o = threadIdx.x & 15, sl = threadIdx.x >> 4;
    const int i = blockIdx.x * 16 + o;
    f32x4 t0 = {0.f, 0.f, 0.f, 0.f}, t1 = t0;
    if (i < n4) {
        int sp = sl;
        for (; sp + 16 < nparts; sp += 32) {
            t0 += partial[(size_t)sp * n4 + i];
            t1 += partial[(size_t)(sp + 16) * n4 + i];
        }
        if (sp < nparts) t0 += partial[(size_t)sp * n4 + i];
    }
    sm[sl][o] = t0 + t1;
    __syncthreads();
    if (sl == 0 && i < n4) {
        f32x4 r[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) r[j] = sm[2 * j][o] + sm[2 * j + 1][o];
        dw[i] = ((r[0] + r[1]) + (r[2] + r[3])) + ((r[4] + r[5]) + (r[6] + r[7]));
    }
}

template <int KT>
static hipError_t launch_kt(const Bwd1x1FusedParams &p, hipStream_t st)
{
    constexpr int NBUF = KT == 8 ? 2 : 3;
    constexpr size_t lds = (size_t)NBUF * (4 * KT + 4) * BF_PLANE;
    static LdsLimitOnce lds_limit;
    {
        const hipError_t e = lds_limit.raise(reinterpret_cast<const void *>(&bwd1x1_fused_bf16<KT, NBUF>));
        if (e != hipSuccess) return e;
    }
    NGC_LAUNCH((bwd1x1_fused_bf16<KT, NBUF>), dim3(p.nparts, p.C / 64), dim3(512), lds, st, p);
    hipError_t e = ngc::launch_result();
    if (e != hipSuccess) return e;
    const int n4 = p.K * p.C / 4;
    NGC_LAUNCH(bwd1x1_fused_reduce, dim3((n4 + 15) / 16), dim3(256), 0, st, reinterpret_cast<const f32x4 *>(p.partial),
               reinterpret_cast<f32x4 *>(p.dw), p.nparts, n4);
    return ngc::launch_result();
}

hipError_t launch_bwd1x1_fused(const Bwd1x1FusedParams &p, hipStream_t st)
{
    switch (p.K / 64) {
    case 1: return launch_kt<1>(p, st);
    case 2: return launch_kt<2>(p, st);
    case 4: return launch_kt<4>(p, st);
    case 8: return launch_kt<8>(p, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace ngc
