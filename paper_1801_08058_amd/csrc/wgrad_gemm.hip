// ConvolutionBackpropFilters as a GEMM over positions, one filter tap per workgroup
// (1x1 layers; strided 3x3 layers run it once per tap) on bf16 MFMA (gfx950).
//
//   dw[k,c,tap] = sum_{m=(n,p,q)} dy[m][k] * X[m @ tap][c]
//
// Workgroup = 8 waves, tile 64*WK (k) x 64*WC (c) of dw for one tap over a chunk of positions.
// Wave (wk, wc, h) owns a 64 x 64 sub-tile as 4x4 MFMA 16x16 tiles (64 accumulator registers)
// and every NH-th 32-position step (NH = 8 / (WK*WC) interleaved step streams = a wave-level
// split of the reduction, summed through LDS in a fixed tree at the end).
// A stage = SP (128 or 64) positions: dy [SP][64 WK] and x [SP][64 WC] go to LDS in their natural
// channel-contiguous form with direct global->LDS loads (out-of-range lanes deliver zeros =
// padding and the tail of the chunk); MFMA operands (8 consecutive positions per lane) are
// fetched with the LDS transpose load ds_read_b64_tr_b16.  Two stages, one barrier per stage.
// Partials go to the workspace in register order; wgrad_gemm_reduce adds the parts in index
// order (deterministic) and writes dw as [K][C][R][S].
// Layout propagation (1x1, stride 1, no padding, H*W % 8 == 0): with XN / DN the x / dy operand is
// read from an NCHW tensor.  Positions are contiguous there, so a load unit is 8 positions of one
// channel, a 32-position block of a plane sits in LDS as [16 positions][16 channels][16 positions]
// and the operand is two plain ds_read_b64 (the same position-to-lane assignment as the transposed
// loads of the other operand; 64 lanes cover 512 contiguous bytes).
#include "common.h"

namespace ngc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void lds_void_g;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4_g;

constexpr unsigned WGG_OOB = 0x80000000u;

__device__ __forceinline__ bf16x8 tr_frag_g(const unsigned char *lo)
{
    // two 4x16 transposed blocks (positions +0..3 and +16..19) -> this lane's 8 reduction elements
    const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_g *)lo);
    const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_g *)(lo + 512));
    const s16x8 r = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

typedef __attribute__((address_space(3))) s16x4 lds_s16x4_n;

__device__ __forceinline__ bf16x8 nchw_frag_g(const unsigned char *lo)
{
    // positions +0..3 and +16..19 of this lane's channel row
    const s16x4 a = *(const lds_s16x4_n *)lo;
    const s16x4 b = *(const lds_s16x4_n *)(lo + 512);
    const s16x8 r = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

// SP = positions per stage (128, or 64: half the LDS, two workgroups per compute unit);
// XN / DN: x / dy is an NCHW tensor (else 16-channel blocked); R3: rank-3 spatial tensors (blocked), positions
// (n, o, p, q) and taps (t, r, s)
// XO: XCD-ordered one-dimensional grid (always with R3)
template <int WK, int WC, int SP, bool XN, bool DN, bool R3 = false, bool XO = R3>
__global__ __launch_bounds__(512) void wgrad_gemm_bf16(const WgradGemmParams p)
{
    preload_kernargs(p);
    static_assert(!(R3 && (XN || DN)), "rank-3 tensors are read blocked");
    static_assert(XO || !R3, "rank-3 launches use the XCD-ordered grid");
    constexpr int NW = 8;
    constexpr int NH = NW / (WK * WC);
    constexpr int NPL = 4 * (WK + WC);            // 16-channel planes per stage: dy first, then x
    constexpr int WGG_SP = SP;
    constexpr int WGG_PLANE = SP * 32 + 128;      // bytes per 16-channel plane of a stage
    constexpr int BLK = SP / 32;                  // 32-position blocks per plane = steps per stage
    constexpr int NITEM = NPL * BLK / NW;         // load items (plane, block) per wave and stage
    constexpr int MS = (BLK + NH - 1) / NH;       // steps of a stage per wave, at most
    static_assert((SP == 128 || SP == 64) && NH >= 2 && MS <= 2, "stage shape");
    constexpr int STAGE = NPL * WGG_PLANE;
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wk = wave % WK;
    const int wc = (wave / WK) % WC;
    const int wh = wave / (WK * WC);
    const int L = lane & 15;
    const int grp = lane >> 4;

    // XO: one-dimensional grid.  Workgroup ids go round-robin to the 8 XCDs (one L2 each): position chunk `part`
    // lives on XCD part % 8 and its (tile, tap) workgroups are consecutive there, so the taps of a chunk share its
    // x and dy through that L2 instead of every XCD streaming every tensor once per tap.
    int part = blockIdx.x, tile_id = blockIdx.y, tap = blockIdx.z, ntap_grid = gridDim.z, ntile_grid = gridDim.y;
    if constexpr (XO) {
        ntap_grid = (R3 ? p.T : 1) * p.R * p.S;
        ntile_grid = p.ktiles * p.ctiles;
        const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3, per = ntap_grid * ntile_grid;
        const int pl = j / per, r = j - pl * per;
        part = pl * 8 + xcd;
        if (part >= p.nparts) return;                    // uniform per workgroup
        tile_id = r / ntap_grid;
        tap = r - tile_id * ntap_grid;
    }
    const int kt = tile_id / p.ctiles;
    const int ct = tile_id - kt * p.ctiles;
    int tap2 = tap, dd_off = 0;
    if constexpr (R3) {
        const int tt = tap / (p.R * p.S);
        tap2 = tap - tt * (p.R * p.S);
        dd_off = tt * p.dil_d - p.pbd;
    }
    const int tr = tap2 / p.S, ts = tap2 - tr * p.S;
    const int dh_off = tr * p.dil_h - p.pbh;
    const int dw_off = ts * p.dil_w - p.pbw;

    const uint32_t m_begin = (uint32_t)part * p.chunk;
    const uint32_t m_end = (m_begin + p.chunk < p.M) ? m_begin + p.chunk : p.M;
    const int nstages = (m_begin < m_end) ? (int)((m_end - m_begin + WGG_SP - 1) / WGG_SP) : 0;

    const int PQ = R3 ? p.O * p.P * p.Q : p.P * p.Q;     // positions / pixels per 16-channel plane of an image
    const int HW = R3 ? p.D * p.H * p.W : p.H * p.W;
    const int KB = p.K >> 4, CB = p.C >> 4;
    const int kb0 = kt * 4 * WK, cb0 = ct * 4 * WC;

    __amdgpu_buffer_rsrc_t rs_dy = __builtin_amdgcn_make_buffer_rsrc((void *)p.dy, 0, (int)p.dy_bytes, 0x00020000);
    __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, (int)p.x_bytes, 0x00020000);

    // load items of a stage: item = plane * BLK + block (32 positions); wave w takes items w, w+8, ...
    // -> always block w % BLK, so one position decode per stage and lane
    const int my_blk = wave % BLK;
    auto issue_loads = [&](int s, int buf) {
        unsigned char *base = smem + buf * STAGE;
        const uint32_t m = m_begin + (uint32_t)(s * WGG_SP + my_blk * 32 + (lane >> 1));
        const bool in = m < m_end;
        const uint32_t mm = in ? m : 0;
        uint32_t n, rem, rem2;
        int slice = 0;                                                   // first pixel of the depth slice read
        bool zin = true;
        if constexpr (R3) {
            n = fd_div(mm, p.div_opq);
            rem = mm - n * p.div_opq.d;
            const uint32_t o = fd_div(rem, p.div_pq);
            rem2 = rem - o * p.div_pq.d;
            const int z = (int)o * p.sd + dd_off;
            zin = (unsigned)z < (unsigned)p.D;
            slice = z * p.H * p.W;
        } else {
            n = fd_div(mm, p.div_pq);
            rem = mm - n * p.div_pq.d;
            rem2 = rem;
        }
        const uint32_t pp = fd_div(rem2, p.div_q);
        const uint32_t qq = rem2 - pp * p.div_q.d;
        const int h = (int)pp * p.sh + dh_off;
        const int w = (int)qq * p.sw + dw_off;
        const bool xin = in && zin && (unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W;
        const unsigned half = (lane & 1) * 16;
        const unsigned dy_off = (unsigned)(((n * KB + kb0) * PQ + rem) * 32) + half;
        const unsigned x_off = (unsigned)(((n * CB + cb0) * HW + slice + h * p.W + w) * 32) + half;
        // NCHW operands: lane = channel (lane / 2) % 16 of the plane, positions 16 (lane / 32) + 8 (lane % 2) + 0..7
        // of the block (one tap, stride 1, no padding: the input pixel is the output position)
        bool inn = false;
        unsigned dyn_off = 0, xn_off = 0;
        if constexpr (XN || DN) {
            const uint32_t m2 = m_begin + (uint32_t)(s * WGG_SP + my_blk * 32 + 16 * (lane >> 5) + 8 * (lane & 1));
            inn = m2 < m_end;                                            // chunk ends are multiples of 8
            const uint32_t mm2 = inn ? m2 : 0;
            const uint32_t n2 = fd_div(mm2, p.div_pq);
            const uint32_t pp2 = mm2 - n2 * p.div_pq.d;
            const uint32_t ch = (uint32_t)((lane >> 1) & 15);
            dyn_off = (unsigned)((((size_t)n2 * p.K + kb0 * 16 + ch) * PQ + pp2) * 2);
            xn_off = (unsigned)((((size_t)n2 * p.C + cb0 * 16 + ch) * HW + pp2) * 2);
        }
#pragma unroll
        for (int j = 0; j < NITEM; ++j) {
            const int pl = wave / BLK + (NW / BLK) * j;                  // plane index of item wave + 8 j
            unsigned char *dst = base + pl * WGG_PLANE + my_blk * 1024;
            // channel blocks past K / C (multiples of 16; the last tile may be partial) are loaded as zeros
            if (pl < 4 * WK) {
                const bool live = kb0 + pl < KB;
                unsigned off = (in && live) ? dy_off + (unsigned)(pl * PQ * 32) : WGG_OOB;
                if constexpr (DN) off = (inn && live) ? dyn_off + (unsigned)(pl * PQ * 32) : WGG_OOB;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_dy, (lds_void_g *)dst, 16, (int)off, 0, 0, 0);
            } else {
                const bool live = cb0 + (pl - 4 * WK) < CB;
                unsigned off = (xin && live) ? x_off + (unsigned)((pl - 4 * WK) * HW * 32) : WGG_OOB;
                if constexpr (XN) off = (inn && live) ? xn_off + (unsigned)((pl - 4 * WK) * HW * 32) : WGG_OOB;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (lds_void_g *)dst, 16, (int)off, 0, 0, 0);
            }
        }
    };

    f32x4 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[a][b][v] = 0.f;

    // this lane's byte offset inside a plane for step j: positions 32 j + 4 grp + L/4 (+16), column group
    // L%4; the 64 lanes of one load cover 512 contiguous bytes (no bank conflicts)
    const int lane_off = (grp * 4 + (L >> 2)) * 32 + (L & 3) * 8;
    const int lane_off_n = L * 32 + grp * 8;           // NCHW planes: channel row L, positions 4 grp (+16)

    if (nstages > 0) issue_loads(0, 0);
    for (int s = 0; s < nstages; ++s) {
        __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0): this wave's loads of stage s have landed
        __syncthreads();
        if (s + 1 < nstages) issue_loads(s + 1, (s + 1) & 1);
        const unsigned char *dys = smem + (s & 1) * STAGE + (4 * wk) * WGG_PLANE + (DN ? lane_off_n : lane_off);
        const unsigned char *xs = smem + (s & 1) * STAGE + (4 * WK + 4 * wc) * WGG_PLANE + (XN ? lane_off_n : lane_off);
        auto fetch = [&](int j, bf16x8 (&a)[4], bf16x8 (&b)[4]) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                a[i] = DN ? nchw_frag_g(dys + i * WGG_PLANE + j * 1024) : tr_frag_g(dys + i * WGG_PLANE + j * 1024);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                b[i] = XN ? nchw_frag_g(xs + i * WGG_PLANE + j * 1024) : tr_frag_g(xs + i * WGG_PLANE + j * 1024);
        };
        auto multiply = [&](const bf16x8 (&a)[4], const bf16x8 (&b)[4]) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    acc[i][k] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[k], acc[i][k], 0, 0, 0);
        };
        // step streams continue across stages (BLK steps per stage)
        const int j = (wh - (s * BLK) % NH + NH) % NH;
        if (MS == 2) {
            // two steps of this stage belong to the wave: fetch the second while multiplying the first
            bf16x8 a0[4], b0[4], a1[4], b1[4];
            fetch(j, a0, b0);
            fetch(j + NH, a1, b1);
            multiply(a0, b0);
            multiply(a1, b1);
        } else if (j < BLK) {
            bf16x8 a0[4], b0[4];
            fetch(j, a0, b0);
            multiply(a0, b0);
        }
    }
    __syncthreads();

    // ---- fixed-order tree over the NH step streams, then the partial in register order
    f32x4 *red = reinterpret_cast<f32x4 *>(smem);
    const int sub = wk * WC + wc;
#pragma unroll
    for (int stride = NH / 2; stride >= 1; stride >>= 1) {
        if (wh >= stride && wh < 2 * stride) {
            f32x4 *dst = red + ((wh - stride) * (WK * WC) + sub) * (16 * 64);
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) dst[(a * 4 + b) * 64 + lane] = acc[a][b];
        }
        __syncthreads();
        if (wh < stride) {
            const f32x4 *src = red + (wh * (WK * WC) + sub) * (16 * 64);
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[a][b] += src[(a * 4 + b) * 64 + lane];
        }
        __syncthreads();
    }
    if (wh == 0) {
        // partial[part][tap][tile][sub][kb][cq][lane] (float4 per lane)
        const size_t tile = (size_t)tile_id;
        f32x4 *out = reinterpret_cast<f32x4 *>(p.partial) +
                     ((((size_t)part * ntap_grid + tap) * ntile_grid + tile) * (WK * WC) + sub) * (16 * 64);
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) out[(a * 4 + b) * 64 + lane] = acc[a][b];
    }
}

// dw[k][c][tap] = sum over parts (index order).  Element i (float4) of a part:
// i = ((((tap * tiles + tile) * WK*WC + sub) * 4 + kb) * 4 + cq) * 64 + lane; tiles cover K and C rounded up
// to the tile size, elements outside [K] x [C] are dropped here.
// 256 threads = 256 / SL outputs x SL interleaved part slices (SL = 16 when there are 16 parts or more: more loads
// in flight per output; 8 otherwise), joined in a fixed tree.
template <int SL>
__global__ __launch_bounds__(256) void wgrad_gemm_reduce(const f32x4 *__restrict__ partial, float *__restrict__ dw,
                                                        int nparts, int K, int C, int RS, int ktiles, int ctiles, int WK, int WC)
{
    constexpr int NO = 256 / SL;
    __shared__ f32x4 sm[SL == 1 ? 1 : SL][SL == 1 ? 1 : NO];
    const size_t per4 = (size_t)RS * ktiles * ctiles * WK * WC * (64 * 64 / 4);
    const int o = threadIdx.x % NO;
    const int sl = threadIdx.x / NO;
    const size_t i = (size_t)blockIdx.x * NO + o;
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
        const int lane = (int)(i & 63);
        size_t u = i >> 6;
        const int cq = (int)(u & 3); u >>= 2;
        const int kb = (int)(u & 3); u >>= 2;
        const int sub = (int)(u % (WK * WC)); u /= (WK * WC);
        const int tiles = ktiles * ctiles;
        const int tile = (int)(u % tiles);
        const int tap = (int)(u / tiles);
        const int kt = tile / ctiles, ct = tile - kt * ctiles;
        const int wk = sub / WC, wc = sub - wk * WC;
        const int k = (kt * WK + wk) * 64 + kb * 16 + 4 * (lane >> 4);
        const int c = (ct * WC + wc) * 64 + cq * 16 + (lane & 15);
        if (c < C && k < K) {                                // K % 4 == 0
#pragma unroll
            for (int v = 0; v < 4; ++v) dw[((size_t)(k + v) * C + c) * RS + tap] = r[v];
        }
    }
}

static int wgrad_gemm_taps(const WgradGemmParams &p) { return (p.r3 ? p.T : 1) * p.R * p.S; }

template <int WK, int WC, int SP, bool XN, bool DN, bool R3 = false, bool XO = R3>
static hipError_t launch_wgrad_gemm_l(const WgradGemmParams &p, hipStream_t st)
{
    static LdsLimitOnce lds_limit;                  // per template instantiation
    {
        const hipError_t e = lds_limit.raise(reinterpret_cast<const void *>(&wgrad_gemm_bf16<WK, WC, SP, XN, DN, R3, XO>));
        if (e != hipSuccess) return e;
    }
    size_t lds = (size_t)2 * 4 * (WK + WC) * (SP * 32 + 128);
    if (lds < 65536) lds = 65536;                                       // final cross-wave tree
    dim3 grid(p.nparts, p.ktiles * p.ctiles, wgrad_gemm_taps(p));
    if (XO) grid = dim3(8 * ((p.nparts + 7) / 8) * p.ktiles * p.ctiles * wgrad_gemm_taps(p));
    NGC_LAUNCH((wgrad_gemm_bf16<WK, WC, SP, XN, DN, R3, XO>), grid, dim3(512), lds, st, p);
    return ngc::launch_result();
}

template <int WK, int WC, int SP>
static hipError_t launch_wgrad_gemm_t(const WgradGemmParams &p, hipStream_t st)
{
    if (p.r3) {
        if (p.x_nchw || p.dy_nchw) return hipErrorInvalidValue;
        return launch_wgrad_gemm_l<WK, WC, SP, false, false, true>(p, st);
    }
    if (p.xcd_order) {
        if (p.x_nchw && p.dy_nchw) return launch_wgrad_gemm_l<WK, WC, SP, true, true, false, true>(p, st);
        if (p.x_nchw) return launch_wgrad_gemm_l<WK, WC, SP, true, false, false, true>(p, st);
        if (p.dy_nchw) return launch_wgrad_gemm_l<WK, WC, SP, false, true, false, true>(p, st);
        return launch_wgrad_gemm_l<WK, WC, SP, false, false, false, true>(p, st);
    }
    if (p.x_nchw && p.dy_nchw) return launch_wgrad_gemm_l<WK, WC, SP, true, true>(p, st);
    if (p.x_nchw) return launch_wgrad_gemm_l<WK, WC, SP, true, false>(p, st);
    if (p.dy_nchw) return launch_wgrad_gemm_l<WK, WC, SP, false, true>(p, st);
    return launch_wgrad_gemm_l<WK, WC, SP, false, false>(p, st);
}

template <int SP>
static hipError_t launch_wgrad_gemm_sp(const WgradGemmParams &p, hipStream_t st)
{
    if (p.wk == 2 && p.wc == 2) return launch_wgrad_gemm_t<2, 2, SP>(p, st);
    if (p.wk == 2 && p.wc == 1) return launch_wgrad_gemm_t<2, 1, SP>(p, st);
    if (p.wk == 1 && p.wc == 2) return launch_wgrad_gemm_t<1, 2, SP>(p, st);
    if (p.wk == 1 && p.wc == 1) return launch_wgrad_gemm_t<1, 1, SP>(p, st);
    return hipErrorInvalidValue;
}

hipError_t launch_wgrad_gemm(const WgradGemmParams &p, hipStream_t st)
{
    const hipError_t e = p.sp == 64 ? launch_wgrad_gemm_sp<64>(p, st) : launch_wgrad_gemm_sp<128>(p, st);
    if (e != hipSuccess) return e;
    const int taps = wgrad_gemm_taps(p);
    const size_t per4 = (size_t)taps * p.ktiles * p.ctiles * p.wk * p.wc * (64 * 64 / 4);
    if (p.nparts >= 16)
        NGC_LAUNCH(wgrad_gemm_reduce<16>, dim3((unsigned)(per4 / 16)), dim3(256), 0, st,
                   reinterpret_cast<const f32x4 *>(p.partial), p.dw, p.nparts, p.K, p.C, taps, p.ktiles, p.ctiles, p.wk, p.wc);
    else if (p.nparts > 8)
        NGC_LAUNCH(wgrad_gemm_reduce<8>, dim3((unsigned)(per4 / 32)), dim3(256), 0, st,
                   reinterpret_cast<const f32x4 *>(p.partial), p.dw, p.nparts, p.K, p.C, taps, p.ktiles, p.ctiles, p.wk, p.wc);
    else                                                // a handful of parts: one thread per output adds them itself
        NGC_LAUNCH(wgrad_gemm_reduce<1>, dim3((unsigned)(per4 / 256)), dim3(256), 0, st,
                   reinterpret_cast<const f32x4 *>(p.partial), p.dw, p.nparts, p.K, p.C, taps, p.ktiles, p.ctiles, p.wk, p.wc);
    return ngc::launch_result();
}

}  // namespace ngc
