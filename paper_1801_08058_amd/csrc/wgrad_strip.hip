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
// The strip is processed in stages of SR rows.  A stage brings into LDS, with direct
// global->LDS loads (16 bytes per lane; out-of-range lanes deliver zeros, which is the padding
// halo and the tail of the strip):
//     dy tile : [positions][64 k]   as 4 planes of [position][16 k]  (32-byte rows)
//     x patch : [(SR+2) x (Q+2) px][64 c] as 4 planes of [pixel][16 c]
// i.e. both in their natural channel-contiguous form.  The MFMA needs the reduction axis
// (positions) contiguous per lane; the LDS transpose load ds_read_b64_tr_b16 does exactly that:
// 16 lanes read a 4(position) x 16(channel) block and each lane receives one channel's 4
// positions.  Two such loads give a lane its 8 reduction elements of v_mfma_f32_16x16x32_bf16
// (lane group l/16 = positions +8*(l/16)).  Because rows of the transposed block are whole
// 32-byte pixels, a filter tap is just a pixel offset in the address (no alignment problem, no
// shifted copies).
//
// Per 32-position step a wave issues 8 (dy) + 18 (x, 9 taps) transpose loads for 36 MFMAs; x
// fragments run three taps ahead of the MFMAs in a rolling 3-slot buffer (across step
// boundaries), the dy fragments of the wave's next step are fetched during the current one.
// The per-workgroup partial [tap][k][c] goes to the workspace; wgrad_strip_reduce adds the
// workgroups in index order (deterministic) and writes dw as [K][C][R][S].
#include "common.h"

namespace ngc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr unsigned WS_OOB = 0x80000000u;
constexpr int WS_NT = 9;

__device__ __forceinline__ bf16x8 tr_frag(const unsigned char *lo, const unsigned char *hi)
{
    // two 4x16 transposed blocks -> this lane's 8 reduction elements
    const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)lo);
    const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)hi);
    const s16x8 r = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

template <int NW>
__global__ __launch_bounds__(NW * 64) void wgrad_strip_bf16(const WgradStripParams p)
{
    constexpr int NH = NW / 4;               // waves per channel quarter = step interleave
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cq = wave & 3;                 // 16-channel quarter of the 64 c
    const int wh = wave >> 2;                // step parity (NW = 8)
    const int L = lane & 15;                 // lane inside its 16-lane transpose group
    const int grp = lane >> 4;               // reduction group: positions +8*grp

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
    const int stage_bytes = 4 * p.dyplane + 4 * p.xplane;

    __amdgpu_buffer_rsrc_t rs_dy = __builtin_amdgcn_make_buffer_rsrc((void *)p.dy, 0, (int)p.dy_bytes, 0x00020000);
    __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, (int)p.x_bytes, 0x00020000);

    const int npatch = p.PRS * p.PC;
    const int nblk_x = (npatch + 31) >> 5;
    const int steps_full = (p.SR * p.Q + 31) >> 5;           // 32-position steps of a full stage
    const int nblk_dy = steps_full;

    // waves (cq, h) share plane cq (16 k of dy, 16 c of x) of every stage: blocks h, h+NH, ...
    auto issue_loads = [&](int stage_lin, int buf) {
        const int img = n0 + stage_lin / p.nstages;                      // stages run image by image
        const int stage_i = stage_lin - (stage_lin / p.nstages) * p.nstages;
        unsigned char *dys = smem + buf * stage_bytes + cq * p.dyplane;
        unsigned char *xs = smem + buf * stage_bytes + 4 * p.dyplane + cq * p.xplane;
        const int r0 = stage_i * p.SR;                                   // first strip row of the stage
        int rows = rows_strip - r0;
        if (rows > p.SR) rows = p.SR;
        const int nvalid = rows * p.Q;                                   // positions of the stage that exist
        const unsigned dy_base = (unsigned)((((img * KB + kt * 4 + cq) * PQ) + (p0 + r0) * p.Q) * 32);
        for (int blk = wh; blk < nblk_dy; blk += NH) {
            const int pos = blk * 32 + (lane >> 1);
            const unsigned off = (pos < nvalid) ? dy_base + (unsigned)(pos * 32 + (lane & 1) * 16) : WS_OOB;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_dy, (lds_void_t *)(dys + blk * 1024), 16, (int)off, 0, 0, 0);
        }
        const unsigned x_base = (unsigned)(((img * CB + ct * 4 + cq) * HW) * 32);
        const int h0 = p0 + r0 + p.min_dh;
        for (int blk = wh; blk < nblk_x; blk += NH) {
            const uint32_t px = (uint32_t)(blk * 32 + (lane >> 1));
            const uint32_t pr = fd_div(px, p.div_pc);
            const uint32_t pc = px - pr * p.div_pc.d;
            const int h = h0 + (int)pr;
            const int w = p.min_dw + (int)pc;
            const bool ok = px < (uint32_t)npatch && (unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W;
            const unsigned off = ok ? x_base + (unsigned)((h * p.W + w) * 32 + (lane & 1) * 16) : WS_OOB;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (lds_void_t *)(xs + blk * 1024), 16, (int)off, 0, 0, 0);
        }
    };

    f32x4 acc[4][WS_NT];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int t = 0; t < WS_NT; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[a][t][v] = 0.f;

    const int last_pos = p.SR * p.Q - 1;
    // byte offset of this lane inside a transposed 4x16 block: row L/4 (32 B each), 8-byte column group L%4
    const int lane_col = (L & 3) * 8;

    // LDS byte offsets of this lane's two 4-position groups of a 32-position step
    auto step_offsets = [&](int step, int (&dyoff)[2], int (&xoff)[2]) {
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            int pos = step * 32 + grp * 8 + e * 4 + (L >> 2);
            dyoff[e] = pos * 32 + lane_col;
            if (pos > last_pos) pos = last_pos;                          // dy is zero there; keep x in range
            const uint32_t row = fd_div((uint32_t)pos, p.div_q);
            const uint32_t col = (uint32_t)pos - row * p.div_q.d;
            xoff[e] = (int)(row * p.PC + col) * 32 + lane_col;
        }
    };

    const int total_stages = nimg * p.nstages;
    issue_loads(0, 0);
    for (int s = 0; s < total_stages; ++s) {
        __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0): this wave's loads of stage s have landed
        __syncthreads();
        if (s + 1 < total_stages) issue_loads(s + 1, (s + 1) & 1);
        int rows = rows_strip - (s % p.nstages) * p.SR;
        if (rows > p.SR) rows = p.SR;
        const int nsteps = (rows * p.Q + 31) >> 5;          // steps that contain at least one position
        const unsigned char *dys = smem + (s & 1) * stage_bytes;
        const unsigned char *xs = smem + (s & 1) * stage_bytes + 4 * p.dyplane + cq * p.xplane;
        auto load_a = [&](const int (&dyoff)[2], bf16x8 (&a)[4]) {
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) a[kb] = tr_frag(dys + kb * p.dyplane + dyoff[0], dys + kb * p.dyplane + dyoff[1]);
        };
        auto load_b = [&](const int (&xoff)[2], int t) {
            return tr_frag(xs + xoff[0] + p.tap_off[t] * 32, xs + xoff[1] + p.tap_off[t] * 32);
        };

        int j = wh;
        if (j < nsteps) {
            int dyo[2], xo[2], dyn[2], xn[2];
            bf16x8 acur[4], anext[4], b[3];
            step_offsets(j, dyo, xo);
            load_a(dyo, acur);
#pragma unroll
            for (int t = 0; t < 3; ++t) b[t] = load_b(xo, t);
            while (true) {
                const bool has_next = j + NH < nsteps;
                step_offsets(has_next ? j + NH : j, dyn, xn);
#pragma unroll
                for (int kb = 0; kb < 4; ++kb) anext[kb] = acur[kb];
#pragma unroll
                for (int t = 0; t < WS_NT; ++t) {
#pragma unroll
                    for (int kb = 0; kb < 4; ++kb)
                        acc[kb][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(acur[kb], b[t % 3], acc[kb][t], 0, 0, 0);
                    // refill the slot just consumed: tap t+3 of this step, or tap t+3-9 of the next
                    if (t + 3 < WS_NT) b[t % 3] = load_b(xo, t + 3);
                    else if (has_next) b[t % 3] = load_b(xn, t + 3 - WS_NT);
                    if (t == 2 && has_next) load_a(dyn, anext);
                }
                if (!has_next) break;
#pragma unroll
                for (int kb = 0; kb < 4; ++kb) acur[kb] = anext[kb];
#pragma unroll
                for (int e = 0; e < 2; ++e) { dyo[e] = dyn[e]; xo[e] = xn[e]; }
                j += NH;
            }
        }
    }
    __syncthreads();                                        // all stage buffers are free

    // ---- sum the step-parity copies (waves h=1 publish, h=0 add) and write the partial tile.
    // Accumulator register v of tile (kb, t): k = 16 kb + 4*(lane/16) + v, c = 16 cq + lane%16.
    float *red = reinterpret_cast<float *>(smem) + cq * (4 * WS_NT * 4 * 64);     // 144 floats per lane
    if (NH == 2 && wh == 1) {
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
            for (int t = 0; t < WS_NT; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) red[((kb * WS_NT + t) * 4 + v) * 64 + lane] = acc[kb][t][v];
    }
    __syncthreads();
    if (wh == 0) {
        float *out = p.partial + (size_t)blockIdx.x * WS_NT * p.K * p.C;
        const int c = ct * 64 + cq * 16 + L;
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
            for (int t = 0; t < WS_NT; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int k = kt * 64 + kb * 16 + 4 * grp + v;
                    float r = acc[kb][t][v];
                    if (NH == 2) r += red[((kb * WS_NT + t) * 4 + v) * 64 + lane];
                    out[((size_t)t * p.K + k) * p.C + c] = r;
                }
    }
}

// dw[k][c][tap] = sum over workgroup partials (index order) of partial[i][tap][k][c].
// 256 threads = 64 outputs x 4 interleaved partial streams, joined in a fixed order.
__global__ __launch_bounds__(256) void wgrad_strip_reduce(const float *__restrict__ partial, float *__restrict__ dw,
                                                         int nparts, int K, int C, int RS)
{
    __shared__ float sm[4][64];
    const size_t per = (size_t)RS * K * C;
    const int o = threadIdx.x & 63;
    const int sl = threadIdx.x >> 6;
    const size_t i = (size_t)blockIdx.x * 64 + o;
    float acc = 0.f;
    if (i < per) {
        float t0 = 0.f, t1 = 0.f, t2 = 0.f, t3 = 0.f;
        int sp = sl;
        for (; sp + 12 < nparts; sp += 16) {
            t0 += partial[(size_t)sp * per + i];
            t1 += partial[(size_t)(sp + 4) * per + i];
            t2 += partial[(size_t)(sp + 8) * per + i];
            t3 += partial[(size_t)(sp + 12) * per + i];
        }
        for (; sp < nparts; sp += 4) t0 += partial[(size_t)sp * per + i];
        acc = (t0 + t1) + (t2 + t3);
    }
    sm[sl][o] = acc;
    __syncthreads();
    if (sl == 0 && i < per) {
        const float r = (sm[0][o] + sm[1][o]) + (sm[2][o] + sm[3][o]);
        const int c = (int)(i % C);
        const size_t t = i / C;
        const int k = (int)(t % K);
        const int tap = (int)(t / K);
        dw[((size_t)k * C + c) * RS + tap] = r;
    }
}

hipError_t launch_wgrad_strip(const WgradStripParams &p, size_t lds_bytes, hipStream_t st)
{
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&wgrad_strip_bf16<8>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid(p.nparts, (p.K / 64) * p.ctiles);
    hipLaunchKernelGGL(wgrad_strip_bf16<8>, grid, dim3(512), lds_bytes, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t per = (size_t)WS_NT * p.K * p.C;
    hipLaunchKernelGGL(wgrad_strip_reduce, dim3((unsigned)((per + 63) / 64)), dim3(256), 0, st, p.partial, p.dw,
                       p.nparts, p.K, p.C, WS_NT);
    return hipGetLastError();
}

}  // namespace ngc
