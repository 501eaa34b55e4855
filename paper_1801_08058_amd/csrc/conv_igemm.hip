// Implicit-GEMM convolution on bf16 MFMA (gfx950), fp32 accumulate.
//
// One kernel serves Convolution forward and ConvolutionBackpropData.  Both are written as a
// "generalised gather convolution" over 16-channel-blocked tensors:
//
//   out[n, co, i*os+oa, j*os+oa'] = sum_{tap t} sum_{ci} in[n, ci, i*is + t.dh, j*is + t.dw]
//                                                       * wt[t.slab][ci/16][co][ci%16]
//
//   forward      : is = window stride, os = 1, one class, taps (r,s) with dh = r*dil - pad_below
//   backprop-data: is = 1, os = window stride, one class per residue (a,b) of the output pixel
//                  modulo the stride; class (a,b) holds the taps with (a + pad_below - r*dil)
//                  divisible by the stride, dh = that quotient (so no multiply by the zeros of
//                  a zero-stuffed dy), filter slabs in the [r][s][kb][c][ki] layout.
//
// GEMM view per class: M = N*OP*OQ output positions, N = Cout, K = taps * Cin.
// Workgroup = 256 threads = 4 waves; tile BM positions x BN output channels; each wave owns
// 64 positions x 64 channels = 2x2 MFMA 32x32x16 accumulators (64 VGPRs).
// Reduction step = one tap x 32 input channels.  Per step the workgroup gathers
//   X tile  [BM positions][32 ci]   (im2col on the fly, zero outside the image)
//   W tile  [BN co][32 ci]
// from global memory into registers (prefetch of step s+1 overlaps the MFMAs of step s), then
// into a double-buffered LDS stage; one barrier per step.
//
// LDS layout: every tile is split into 4 planes (cb in {0,1}) x (g in {0,1}); plane (cb,g)
// holds, for each row (position or co), the 8 channels 16*cb + 8*g .. +7 as one 16-byte unit.
// An MFMA operand fetch is then one ds_read_b128 per lane with lanes 0-31 reading 32
// consecutive 16-byte units of plane g=0 and lanes 32-63 of plane g=1 (conflict free); plane
// pitch is = 128 mod 256 bytes so the two halves of a wave never share a bank group.
//
// MFMA roles: A = filters (rows = output channels), B = activations (columns = positions).
// v_mfma_f32_32x32x16_bf16: lane l supplies 8 consecutive reduction elements of row/column
// l%32 (group l/32); accumulator register v of lane l is D[8*(v/4) + 4*(l/32) + v%4][l%32].
// A lane therefore ends with 4 consecutive output channels per register quad for its own
// position; one cross-half exchange (lane l <-> l+32) turns that into 8 consecutive channels
// = one 16-byte store into the blocked output, so every store instruction of a wave writes
// whole 32-byte pixel blocks.
#include "common.h"

namespace ngc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

static_assert(sizeof(IgemmParams) <= 4096, "kernel arguments are passed by value: at most 4 KB");

template <int BM, int BN>
struct IgemmCfg {
    static constexpr int WM = BM / 64;                  // waves along positions
    static constexpr int WN = BN / 64;                  // waves along output channels
    static constexpr int XPLANE = BM * 16 + 128;        // bytes
    static constexpr int WPLANE = BN * 16 + 128;
    static constexpr int STAGE = 4 * XPLANE + 4 * WPLANE;
    static constexpr int XE = BM / 128;                 // positions gathered per thread
    static constexpr int WU = BN / 64;                  // filter 16-byte units per thread
    static_assert(WM * WN == 4, "4 waves per workgroup");
};

// R3: rank-3 spatial tensors [N][C/16][D][H][W][16]; positions are (n, o, i, j) and every tap carries a
// depth offset as well.
template <int BM, int BN, bool R3>
__global__ __launch_bounds__(256) void igemm_bf16(const IgemmParams p)
{
    preload_kernargs(p);
    using Cfg = IgemmCfg<BM, BN>;
    __shared__ __align__(16) unsigned char smem[2 * Cfg::STAGE];

    const IgemmClass &cl = p.cls[blockIdx.z];
    const uint32_t m0 = blockIdx.x * BM;
    if (m0 >= cl.M) return;                              // uniform per workgroup
    const int n0 = blockIdx.y * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave % Cfg::WM;
    const int wn = wave / Cfg::WM;
    const int l32 = lane & 31;
    const int lg = lane >> 5;

    const int CBin = p.Cin >> 4;
    const int HWin = p.Hin * p.Win;
    const int DHWin = R3 ? p.Din * HWin : HWin;          // pixel blocks per 16-channel plane of an image

    // ---- gather bookkeeping: this thread loads position rows (tid/2 + 128 e), half g = tid&1
    const int ldg = tid & 1;
    int ld_ih0[Cfg::XE], ld_iw0[Cfg::XE], ld_base[Cfg::XE], ld_id0[Cfg::XE];
    bool ld_ok[Cfg::XE];
#pragma unroll
    for (int e = 0; e < Cfg::XE; ++e) {
        const uint32_t m = m0 + (tid >> 1) + 128 * e;
        ld_ok[e] = m < cl.M;
        const uint32_t mm = ld_ok[e] ? m : 0;
        uint32_t n, rem, o = 0;
        if constexpr (R3) {
            n = fd_div(mm, cl.div_opq);
            const uint32_t rem3 = mm - n * cl.div_opq.d;
            o = fd_div(rem3, cl.div_pq);
            rem = rem3 - o * cl.div_pq.d;
        } else {
            n = fd_div(mm, cl.div_pq);
            rem = mm - n * cl.div_pq.d;
        }
        const uint32_t i = fd_div(rem, cl.div_q);
        const uint32_t j = rem - i * cl.div_q.d;
        ld_ih0[e] = (int)i * p.is_h;
        ld_iw0[e] = (int)j * p.is_w;
        ld_id0[e] = R3 ? (int)o * p.is_d : 0;
        ld_base[e] = (int)n * CBin * DHWin;              // in units of 16-channel pixel blocks
    }
    // filter units: unit q = tid + 256 u -> g = q&1, row = (q/2) % BN, cbi = (q/2) / BN
    const int w_row = (tid >> 1) % BN;
    const int w_cbi0 = (tid >> 1) / BN;                  // 0 for BN=128; 0/1 for BN=64

    uint4 xr[Cfg::XE][2];
    uint4 wr[Cfg::WU];

    const int c32_count = p.Cin >> 5;
    const int nsteps = cl.tap_count * c32_count;

    auto load_global = [&](int tap_i, int c32) {
        const IgemmTap tp = p.taps[cl.tap_begin + tap_i];
#pragma unroll
        for (int e = 0; e < Cfg::XE; ++e) {
            const int ih = ld_ih0[e] + tp.dh;
            const int iw = ld_iw0[e] + tp.dw;
            bool ok = ld_ok[e] && (unsigned)ih < (unsigned)p.Hin && (unsigned)iw < (unsigned)p.Win;
            int slice = 0;
            if constexpr (R3) {
                const int id = ld_id0[e] + tp.dd;
                ok = ok && (unsigned)id < (unsigned)p.Din;
                slice = id * HWin;
            }
#pragma unroll
            for (int cbi = 0; cbi < 2; ++cbi) {
                uint4 v = make_uint4(0, 0, 0, 0);
                if (ok) {
                    const size_t blk = (size_t)(ld_base[e] + (c32 * 2 + cbi) * DHWin + slice + ih * p.Win + iw);
                    v = *reinterpret_cast<const uint4 *>(p.in + blk * 16 + ldg * 8);
                }
                xr[e][cbi] = v;
            }
        }
#pragma unroll
        for (int u = 0; u < Cfg::WU; ++u) {
            const int cbi = (BN == 128) ? u : w_cbi0;
            const size_t row = ((size_t)tp.slab * CBin + (c32 * 2 + cbi)) * p.Cout + n0 + w_row;
            // through a named value: assigned straight from the dereference, wr[] was kept in scratch memory
            const uint4 t = *reinterpret_cast<const uint4 *>(p.wt + row * 16 + ldg * 8);
            wr[u] = t;
        }
    };

    auto store_lds = [&](int stage) {
        unsigned char *xs = smem + stage * Cfg::STAGE;
        unsigned char *ws = xs + 4 * Cfg::XPLANE;
#pragma unroll
        for (int e = 0; e < Cfg::XE; ++e)
#pragma unroll
            for (int cbi = 0; cbi < 2; ++cbi)
                *reinterpret_cast<uint4 *>(xs + (cbi * 2 + ldg) * Cfg::XPLANE + ((tid >> 1) + 128 * e) * 16) = xr[e][cbi];
#pragma unroll
        for (int u = 0; u < Cfg::WU; ++u) {
            const int cbi = (BN == 128) ? u : w_cbi0;
            *reinterpret_cast<uint4 *>(ws + (cbi * 2 + ldg) * Cfg::WPLANE + w_row * 16) = wr[u];
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    if (nsteps > 0) {
        load_global(0, 0);
        store_lds(0);
    }
    __syncthreads();

    int tap_i = 0, c32 = 0;
    for (int s = 0; s < nsteps; ++s) {
        int ntap = tap_i, nc32 = c32 + 1;
        if (nc32 == c32_count) { nc32 = 0; ++ntap; }
        const bool more = (s + 1 < nsteps);
        if (more) load_global(ntap, nc32);

        const unsigned char *xs = smem + (s & 1) * Cfg::STAGE;
        const unsigned char *ws = xs + 4 * Cfg::XPLANE;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 fa[2], fb[2];
#pragma unroll
            for (int a = 0; a < 2; ++a)
                fa[a] = *reinterpret_cast<const bf16x8 *>(ws + (ks * 2 + lg) * Cfg::WPLANE + (wn * 64 + a * 32 + l32) * 16);
#pragma unroll
            for (int b = 0; b < 2; ++b)
                fb[b] = *reinterpret_cast<const bf16x8 *>(xs + (ks * 2 + lg) * Cfg::XPLANE + (wm * 64 + b * 32 + l32) * 16);
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
        }

        if (more) store_lds((s + 1) & 1);
        __syncthreads();
        tap_i = ntap;
        c32 = nc32;
    }

    // ---- epilogue: bias, ReLU, one RNE rounding, 16-byte stores into the blocked output
    const int CBout = p.Cout >> 4;
    const int HWplane = p.Hout * p.Wout;
    const int HWout = R3 ? p.Dout * HWplane : HWplane;   // pixel blocks per 16-channel plane of an image
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const uint32_t m = m0 + wm * 64 + b * 32 + l32;
        const bool ok = m < cl.M;
        const uint32_t mm = ok ? m : 0;
        uint32_t n, rem, o = 0;
        if constexpr (R3) {
            n = fd_div(mm, cl.div_opq);
            const uint32_t rem3 = mm - n * cl.div_opq.d;
            o = fd_div(rem3, cl.div_pq);
            rem = rem3 - o * cl.div_pq.d;
        } else {
            n = fd_div(mm, cl.div_pq);
            rem = mm - n * cl.div_pq.d;
        }
        const uint32_t i = fd_div(rem, cl.div_q);
        const uint32_t j = rem - i * cl.div_q.d;
        const int oh = (int)i * p.os_h + cl.oa_h;
        const int ow = (int)j * p.os_w + cl.oa_w;
        size_t pix = (size_t)n * CBout * HWout + (size_t)oh * p.Wout + ow;
        if constexpr (R3) pix += (size_t)((int)o * p.os_d + cl.oa_d) * HWplane;
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            const int co_base = n0 + wn * 64 + a * 32;     // first output channel of this 32-row fragment
#pragma unroll
            for (int h = 0; h < 2; ++h) {                  // 16-channel block inside the fragment
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = acc[a][b][8 * h + e];
                // v[0..3] -> channels 16h + 4*lg + 0..3 ; v[4..7] -> channels 16h + 8 + 4*lg + 0..3
                if (p.bias) {
                    const float4 b0 = *reinterpret_cast<const float4 *>(p.bias + co_base + 16 * h + 4 * lg);
                    const float4 b1 = *reinterpret_cast<const float4 *>(p.bias + co_base + 16 * h + 8 + 4 * lg);
                    v[0] += b0.x; v[1] += b0.y; v[2] += b0.z; v[3] += b0.w;
                    v[4] += b1.x; v[5] += b1.y; v[6] += b1.z; v[7] += b1.w;
                }
                const bool relu_on = p.relu != 0;                        // ReLU on the rounded pairs: see relu_bf16x2
                const uint32_t p0 = relu_bf16x2(pack_bf16x2_hw(v[0], v[1]), relu_on), p1 = relu_bf16x2(pack_bf16x2_hw(v[2], v[3]), relu_on);
                const uint32_t p2 = relu_bf16x2(pack_bf16x2_hw(v[4], v[5]), relu_on), p3 = relu_bf16x2(pack_bf16x2_hw(v[6], v[7]), relu_on);
                // lg=0 owns channels {0-3, 8-11}, lg=1 owns {4-7, 12-15}; swap so that
                // lg=0 ends with 0-7 and lg=1 with 8-15
                uint4 o = lane_pair_exchange(p0, p1, p2, p3);
                if (ok) {
                    const size_t blk = pix + (size_t)((co_base >> 4) + h) * HWout;
                    if (p.mask) o = relu_keep8(o, *reinterpret_cast<const uint4 *>(p.mask + blk * 16 + lg * 8));
                    store16_result(p.out + blk * 16 + lg * 8, o, p.os_h == 1 && p.os_w == 1);
                }
            }
        }
    }
}

template <bool R3>
static hipError_t launch_igemm_r(const IgemmParams &p, int bn, uint32_t max_m, hipStream_t st)
{
    if (bn == 128) {
        dim3 grid((max_m + 127) / 128, p.Cout / 128, p.ncls);
        NGC_LAUNCH((igemm_bf16<128, 128, R3>), grid, dim3(256), 0, st, p);
    } else {
        dim3 grid((max_m + 255) / 256, p.Cout / 64, p.ncls);
        NGC_LAUNCH((igemm_bf16<256, 64, R3>), grid, dim3(256), 0, st, p);
    }
    return ngc::launch_result();
}

hipError_t launch_igemm(const IgemmParams &p, int bn, uint32_t max_m, hipStream_t st)
{
    return launch_igemm_r<false>(p, bn, max_m, st);
}

hipError_t launch_igemm3(const IgemmParams &p, int bn, uint32_t max_m, hipStream_t st)
{
    return launch_igemm_r<true>(p, bn, max_m, st);
}

}  // namespace ngc
