// Low-channel "stem" convolution forward (C <= 3, 7x7, stride 2, pad_w 3) on bf16 MFMA (gfx950).
//
// x stays in NCHW (a 16-channel-blocked copy of a 3-channel tensor would be 5.3x its size); y is
// written 16-channel-blocked with the fused bias + ReLU epilogue.  The op is bound by the write
// of y (51 flop per byte of y), so the kernel is organised around streaming: one workgroup per
// tile of TP output rows x full width, several workgroups resident per CU so that one's patch
// load, another's MFMAs and a third's stores overlap.
//
// Implicit GEMM: rows = 64 output channels, columns = positions, reduction = (c, r) pairs x 8
// "slots".  For a fixed (c, r) the 7 taps s = 0..6 of position (p, q) are the 7 consecutive
// input pixels 2q-3 .. 2q+3 of input row 2p-pad+r; with one extra pixel in front (slot 0, weight
// 0) they are 8 consecutive bf16 starting at the even column 2q-4: exactly the 8 reduction
// elements one MFMA lane supplies, and dword-aligned in an LDS copy of the input row.  One
// v_mfma_f32_32x32x16_bf16 consumes two (c, r) pairs (lane groups 0 / 1); 21 pairs -> 11 MFMAs
// per 32 positions x 32 channels (147 of 176 reduction slots useful).
// The 22 filter fragments of a lane live in registers for the whole workgroup.
#include "common.h"

namespace ngc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int STEM_KSTEPS = 11;      // ceil(21 pairs / 2)

__global__ __launch_bounds__(256) void conv_stem_fwd_bf16(const StemFwdParams p)
{
    preload_kernargs(p);
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l32 = lane & 31;
    const int lg = lane >> 5;

    const int tile = blockIdx.x;
    const int n = tile / p.tiles_per_img;
    const int p0 = (tile - n * p.tiles_per_img) * p.TP;
    const int k0 = blockIdx.y * 64;

    const int rows_in = 2 * p.TP + 5;
    const int RP = 2 * p.W + 16;                      // LDS row pitch in bytes: 8 pad + W bf16 + 8 pad
    const int patch_bytes = p.C * rows_in * RP;
    unsigned char *wlds = smem + ((patch_bytes + 15) & ~15);
    const int npairs = p.C * 7;
    const int CRS = p.C * 49;

    // ---- stage the 64 x (C*49) filter slab (contiguous in KCRS) and the input patch
    {
        const uint4 *src = reinterpret_cast<const uint4 *>(p.w + (size_t)k0 * CRS);
        const int n16 = (64 * CRS * 2) / 16;          // 64*CRS*2 bytes is a multiple of 16 (64*2 = 128)
        for (int i = tid; i < n16; i += 256) reinterpret_cast<uint4 *>(wlds)[i] = src[i];
    }
    {
        const int cpr = p.W >> 3;                     // 16-byte chunks per input row
        const int total = p.C * rows_in * cpr;
        for (int i = tid; i < total; i += 256) {
            const int rr = (int)fd_div((uint32_t)i, p.div_cpr);          // c * rows_in + row
            const int ch = i - rr * cpr;
            const int c = (int)fd_div((uint32_t)rr, p.div_rows);
            const int row = rr - c * rows_in;
            const int h = 2 * p0 - p.pbh + row;
            uint4 v = make_uint4(0, 0, 0, 0);
            if ((unsigned)h < (unsigned)p.H)
                v = *reinterpret_cast<const uint4 *>(p.x + (((size_t)n * p.C + c) * p.H + h) * p.W + ch * 8);
            unsigned char *dst = smem + rr * RP + 8 + ch * 16;
            *reinterpret_cast<uint2 *>(dst) = make_uint2(v.x, v.y);
            *reinterpret_cast<uint2 *>(dst + 8) = make_uint2(v.z, v.w);
            if (ch == 0) *reinterpret_cast<uint2 *>(smem + rr * RP) = make_uint2(0, 0);
            if (ch == cpr - 1) *reinterpret_cast<uint2 *>(smem + rr * RP + RP - 8) = make_uint2(0, 0);
        }
    }
    __syncthreads();

    // ---- this lane's filter fragments: step t, lane group lg -> pair 2t+lg = (c, r); slot j>0 = tap s=j-1
    bf16x8 wa[STEM_KSTEPS][2];
    int rowoff[STEM_KSTEPS];
#pragma unroll
    for (int t = 0; t < STEM_KSTEPS; ++t) {
        const int pair = 2 * t + lg;
        const bool real = pair < npairs;
        const int c = real ? pair / 7 : 0;
        const int r = real ? pair - c * 7 : 0;
        rowoff[t] = (c * rows_in + r) * RP;
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            const uint16_t *wk = reinterpret_cast<const uint16_t *>(wlds) + (size_t)(a * 32 + l32) * CRS + (c * 7 + r) * 7;
            union { uint16_t h[8]; bf16x8 v; } u;
            u.h[0] = 0;
#pragma unroll
            for (int j = 1; j < 8; ++j) u.h[j] = real ? wk[j - 1] : (uint16_t)0;
            wa[t][a] = u.v;
        }
    }

    const int npos = p.TP * p.Q;
    const int nfrags = (npos + 31) >> 5;
    const int CBout = p.K >> 4;
    const int PQ = p.P * p.Q;

    float4 bv[2][2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            bv[a][h][0] = bv[a][h][1] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (p.bias) {
                bv[a][h][0] = *reinterpret_cast<const float4 *>(p.bias + k0 + a * 32 + 16 * h + 4 * lg);
                bv[a][h][1] = *reinterpret_cast<const float4 *>(p.bias + k0 + a * 32 + 16 * h + 8 + 4 * lg);
            }
        }

    // y below 2 GiB: 16-byte stores with 32-bit offsets into a buffer descriptor, positions outside the tile get an
    // out-of-range offset (no 64-bit address arithmetic, no divergent branch per store)
    const bool store32 = p.y_bytes != 0;
    __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc((void *)p.y, 0, (int)p.y_bytes, 0x00020000);
    const int relu_on = p.relu;
    for (int f = wave; f < nfrags; f += 4) {
        const uint32_t m = (uint32_t)(f * 32 + l32);
        bool ok = m < (uint32_t)npos;
        const uint32_t mm = ok ? m : 0;
        const uint32_t pr = fd_div(mm, p.div_q);
        const uint32_t q = mm - pr * p.div_q.d;
        ok = ok && (p0 + (int)pr) < p.P;
        const unsigned char *base = smem + (2 * pr) * RP + q * 4;

        f32x16 acc[2];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][v] = 0.f;
#pragma unroll
        for (int t = 0; t < STEM_KSTEPS; ++t) {
            const uint32_t *src = reinterpret_cast<const uint32_t *>(base + rowoff[t]);
            union { uint32_t d[4]; bf16x8 v; } u;
            u.d[0] = src[0]; u.d[1] = src[1]; u.d[2] = src[2]; u.d[3] = src[3];
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa[t][0], u.v, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa[t][1], u.v, acc[1], 0, 0, 0);
        }

        // epilogue: bias, ReLU, one RNE rounding, lane-pair exchange, 16-byte stores
        const size_t pix = (size_t)n * CBout * PQ + (size_t)(p0 + pr) * p.Q + q;
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            const int co_base = k0 + a * 32;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = acc[a][8 * h + e];
                const float4 b0 = bv[a][h][0], b1 = bv[a][h][1];
                v[0] += b0.x; v[1] += b0.y; v[2] += b0.z; v[3] += b0.w;
                v[4] += b1.x; v[5] += b1.y; v[6] += b1.z; v[7] += b1.w;
                const uint32_t q0 = relu_bf16x2(pack_bf16x2_hw(v[0], v[1]), relu_on), q1 = relu_bf16x2(pack_bf16x2_hw(v[2], v[3]), relu_on);
                const uint32_t q2 = relu_bf16x2(pack_bf16x2_hw(v[4], v[5]), relu_on), q3 = relu_bf16x2(pack_bf16x2_hw(v[6], v[7]), relu_on);
                const uint4 o = lane_pair_exchange(q0, q1, q2, q3);
                if (store32) {
                    const unsigned off = ok ? ((unsigned)pix + (unsigned)(((co_base >> 4) + h) * PQ)) * 32u + (unsigned)(lg * 16)
                                            : 0x80000000u;
                    ngc_u32x4 ov = {o.x, o.y, o.z, o.w};
                    __builtin_amdgcn_raw_buffer_store_b128(ov, rs_y, (int)off, 0, NGC_ST_AUX);
                } else if (ok) {
                    const size_t blk = pix + (size_t)((co_base >> 4) + h) * PQ;
                    store16_result(p.y + blk * 16 + lg * 8, o, true);
                }
            }
        }
    }
}

hipError_t launch_stem_fwd(const StemFwdParams &p, size_t lds_bytes, hipStream_t st)
{
    dim3 grid(p.N * p.tiles_per_img, p.K / 64);
    NGC_LAUNCH(conv_stem_fwd_bf16, grid, dim3(256), lds_bytes, st, p);
    return ngc::launch_result();
}

}  // namespace ngc
