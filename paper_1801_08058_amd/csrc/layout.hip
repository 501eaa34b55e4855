// Data-layout conversion kernels: NCHW <-> 16-channel-blocked, and the filter re-layouts.
// Pure permutations of bit patterns (paper Abstract / Sec. 2: data layout abstraction).
// HBM bound: 1 read + 1 write per element.  The fast 2-byte path transposes a
// 16(channel) x 256(pixel) tile through LDS so that both the NCHW side (contiguous in
// pixels) and the blocked side (contiguous in channels, then pixels) move as full lines.
#include "common.h"

namespace ngc {

constexpr int LT_PIX = 256;          // pixels per tile
constexpr int LT_PITCH = LT_PIX + 2; // LDS row pitch in elements (odd dword count: 129 dwords)

// ---- NCHW -> blocked, 2-byte elements.  grid = (ceil(HW/256), CB, N), block = 256.
// V = pixels per global read (1, 2, 4 or 8), chosen by the host from the alignment of HW.
template <int V>
__global__ __launch_bounds__(256) void nchw_to_blocked16_b16(const uint16_t *__restrict__ src,
                                                             uint16_t *__restrict__ dst, int C, int HW)
{
    __shared__ __align__(16) uint16_t tile[16 * LT_PITCH];
    const int tid = threadIdx.x;
    const int px0 = blockIdx.x * LT_PIX;
    const int cb = blockIdx.y;
    const int n = blockIdx.z;
    const int CB = gridDim.y;

    // read phase: 16 channel rows x 256 pixels, V pixels per access
    constexpr int ACC_PER_ROW = LT_PIX / V;
    constexpr int ITERS = 16 * ACC_PER_ROW / 256;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int a = tid + 256 * it;
        const int ci = a / ACC_PER_ROW;
        const int px = (a % ACC_PER_ROW) * V;
        const int c = cb * 16 + ci;
        uint16_t v[V];
#pragma unroll
        for (int e = 0; e < V; ++e) v[e] = 0;
        if (c < C && px0 + px < HW) {                     // HW % V == 0 so a vector is all-in or all-out
            const uint16_t *g = src + ((size_t)n * C + c) * HW + px0 + px;
            if constexpr (V == 8) {
                uint4 q = *reinterpret_cast<const uint4 *>(g);
                v[0] = q.x & 0xFFFF; v[1] = q.x >> 16; v[2] = q.y & 0xFFFF; v[3] = q.y >> 16;
                v[4] = q.z & 0xFFFF; v[5] = q.z >> 16; v[6] = q.w & 0xFFFF; v[7] = q.w >> 16;
            } else if constexpr (V == 4) {
                uint2 q = *reinterpret_cast<const uint2 *>(g);
                v[0] = q.x & 0xFFFF; v[1] = q.x >> 16; v[2] = q.y & 0xFFFF; v[3] = q.y >> 16;
            } else if constexpr (V == 2) {
                uint32_t q = *reinterpret_cast<const uint32_t *>(g);
                v[0] = q & 0xFFFF; v[1] = q >> 16;
            } else {
                v[0] = *g;
            }
        }
#pragma unroll
        for (int e = 0; e < V; ++e) tile[ci * LT_PITCH + px + e] = v[e];
    }
    __syncthreads();

    // write phase: per pixel 16 channels = 32 B; each thread writes 16 B (8 channels)
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int a = tid + 256 * it;
        const int px = a >> 1;
        const int half = a & 1;
        if (px0 + px < HW) {
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t lo = tile[(half * 8 + 2 * e) * LT_PITCH + px];
                const uint32_t hi = tile[(half * 8 + 2 * e + 1) * LT_PITCH + px];
                w[e] = lo | (hi << 16);
            }
            uint16_t *g = dst + (((size_t)n * CB + cb) * HW + px0 + px) * 16 + half * 8;
            store16_result(g, make_uint4(w[0], w[1], w[2], w[3]), true);
        }
    }
}

// ---- blocked -> NCHW, 2-byte elements.  Same tiling, phases swapped.
template <int V>
__global__ __launch_bounds__(256) void blocked16_to_nchw_b16(const uint16_t *__restrict__ src,
                                                             uint16_t *__restrict__ dst, int C, int HW)
{
    __shared__ __align__(16) uint16_t tile[16 * LT_PITCH];
    const int tid = threadIdx.x;
    const int px0 = blockIdx.x * LT_PIX;
    const int cb = blockIdx.y;
    const int n = blockIdx.z;
    const int CB = gridDim.y;

#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int a = tid + 256 * it;
        const int px = a >> 1;
        const int half = a & 1;
        uint4 q = make_uint4(0, 0, 0, 0);
        if (px0 + px < HW)
            q = *reinterpret_cast<const uint4 *>(src + (((size_t)n * CB + cb) * HW + px0 + px) * 16 + half * 8);
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            tile[(half * 8 + 2 * e) * LT_PITCH + px] = (uint16_t)(w[e] & 0xFFFF);
            tile[(half * 8 + 2 * e + 1) * LT_PITCH + px] = (uint16_t)(w[e] >> 16);
        }
    }
    __syncthreads();

    constexpr int ACC_PER_ROW = LT_PIX / V;
    constexpr int ITERS = 16 * ACC_PER_ROW / 256;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int a = tid + 256 * it;
        const int ci = a / ACC_PER_ROW;
        const int px = (a % ACC_PER_ROW) * V;
        const int c = cb * 16 + ci;
        if (c < C && px0 + px < HW) {
            uint16_t v[V];
#pragma unroll
            for (int e = 0; e < V; ++e) v[e] = tile[ci * LT_PITCH + px + e];
            uint16_t *g = dst + ((size_t)n * C + c) * HW + px0 + px;
            if constexpr (V == 8) {
                *reinterpret_cast<uint4 *>(g) = make_uint4(v[0] | ((uint32_t)v[1] << 16), v[2] | ((uint32_t)v[3] << 16),
                                                           v[4] | ((uint32_t)v[5] << 16), v[6] | ((uint32_t)v[7] << 16));
            } else if constexpr (V == 4) {
                *reinterpret_cast<uint2 *>(g) = make_uint2(v[0] | ((uint32_t)v[1] << 16), v[2] | ((uint32_t)v[3] << 16));
            } else if constexpr (V == 2) {
                *reinterpret_cast<uint32_t *>(g) = v[0] | ((uint32_t)v[1] << 16);
            } else {
                *g = v[0];
            }
        }
    }
}

// ---- generic element-wise permutation (any element size, any direction): one thread per
// destination element.  Used for 4-byte elements and same-layout copies.
template <typename E>
__global__ __launch_bounds__(256) void layout_generic(const E *__restrict__ src, E *__restrict__ dst, int N, int C,
                                                      int H, int W, int src_layout, int dst_layout, size_t total)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    int n, c, h, w;
    size_t t = i;
    if (dst_layout == NGC_NCHW) {
        w = t % W; t /= W; h = t % H; t /= H; c = t % C; n = (int)(t / C);
    } else {
        const int CB = (C + 15) >> 4;
        const int ci = t % 16; t /= 16; w = t % W; t /= W; h = t % H; t /= H;
        const int cb = t % CB; n = (int)(t / CB);
        c = cb * 16 + ci;
    }
    E v = 0;
    if (c < C) v = src[data_index(src_layout, C, H, W, n, c, h, w)];
    dst[i] = v;
}

// ---- filter re-layout KCRS -> blocked (forward or backprop-data form); one thread per
// destination element, padded lanes written as +0.
template <typename E>
__global__ __launch_bounds__(256) void filter_to_blocked(const E *__restrict__ src, E *__restrict__ dst, int K, int C,
                                                         int R, int S, int dst_layout, size_t total)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    size_t t = i;
    const int lane = t % 16; t /= 16;
    int k, c;
    if (dst_layout == NGC_BLOCKED_FWD) {                // [r][s][cb][k][ci]
        const int CB = (C + 15) >> 4;
        k = t % K; t /= K;
        const int cb = t % CB; t /= CB;
        c = cb * 16 + lane;
    } else {                                            // [r][s][kb][c][ki]
        const int KB = (K + 15) >> 4;
        c = t % C; t /= C;
        const int kb = t % KB; t /= KB;
        k = kb * 16 + lane;
    }
    const int s = t % S;
    const int r = (int)(t / S);
    E v = 0;
    if (k < K && c < C) v = src[(((size_t)k * C + c) * R + r) * S + s];
    dst[i] = v;
}

// Combined filter of a stride-2 backprop-data written as a stride-1 convolution over 2x2 output
// blocks: wu[ut][k/16][col][k%16], col = (2a+b)*C + c (64 columns, the rest zero), union tap
// ut = (dr - dr_min)*nds + (ds - ds_min); entry = w[k][c][r][s] with r = a + pad_h - 2 dr,
// s = b + pad_w - 2 ds when that tap exists, else 0.
__global__ __launch_bounds__(256) void subpixel_filter(const uint16_t *__restrict__ w, uint16_t *__restrict__ wu, int K,
                                                       int C, int R, int S, int pbh, int pbw, int dr_min, int ds_min,
                                                       int nds, int BH, int BW, int sh, int sw, size_t total)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    size_t t = i;
    const int ki = t % 16; t /= 16;
    const int col = t % 64; t /= 64;
    const int KB = K >> 4;
    const int kb = t % KB; t /= KB;
    const int ut = (int)t;
    const int dr = dr_min + ut / nds, ds = ds_min + ut % nds;
    uint16_t v = 0;
    if (col < BH * BW * C) {
        const int ab = col / C, c = col - ab * C;
        const int a = ab / BW, b = ab - a * BW;
        const int r = a + pbh - sh * dr, s = b + pbw - sw * ds;
        if (r >= 0 && r < R && s >= 0 && s < S) v = w[(((size_t)(kb * 16 + ki) * C + c) * R + r) * S + s];
    }
    wu[i] = v;
}

hipError_t launch_subpixel_filter(int K, int C, int R, int S, int pbh, int pbw, int dr_min, int ndr, int ds_min, int nds,
                                  int BH, int BW, int sh, int sw, const uint16_t *w_kcrs, uint16_t *wu, hipStream_t st)
{
    const size_t total = (size_t)ndr * nds * K * 64;
    NGC_LAUNCH(subpixel_filter, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, w_kcrs, wu, K, C, R, S, pbh, pbw,
               dr_min, ds_min, nds, BH, BW, sh, sw, total);
    return ngc::launch_result();
}

static bool aligned_to(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

hipError_t launch_layout_convert(int elem_bytes, int n, int c, int h, int w, const void *src, int src_layout,
                                 void *dst, int dst_layout, hipStream_t st)
{
    const int HW = h * w;
    const int CB = (c + 15) / 16;
    const bool fast = elem_bytes == 2 && src_layout != dst_layout && CB <= 65535 && n <= 65535 &&
                      aligned_to(src, 16) && aligned_to(dst, 16);
    if (fast) {
        dim3 grid((HW + LT_PIX - 1) / LT_PIX, CB, n), block(256);
        const uint16_t *s = static_cast<const uint16_t *>(src);
        uint16_t *d = static_cast<uint16_t *>(dst);
        const int v = (HW % 8 == 0) ? 8 : (HW % 4 == 0) ? 4 : (HW % 2 == 0) ? 2 : 1;
        if (src_layout == NGC_NCHW) {
            if (v == 8) NGC_LAUNCH(nchw_to_blocked16_b16<8>, grid, block, 0, st, s, d, c, HW);
            else if (v == 4) NGC_LAUNCH(nchw_to_blocked16_b16<4>, grid, block, 0, st, s, d, c, HW);
            else if (v == 2) NGC_LAUNCH(nchw_to_blocked16_b16<2>, grid, block, 0, st, s, d, c, HW);
            else NGC_LAUNCH(nchw_to_blocked16_b16<1>, grid, block, 0, st, s, d, c, HW);
        } else {
            if (v == 8) NGC_LAUNCH(blocked16_to_nchw_b16<8>, grid, block, 0, st, s, d, c, HW);
            else if (v == 4) NGC_LAUNCH(blocked16_to_nchw_b16<4>, grid, block, 0, st, s, d, c, HW);
            else if (v == 2) NGC_LAUNCH(blocked16_to_nchw_b16<2>, grid, block, 0, st, s, d, c, HW);
            else NGC_LAUNCH(blocked16_to_nchw_b16<1>, grid, block, 0, st, s, d, c, HW);
        }
        return ngc::launch_result();
    }
    const size_t total = (dst_layout == NGC_NCHW) ? (size_t)n * c * HW : (size_t)n * CB * HW * 16;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (elem_bytes == 2)
        NGC_LAUNCH(layout_generic<uint16_t>, dim3(blocks), dim3(256), 0, st, static_cast<const uint16_t *>(src),
                           static_cast<uint16_t *>(dst), n, c, h, w, src_layout, dst_layout, total);
    else
        NGC_LAUNCH(layout_generic<uint32_t>, dim3(blocks), dim3(256), 0, st, static_cast<const uint32_t *>(src),
                           static_cast<uint32_t *>(dst), n, c, h, w, src_layout, dst_layout, total);
    return ngc::launch_result();
}

hipError_t launch_filter_convert(int elem_bytes, int K, int C, int R, int S, const void *w_kcrs, void *dst,
                                 int dst_layout, hipStream_t st)
{
    const size_t total = (dst_layout == NGC_BLOCKED_FWD) ? (size_t)R * S * ((C + 15) / 16) * K * 16
                                                         : (size_t)R * S * ((K + 15) / 16) * C * 16;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (elem_bytes == 2)
        NGC_LAUNCH(filter_to_blocked<uint16_t>, dim3(blocks), dim3(256), 0, st,
                           static_cast<const uint16_t *>(w_kcrs), static_cast<uint16_t *>(dst), K, C, R, S, dst_layout,
                           total);
    else
        NGC_LAUNCH(filter_to_blocked<uint32_t>, dim3(blocks), dim3(256), 0, st,
                           static_cast<const uint32_t *>(w_kcrs), static_cast<uint32_t *>(dst), K, C, R, S, dst_layout,
                           total);
    return ngc::launch_result();
}

}  // namespace ngc
