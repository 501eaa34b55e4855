// Direct (one thread per output element) kernels for Convolution over three spatial axes
// (N, C, D, H, W): every attribute combination, both element types, both data layouts, filters
// [K][C][T][R][S].  They serve fp32 and the shapes the MFMA kernels do not cover.  fp32
// accumulation in a fixed order; results are deterministic.
#include "common.h"

namespace ngc {

template <typename T> __device__ __forceinline__ float ld3(const T *p, size_t i);
template <> __device__ __forceinline__ float ld3<float>(const float *p, size_t i) { return p[i]; }
template <> __device__ __forceinline__ float ld3<uint16_t>(const uint16_t *p, size_t i) { return bf16_bits_to_float(p[i]); }

template <typename T> __device__ __forceinline__ void st3(T *p, size_t i, float v);
template <> __device__ __forceinline__ void st3<float>(float *p, size_t i, float v) { p[i] = v; }
template <> __device__ __forceinline__ void st3<uint16_t>(uint16_t *p, size_t i, float v) { p[i] = (uint16_t)float_to_bf16_bits(v); }

__device__ __forceinline__ size_t index3(int layout, int C, int D, int H, int W, int n, int c, int z, int h, int w)
{
    if (layout == NGC_NCHW) return ((((size_t)n * C + c) * D + z) * H + h) * W + w;
    const int CB = (C + 15) >> 4;
    return (((((size_t)n * CB + (c >> 4)) * D + z) * H + h) * W + w) * 16 + (c & 15);
}

// i-th physical element -> logical coordinates; for the blocked layout c may be >= C (a padding lane)
__device__ __forceinline__ void decode3(int layout, int C, int D, int H, int W, size_t i, int &n, int &c, int &z, int &h, int &w)
{
    size_t t = i;
    int ci = 0;
    if (layout != NGC_NCHW) { ci = t % 16; t /= 16; }
    w = t % W; t /= W; h = t % H; t /= H; z = t % D; t /= D;
    if (layout == NGC_NCHW) {
        c = t % C; n = (int)(t / C);
    } else {
        const int CB = (C + 15) >> 4;
        c = (int)(t % CB) * 16 + ci; n = (int)(t / CB);
    }
}

__device__ __forceinline__ size_t filter_index3(const ngc_conv3d_desc &d, int k, int c, int t, int r, int s)
{
    return ((((size_t)k * d.c + c) * d.t + t) * d.r + r) * d.s + s;
}

template <typename T>
__global__ __launch_bounds__(256) void direct3_fwd(ngc_conv3d_desc d, int O, int P, int Q, const T *__restrict__ x,
                                                   const T *__restrict__ w, const float *__restrict__ bias, T *__restrict__ y,
                                                   size_t total)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    int n, k, o, p, q;
    decode3(d.y_layout, d.k, O, P, Q, i, n, k, o, p, q);
    float z = 0.f;
    if (k < d.k) {
        float acc = 0.f;
        for (int c = 0; c < d.c; ++c)
            for (int t = 0; t < d.t; ++t) {
                const int iz = o * d.stride_d - d.pad_below_d + t * d.dil_d;
                if (iz < 0 || iz >= d.d) continue;
                for (int r = 0; r < d.r; ++r) {
                    const int ih = p * d.stride_h - d.pad_below_h + r * d.dil_h;
                    if (ih < 0 || ih >= d.h) continue;
                    for (int s = 0; s < d.s; ++s) {
                        const int iw = q * d.stride_w - d.pad_below_w + s * d.dil_w;
                        if (iw < 0 || iw >= d.w) continue;
                        acc = fmaf(ld3(x, index3(d.x_layout, d.c, d.d, d.h, d.w, n, c, iz, ih, iw)),
                                   ld3(w, filter_index3(d, k, c, t, r, s)), acc);
                    }
                }
            }
        z = acc;
        if (d.epilogue & NGC_EPI_BIAS) z += bias[k];
        if (d.epilogue & NGC_EPI_RELU) z = fmaxf(z, 0.f);
    }
    st3(y, i, z);
}

template <typename T>
__global__ __launch_bounds__(256) void direct3_bwd_data(ngc_conv3d_desc d, int O, int P, int Q, const T *__restrict__ dy,
                                                        const T *__restrict__ w, const T *__restrict__ mask, T *__restrict__ dx,
                                                        size_t total)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    int n, c, z, h, ww;
    decode3(d.x_layout, d.c, d.d, d.h, d.w, i, n, c, z, h, ww);
    float acc = 0.f;
    if (c < d.c) {
        for (int k = 0; k < d.k; ++k)
            for (int t = 0; t < d.t; ++t) {
                const int on = z + d.pad_below_d - t * d.dil_d;
                if (on < 0 || on % d.stride_d != 0 || on / d.stride_d >= O) continue;
                for (int r = 0; r < d.r; ++r) {
                    const int pn = h + d.pad_below_h - r * d.dil_h;
                    if (pn < 0 || pn % d.stride_h != 0 || pn / d.stride_h >= P) continue;
                    for (int s = 0; s < d.s; ++s) {
                        const int qn = ww + d.pad_below_w - s * d.dil_w;
                        if (qn < 0 || qn % d.stride_w != 0 || qn / d.stride_w >= Q) continue;
                        acc = fmaf(ld3(dy, index3(d.y_layout, d.k, O, P, Q, n, k, on / d.stride_d, pn / d.stride_h, qn / d.stride_w)),
                                   ld3(w, filter_index3(d, k, c, t, r, s)), acc);
                    }
                }
            }
    }
    if (mask && !(ld3(mask, i) > 0.f)) acc = 0.f;         // ReLU backprop: same shape / layout as dx
    st3(dx, i, acc);
}

// one workgroup per dw element; threads stride over (n,o,p,q); fixed-order tree reduction in LDS
template <typename T>
__global__ __launch_bounds__(256) void direct3_bwd_filters(ngc_conv3d_desc d, int O, int P, int Q, const T *__restrict__ x,
                                                           const T *__restrict__ dy, float *__restrict__ dw)
{
    __shared__ float red[256];
    size_t u = blockIdx.x;
    const int s = u % d.s; u /= d.s;
    const int r = u % d.r; u /= d.r;
    const int t = u % d.t; u /= d.t;
    const int c = u % d.c;
    const int k = (int)(u / d.c);
    const unsigned total = (unsigned)d.n * O * P * Q;
    float acc = 0.f;
    for (unsigned m = threadIdx.x; m < total; m += 256) {
        unsigned v = m;
        const int q = v % Q; v /= Q;
        const int p = v % P; v /= P;
        const int o = v % O;
        const int n = v / O;
        const int iz = o * d.stride_d - d.pad_below_d + t * d.dil_d;
        const int ih = p * d.stride_h - d.pad_below_h + r * d.dil_h;
        const int iw = q * d.stride_w - d.pad_below_w + s * d.dil_w;
        if (iz < 0 || iz >= d.d || ih < 0 || ih >= d.h || iw < 0 || iw >= d.w) continue;
        acc = fmaf(ld3(dy, index3(d.y_layout, d.k, O, P, Q, n, k, o, p, q)),
                   ld3(x, index3(d.x_layout, d.c, d.d, d.h, d.w, n, c, iz, ih, iw)), acc);
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) dw[blockIdx.x] = red[0];
}

static size_t phys3(int layout, int n, int c, int d, int h, int w)
{
    return (size_t)n * (layout == NGC_NCHW ? c : (c + 15) / 16 * 16) * d * h * w;
}

hipError_t launch_direct3_fwd(const ngc_conv3d_desc &d, int O, int P, int Q, const void *x, const void *w, const float *bias,
                              void *y, hipStream_t stm)
{
    const size_t total = phys3(d.y_layout, d.n, d.k, O, P, Q);
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (d.dtype == NGC_F32)
        NGC_LAUNCH(direct3_fwd<float>, dim3(blocks), dim3(256), 0, stm, d, O, P, Q, static_cast<const float *>(x),
                   static_cast<const float *>(w), bias, static_cast<float *>(y), total);
    else
        NGC_LAUNCH(direct3_fwd<uint16_t>, dim3(blocks), dim3(256), 0, stm, d, O, P, Q, static_cast<const uint16_t *>(x),
                   static_cast<const uint16_t *>(w), bias, static_cast<uint16_t *>(y), total);
    return ngc::launch_result();
}

hipError_t launch_direct3_bwd_data(const ngc_conv3d_desc &d, int O, int P, int Q, const void *dy, const void *w, const void *mask,
                                   void *dx, hipStream_t stm)
{
    const size_t total = phys3(d.x_layout, d.n, d.c, d.d, d.h, d.w);
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (d.dtype == NGC_F32)
        NGC_LAUNCH(direct3_bwd_data<float>, dim3(blocks), dim3(256), 0, stm, d, O, P, Q, static_cast<const float *>(dy),
                   static_cast<const float *>(w), static_cast<const float *>(mask), static_cast<float *>(dx), total);
    else
        NGC_LAUNCH(direct3_bwd_data<uint16_t>, dim3(blocks), dim3(256), 0, stm, d, O, P, Q, static_cast<const uint16_t *>(dy),
                   static_cast<const uint16_t *>(w), static_cast<const uint16_t *>(mask), static_cast<uint16_t *>(dx), total);
    return ngc::launch_result();
}

hipError_t launch_direct3_bwd_filters(const ngc_conv3d_desc &d, int O, int P, int Q, const void *x, const void *dy, float *dw,
                                      hipStream_t stm)
{
    const unsigned blocks = (unsigned)((size_t)d.k * d.c * d.t * d.r * d.s);
    if (d.dtype == NGC_F32)
        NGC_LAUNCH(direct3_bwd_filters<float>, dim3(blocks), dim3(256), 0, stm, d, O, P, Q, static_cast<const float *>(x),
                   static_cast<const float *>(dy), dw);
    else
        NGC_LAUNCH(direct3_bwd_filters<uint16_t>, dim3(blocks), dim3(256), 0, stm, d, O, P, Q, static_cast<const uint16_t *>(x),
                   static_cast<const uint16_t *>(dy), dw);
    return ngc::launch_result();
}

}  // namespace ngc
