// Direct (one thread per output element) kernels for the Convolution op family.
// They accept every attribute combination the ops define (any stride, padding below /
// above, dilation), both element types and both data layouts, with filters in KCRS.
// They serve the fp32 configuration and every shape the MFMA kernels do not cover.
// fp32 accumulation in a fixed order; results are deterministic.
#include "common.h"

namespace ngc {

template <typename T> __device__ __forceinline__ float ld(const T *p, size_t i);
template <> __device__ __forceinline__ float ld<float>(const float *p, size_t i) { return p[i]; }
template <> __device__ __forceinline__ float ld<uint16_t>(const uint16_t *p, size_t i) { return bf16_bits_to_float(p[i]); }

template <typename T> __device__ __forceinline__ void st(T *p, size_t i, float v);
template <> __device__ __forceinline__ void st<float>(float *p, size_t i, float v) { p[i] = v; }
template <> __device__ __forceinline__ void st<uint16_t>(uint16_t *p, size_t i, float v) { p[i] = (uint16_t)float_to_bf16_bits(v); }

// Decode the i-th *physical* element of an [N,C,H,W] tensor stored in `layout` into logical
// coordinates.  For the blocked layout c may be >= C (a padding lane).
__device__ __forceinline__ void decode(int layout, int C, int H, int W, size_t i, int &n, int &c, int &h, int &w)
{
    size_t t = i;
    if (layout == NGC_NCHW) {
        w = t % W; t /= W; h = t % H; t /= H; c = t % C; n = (int)(t / C);
    } else {
        const int CB = (C + 15) >> 4;
        const int ci = t % 16; t /= 16; w = t % W; t /= W; h = t % H; t /= H;
        const int cb = t % CB; n = (int)(t / CB);
        c = cb * 16 + ci;
    }
}

template <typename T>
__global__ __launch_bounds__(256) void direct_fwd(ngc_conv_desc d, int P, int Q, const T *__restrict__ x,
                                                  const T *__restrict__ w, const float *__restrict__ bias,
                                                  T *__restrict__ y, size_t total)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    int n, k, p, q;
    decode(d.y_layout, d.k, P, Q, i, n, k, p, q);
    float z = 0.f;
    if (k < d.k) {
        float acc = 0.f;
        for (int c = 0; c < d.c; ++c)
            for (int r = 0; r < d.r; ++r) {
                const int ih = p * d.stride_h - d.pad_below_h + r * d.dil_h;
                if (ih < 0 || ih >= d.h) continue;
                for (int s = 0; s < d.s; ++s) {
                    const int iw = q * d.stride_w - d.pad_below_w + s * d.dil_w;
                    if (iw < 0 || iw >= d.w) continue;
                    acc = fmaf(ld(x, data_index(d.x_layout, d.c, d.h, d.w, n, c, ih, iw)),
                               ld(w, (((size_t)k * d.c + c) * d.r + r) * d.s + s), acc);
                }
            }
        z = acc;
        if (d.epilogue & NGC_EPI_BIAS) z += bias[k];
        if (d.epilogue & NGC_EPI_RELU) z = fmaxf(z, 0.f);
    }
    st(y, i, z);
}

template <typename T>
__global__ __launch_bounds__(256) void direct_bwd_data(ngc_conv_desc d, int P, int Q, const T *__restrict__ dy,
                                                       const T *__restrict__ w, const T *__restrict__ mask,
                                                       T *__restrict__ dx, size_t total)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    int n, c, h, ww;
    decode(d.x_layout, d.c, d.h, d.w, i, n, c, h, ww);
    float acc = 0.f;
    if (c < d.c) {
        // taps outermost: which output position a tap reaches (two integer divisions) is decided once per tap, not
        // once per tap and output channel
        for (int r = 0; r < d.r; ++r) {
            const int pn = h + d.pad_below_h - r * d.dil_h;
            if (pn < 0 || pn % d.stride_h != 0) continue;
            const int p = pn / d.stride_h;
            if (p >= P) continue;
            for (int s = 0; s < d.s; ++s) {
                const int qn = ww + d.pad_below_w - s * d.dil_w;
                if (qn < 0 || qn % d.stride_w != 0) continue;
                const int q = qn / d.stride_w;
                if (q >= Q) continue;
                const size_t wrs = ((size_t)c * d.r + r) * d.s + s, wk = (size_t)d.c * d.r * d.s;
                for (int k = 0; k < d.k; ++k)
                    acc = fmaf(ld(dy, data_index(d.y_layout, d.k, P, Q, n, k, p, q)), ld(w, k * wk + wrs), acc);
            }
        }
    }
    if (mask && !(ld(mask, i) > 0.f)) acc = 0.f;          // ReLU backprop: same shape / layout as dx
    st(dx, i, acc);
}

// one workgroup per dw element; threads stride over (n,p,q); fixed-order tree reduction in LDS
template <typename T>
__global__ __launch_bounds__(256) void direct_bwd_filters(ngc_conv_desc d, int P, int Q, const T *__restrict__ x,
                                                          const T *__restrict__ dy, float *__restrict__ dw)
{
    __shared__ float red[256];
    size_t t = blockIdx.x;
    const int s = t % d.s; t /= d.s;
    const int r = t % d.r; t /= d.r;
    const int c = t % d.c;
    const int k = (int)(t / d.c);
    const unsigned total = (unsigned)d.n * P * Q;
    float acc = 0.f;
    for (unsigned m = threadIdx.x; m < total; m += 256) {
        const int q = m % Q;
        const unsigned u = m / Q;
        const int p = u % P;
        const int n = u / P;
        const int ih = p * d.stride_h - d.pad_below_h + r * d.dil_h;
        const int iw = q * d.stride_w - d.pad_below_w + s * d.dil_w;
        if (ih < 0 || ih >= d.h || iw < 0 || iw >= d.w) continue;
        acc = fmaf(ld(dy, data_index(d.y_layout, d.k, P, Q, n, k, p, q)),
                   ld(x, data_index(d.x_layout, d.c, d.h, d.w, n, c, ih, iw)), acc);
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) dw[blockIdx.x] = red[0];
}

static size_t phys_elems(int layout, int n, int c, int h, int w)
{
    return layout == NGC_NCHW ? (size_t)n * c * h * w : (size_t)n * ((c + 15) / 16) * h * w * 16;
}

hipError_t launch_direct_fwd(const ngc_conv_desc &d, int P, int Q, const void *x, const void *w, const float *bias,
                             void *y, hipStream_t stm)
{
    const size_t total = phys_elems(d.y_layout, d.n, d.k, P, Q);
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (d.dtype == NGC_F32)
        NGC_LAUNCH(direct_fwd<float>, dim3(blocks), dim3(256), 0, stm, d, P, Q, static_cast<const float *>(x),
                           static_cast<const float *>(w), bias, static_cast<float *>(y), total);
    else
        NGC_LAUNCH(direct_fwd<uint16_t>, dim3(blocks), dim3(256), 0, stm, d, P, Q,
                           static_cast<const uint16_t *>(x), static_cast<const uint16_t *>(w), bias,
                           static_cast<uint16_t *>(y), total);
    return ngc::launch_result();
}

hipError_t launch_direct_bwd_data(const ngc_conv_desc &d, int P, int Q, const void *dy, const void *w, const void *mask,
                                  void *dx, hipStream_t stm)
{
    const size_t total = phys_elems(d.x_layout, d.n, d.c, d.h, d.w);
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (d.dtype == NGC_F32)
        NGC_LAUNCH(direct_bwd_data<float>, dim3(blocks), dim3(256), 0, stm, d, P, Q,
                           static_cast<const float *>(dy), static_cast<const float *>(w),
                           static_cast<const float *>(mask), static_cast<float *>(dx), total);
    else
        NGC_LAUNCH(direct_bwd_data<uint16_t>, dim3(blocks), dim3(256), 0, stm, d, P, Q,
                           static_cast<const uint16_t *>(dy), static_cast<const uint16_t *>(w),
                           static_cast<const uint16_t *>(mask), static_cast<uint16_t *>(dx), total);
    return ngc::launch_result();
}

hipError_t launch_direct_bwd_filters(const ngc_conv_desc &d, int P, int Q, const void *x, const void *dy, float *dw,
                                     hipStream_t stm)
{
    const unsigned blocks = (unsigned)((size_t)d.k * d.c * d.r * d.s);
    if (d.dtype == NGC_F32)
        NGC_LAUNCH(direct_bwd_filters<float>, dim3(blocks), dim3(256), 0, stm, d, P, Q,
                           static_cast<const float *>(x), static_cast<const float *>(dy), dw);
    else
        NGC_LAUNCH(direct_bwd_filters<uint16_t>, dim3(blocks), dim3(256), 0, stm, d, P, Q,
                           static_cast<const uint16_t *>(x), static_cast<const uint16_t *>(dy), dw);
    return ngc::launch_result();
}

}  // namespace ngc
