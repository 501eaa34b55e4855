// Softmax over the last axis of a [rows, cols] tensor and its backprop (gfx950).  The paper names
// softmax next to convolution as a kernel a backend supplies (Sec. 4); backward graphs come from
// autodiff of the forward ops (Sec. 3).
//
//   y[i][j]  = exp(x[i][j] - m_i) / sum_k exp(x[i][k] - m_i),  m_i = max_k x[i][k]
//   dx[i][j] = y[i][j] * (dy[i][j] - sum_k dy[i][k] y[i][k])
//
// Bound: HBM (each tensor once).  The row lives in registers: a thread keeps V 16-byte vectors of
// it (all loads of the row are in flight at once), the row maximum and sum are butterfly
// reductions over the 64 lanes of a wave (rows of up to 4 vectors per lane) or, for longer rows,
// over the 256 threads of a workgroup through LDS; results leave as 16-byte stores - one read and
// one write of the row, fp32 arithmetic, one rounding.  Rows too long for the registers (or not
// 16-byte aligned) take a workgroup-per-row kernel that walks the row three (backprop: two) times
// element by element.
#include "common.h"

#include <math.h>

namespace ngc {

template <typename T> struct SmElem;
template <> struct SmElem<uint16_t> {                  // bf16 bit patterns, 8 per 16 bytes
    static constexpr int E = 8;
    __device__ static void unpack(const uint4 &v, float (&f)[8])
    {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            f[2 * j] = __uint_as_float(w[j] << 16);
            f[2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
        }
    }
    __device__ static uint4 pack(const float (&f)[8])
    {
        return make_uint4(pack_bf16x2_hw(f[0], f[1]), pack_bf16x2_hw(f[2], f[3]), pack_bf16x2_hw(f[4], f[5]),
                          pack_bf16x2_hw(f[6], f[7]));
    }
    __device__ static float load(const uint16_t *p) { return bf16_bits_to_float(*p); }
    __device__ static void store(uint16_t *p, float v) { *p = (uint16_t)(pack_bf16x2_hw(v, 0.f) & 0xFFFFu); }
    // bf16 results carry 8 bits: the hardware exp2 (1 ulp of fp32) is far inside the rounding
    __device__ static float exp_of(float d) { return __builtin_amdgcn_exp2f(d * 1.44269504088896341f); }
};
template <> struct SmElem<float> {
    static constexpr int E = 4;
    __device__ static void unpack(const uint4 &v, float (&f)[4])
    {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
    __device__ static uint4 pack(const float (&f)[4])
    {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    }
    __device__ static float load(const float *p) { return *p; }
    __device__ static void store(float *p, float v) { *p = v; }
    __device__ static float exp_of(float d) { return expf(d); }
};

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);       // butterfly: every lane ends with the same sum
    return v;
}

// reduction over the NW waves of a workgroup (fixed order); sm holds NW floats
template <int NW>
__device__ __forceinline__ float block_reduce(float v, bool is_max, float *sm)
{
    v = is_max ? wave_max(v) : wave_sum(v);
    const int wave = threadIdx.x >> 6;
    __syncthreads();                                                     // sm may still be read from the last call
    if ((threadIdx.x & 63) == 0) sm[wave] = v;
    __syncthreads();
    float r = sm[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) r = is_max ? fmaxf(r, sm[w]) : r + sm[w];
    return r;
}

// The row in registers: V vectors of 16 bytes per thread, NT = 64 threads (one wave per row, 4 rows per
// workgroup) or 256 / 1024 (one workgroup per row, reductions through LDS): cols <= NT * E * V,
// cols % E == 0, 16-byte aligned tensors.  BWD: a = y, b = dy, out = dx; else a = x, out = y (b unused).
template <typename T, int V, bool BWD, int NT>
__global__ __launch_bounds__(NT == 64 ? 256 : NT) void softmax_rows_reg(const T *__restrict__ a, const T *__restrict__ b, T *__restrict__ out,
                                                        uint32_t rows, int cols)
{
    constexpr int E = SmElem<T>::E;
    constexpr int NW = NT == 64 ? 1 : NT / 64;
    __shared__ float sm[NW];
    const int lane = threadIdx.x & (NT - 1);
    const uint32_t row = NT == 64 ? blockIdx.x * 4 + (threadIdx.x >> 6) : blockIdx.x;
    if (row >= rows) return;                                             // wave-uniform (NT == 64 only)
    const size_t base = (size_t)row * cols;
    const int nvec = cols / E;
    float va[V][E], vb[BWD ? V : 1][E];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        const int vi = j * NT + lane;
        if (vi < nvec) {
            SmElem<T>::unpack(*reinterpret_cast<const uint4 *>(a + base + (size_t)vi * E), va[j]);
            if (BWD) SmElem<T>::unpack(*reinterpret_cast<const uint4 *>(b + base + (size_t)vi * E), vb[BWD ? j : 0]);
        } else {
#pragma unroll
            for (int e = 0; e < E; ++e) {
                va[j][e] = BWD ? 0.f : -INFINITY;                         // exp(-inf - m) = 0; 0 * dy = 0
                if (BWD) vb[BWD ? j : 0][e] = 0.f;
            }
        }
    }
    if (BWD) {
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < V; ++j)
#pragma unroll
            for (int e = 0; e < E; ++e) s += va[j][e] * vb[BWD ? j : 0][e];
        s = NT == 64 ? wave_sum(s) : block_reduce<NW>(s, false, sm);
#pragma unroll
        for (int j = 0; j < V; ++j)
#pragma unroll
            for (int e = 0; e < E; ++e) va[j][e] = va[j][e] * (vb[BWD ? j : 0][e] - s);
    } else {
        float m = -INFINITY;
#pragma unroll
        for (int j = 0; j < V; ++j)
#pragma unroll
            for (int e = 0; e < E; ++e) m = fmaxf(m, va[j][e]);
        m = NT == 64 ? wave_max(m) : block_reduce<NW>(m, true, sm);
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < V; ++j)
#pragma unroll
            for (int e = 0; e < E; ++e) {
                va[j][e] = SmElem<T>::exp_of(va[j][e] - m);
                s += va[j][e];
            }
        s = NT == 64 ? wave_sum(s) : block_reduce<NW>(s, false, sm);
        const float inv = 1.0f / s;
#pragma unroll
        for (int j = 0; j < V; ++j)
#pragma unroll
            for (int e = 0; e < E; ++e) va[j][e] *= inv;
    }
#pragma unroll
    for (int j = 0; j < V; ++j) {
        const int vi = j * NT + lane;
        if (vi < nvec) store16_result(out + base + (size_t)vi * E, SmElem<T>::pack(va[j]), true);
    }
}

// Any cols / alignment: one workgroup per row, element-wise passes (the row comes from L2 after the first).
template <typename T, bool BWD>
__global__ __launch_bounds__(256) void softmax_rows_block(const T *__restrict__ a, const T *__restrict__ b, T *__restrict__ out,
                                                          uint32_t rows, int cols)
{
    __shared__ float sm[4];
    const size_t base = (size_t)blockIdx.x * cols;
    const int tid = threadIdx.x;
    if (BWD) {
        float s = 0.f;
        for (int j = tid; j < cols; j += 256) s += SmElem<T>::load(a + base + j) * SmElem<T>::load(b + base + j);
        s = block_reduce<4>(s, false, sm);
        for (int j = tid; j < cols; j += 256)
            SmElem<T>::store(out + base + j, SmElem<T>::load(a + base + j) * (SmElem<T>::load(b + base + j) - s));
        return;
    }
    float m = -INFINITY;
    for (int j = tid; j < cols; j += 256) m = fmaxf(m, SmElem<T>::load(a + base + j));
    m = block_reduce<4>(m, true, sm);
    float s = 0.f;
    for (int j = tid; j < cols; j += 256) s += SmElem<T>::exp_of(SmElem<T>::load(a + base + j) - m);
    s = block_reduce<4>(s, false, sm);
    const float inv = 1.0f / s;
    for (int j = tid; j < cols; j += 256) SmElem<T>::store(out + base + j, SmElem<T>::exp_of(SmElem<T>::load(a + base + j) - m) * inv);
}

// Kernel choice for a row length: V = vectors per thread of the register-resident kernels (one wave per row,
// or 256 + V / 1024 + V: one workgroup of that many threads per row), 0 = the element-wise kernel.
int softmax_vectors(int dtype, int cols, bool bwd, bool aligned)
{
    const int E = dtype == NGC_BF16 ? 8 : 4;
    if (!aligned || cols % E != 0) return 0;
    const int nvec = cols / E;
    (void)bwd;
    for (int v = 1; v <= 4; v *= 2)
        if (nvec <= 64 * v) return v;                  // up to 4 vectors per lane: a wave per row
    for (int v = 2; v <= 4; v *= 2)
        if (nvec <= 256 * v) return 256 + v;           // longer rows: 256 threads per row,
    for (int v = 2; v <= 4; v *= 2)
        if (nvec <= 1024 * v) return 1024 + v;         // then 1024 (more loads in flight than more vectors per thread)
    return 0;
}

template <typename T, bool BWD>
static hipError_t launch_softmax_t(const T *a, const T *b, T *out, uint32_t rows, int cols, int V, hipStream_t st)
{
    const dim3 grid_w((rows + 3) / 4), grid_r(rows), block(256);
    switch (V) {
    case 1: NGC_LAUNCH((softmax_rows_reg<T, 1, BWD, 64>), grid_w, block, 0, st, a, b, out, rows, cols); break;
    case 2: NGC_LAUNCH((softmax_rows_reg<T, 2, BWD, 64>), grid_w, block, 0, st, a, b, out, rows, cols); break;
    case 4: NGC_LAUNCH((softmax_rows_reg<T, 4, BWD, 64>), grid_w, block, 0, st, a, b, out, rows, cols); break;
    case 256 + 2: NGC_LAUNCH((softmax_rows_reg<T, 2, BWD, 256>), grid_r, block, 0, st, a, b, out, rows, cols); break;
    case 256 + 4: NGC_LAUNCH((softmax_rows_reg<T, 4, BWD, 256>), grid_r, block, 0, st, a, b, out, rows, cols); break;
    case 1024 + 2: NGC_LAUNCH((softmax_rows_reg<T, 2, BWD, 1024>), grid_r, dim3(1024), 0, st, a, b, out, rows, cols); break;
    case 1024 + 4: NGC_LAUNCH((softmax_rows_reg<T, 4, BWD, 1024>), grid_r, dim3(1024), 0, st, a, b, out, rows, cols); break;
    case 0: NGC_LAUNCH((softmax_rows_block<T, BWD>), grid_r, block, 0, st, a, b, out, rows, cols); break;
    default: return hipErrorInvalidValue;
    }
    return ngc::launch_result();
}

hipError_t launch_softmax(int dtype, bool bwd, const void *a, const void *b, void *out, uint32_t rows, int cols, int V, hipStream_t st)
{
    if (dtype == NGC_BF16) {
        const uint16_t *pa = static_cast<const uint16_t *>(a), *pb = static_cast<const uint16_t *>(b);
        return bwd ? launch_softmax_t<uint16_t, true>(pa, pb, static_cast<uint16_t *>(out), rows, cols, V, st)
                   : launch_softmax_t<uint16_t, false>(pa, pb, static_cast<uint16_t *>(out), rows, cols, V, st);
    }
    const float *pa = static_cast<const float *>(a), *pb = static_cast<const float *>(b);
    return bwd ? launch_softmax_t<float, true>(pa, pb, static_cast<float *>(out), rows, cols, V, st)
               : launch_softmax_t<float, false>(pa, pb, static_cast<float *>(out), rows, cols, V, st);
}

}  // namespace ngc
