// Bias gradient of the compounded bias + ReLU forward op: db[k] = sum_{n,p,q} dy[n,k,p,q] in fp32
// (the adjoint of broadcasting the bias over n, p, q; derivative graphs come from autodiff of the
// forward ops, Sec. 3 of the paper).  Bound: HBM (one pass over dy).
//
// Two stages, no atomics: workgroup (part, channel block) sums its chunk of the N*P*Q positions
// with a fixed assignment of positions to threads and a fixed LDS tree, and writes a partial;
// the second kernel adds the parts with a fixed assignment as well.  Results do not depend on timing.
#include "common.h"

namespace ngc {

// bf16, 16-channel-blocked dy: thread t = (position slot t/2, 8-channel half t%2), 16-byte loads
__global__ __launch_bounds__(256) void bias_grad_blocked_bf16(const uint16_t *__restrict__ dy, float *__restrict__ partial,
                                                              int KB, int PQ, uint32_t M, uint32_t chunk, FastDiv div_pq)
{
    __shared__ float sm[256][9];                        // 9: pad against bank conflicts of the 8-float rows
    const int tid = threadIdx.x;
    const int half = tid & 1, slot = tid >> 1;
    const int kb = blockIdx.y;
    const uint32_t m_begin = blockIdx.x * chunk;
    const uint32_t m_end = (m_begin + chunk < M) ? m_begin + chunk : M;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (uint32_t m = m_begin + (uint32_t)slot; m < m_end; m += 128) {
        const uint32_t n = fd_div(m, div_pq);
        const uint32_t pos = m - n * div_pq.d;
        const uint4 v = *reinterpret_cast<const uint4 *>(dy + (((size_t)n * KB + kb) * PQ + pos) * 16 + half * 8);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc[2 * j] += __uint_as_float(w[j] << 16);
            acc[2 * j + 1] += __uint_as_float(w[j] & 0xFFFF0000u);
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) sm[tid][j] = acc[j];
    __syncthreads();
    for (int stride = 64; stride >= 1; stride >>= 1) {  // tree over the 128 position slots (rows tid = 2*slot + half)
        if (slot < stride) {
#pragma unroll
            for (int j = 0; j < 8; ++j) sm[tid][j] += sm[tid + 2 * stride][j];
        }
        __syncthreads();
    }
    if (tid < 16) partial[((size_t)blockIdx.x * KB + kb) * 16 + tid] = sm[tid >> 3][tid & 7];
}

// any element type / layout: one workgroup per (part, channel)
template <typename T>
__global__ __launch_bounds__(256) void bias_grad_generic(const T *__restrict__ dy, float *__restrict__ partial, int layout,
                                                         int K, int KP, int P, int Q, uint32_t M, uint32_t chunk, FastDiv div_pq,
                                                         FastDiv div_q)
{
    __shared__ float sm[256];
    const int tid = threadIdx.x;
    const int k = blockIdx.y;
    const uint32_t m_begin = blockIdx.x * chunk;
    const uint32_t m_end = (m_begin + chunk < M) ? m_begin + chunk : M;
    float acc = 0.f;
    for (uint32_t m = m_begin + (uint32_t)tid; m < m_end; m += 256) {
        const uint32_t n = fd_div(m, div_pq);
        const uint32_t pos = m - n * div_pq.d;
        const uint32_t p = fd_div(pos, div_q);
        const uint32_t q = pos - p * div_q.d;
        const size_t idx = data_index(layout, K, P, Q, (int)n, k, (int)p, (int)q);
        if (sizeof(T) == 4) acc += reinterpret_cast<const float *>(dy)[idx];
        else acc += bf16_bits_to_float(reinterpret_cast<const uint16_t *>(dy)[idx]);
    }
    sm[tid] = acc;
    __syncthreads();
    for (int stride = 128; stride >= 1; stride >>= 1) {
        if (tid < stride) sm[tid] += sm[tid + stride];
        __syncthreads();
    }
    if (tid == 0) partial[(size_t)blockIdx.x * KP + k] = sm[0];
}

// db[k] = sum over parts; KP = channels per part row of `partial` (a multiple of 16, rows 64-byte aligned).
// One workgroup per 16 channels: thread (lane = tid / 4, quad = tid % 4) adds the float4 of channels
// 4 quad .. 4 quad + 3 of parts lane, lane + 64, ... in index order (independent 16-byte loads, so they
// pipeline), then a fixed LDS tree joins the 64 lanes.
__global__ __launch_bounds__(256) void bias_grad_reduce(const float *__restrict__ partial, float *__restrict__ db, int nparts,
                                                        int K, int KP)
{
    __shared__ float4 sm[256];
    const int tid = threadIdx.x;
    const int c0 = blockIdx.x * 16 + (tid & 3) * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 8
    for (int s = tid >> 2; s < nparts; s += 64) {
        const float4 v = *reinterpret_cast<const float4 *>(partial + (size_t)s * KP + c0);
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    sm[tid] = acc;
    __syncthreads();
    for (int stride = 128; stride >= 4; stride >>= 1) {
        if (tid < stride) {
            const float4 o = sm[tid + stride];
            float4 m = sm[tid];
            m.x += o.x; m.y += o.y; m.z += o.z; m.w += o.w;
            sm[tid] = m;
        }
        __syncthreads();
    }
    if (tid < 4) {
        const float4 r = sm[tid];
        const float out[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (c0 + e < K) db[c0 + e] = out[e];
    }
}

// position chunks: enough workgroups to fill the chip, at most 256 chunks of at least 128 positions
int bias_grad_parts(const ngc_conv_desc &d, int P, int Q)
{
    const uint32_t M = (uint32_t)d.n * P * Q;
    const bool blocked = d.dtype == NGC_BF16 && d.y_layout == NGC_NCHW16C;
    const uint32_t rows = blocked ? (uint32_t)(d.k + 15) / 16 : (uint32_t)d.k;
    uint32_t parts = (2048 + rows - 1) / rows;
    if (parts > 256) parts = 256;                       // keeps the second stage short
    const uint32_t max_parts = (M + 127) / 128;
    if (parts > max_parts) parts = max_parts;
    if (parts < 1) parts = 1;
    return (int)parts;
}

// db[k] = sum of nparts rows of `partial` (row pitch KP floats)
hipError_t launch_bias_grad_reduce(const float *partial, float *db, int nparts, int K, int KP, hipStream_t st)
{
    NGC_LAUNCH(bias_grad_reduce, dim3((K + 15) / 16), dim3(256), 0, st, partial, db, nparts, K, KP);
    return ngc::launch_result();
}

hipError_t launch_bias_grad(const ngc_conv_desc &d, int P, int Q, const void *dy, float *db, float *partial, int nparts,
                            hipStream_t st)
{
    const uint32_t M = (uint32_t)d.n * P * Q;
    const uint32_t chunk = (M + nparts - 1) / nparts;
    const FastDiv div_pq = make_fastdiv((uint32_t)(P * Q)), div_q = make_fastdiv((uint32_t)Q);
    const bool blocked = d.dtype == NGC_BF16 && d.y_layout == NGC_NCHW16C;
    const int KB = (d.k + 15) / 16;
    const int KP = KB * 16;                             // row pitch of the partials: K rounded up to 16
    if (blocked)
        NGC_LAUNCH(bias_grad_blocked_bf16, dim3(nparts, KB), dim3(256), 0, st, static_cast<const uint16_t *>(dy), partial, KB,
                   P * Q, M, chunk, div_pq);
    else if (d.dtype == NGC_F32)
        NGC_LAUNCH(bias_grad_generic<float>, dim3(nparts, d.k), dim3(256), 0, st, static_cast<const float *>(dy), partial,
                   d.y_layout, d.k, KP, P, Q, M, chunk, div_pq, div_q);
    else
        NGC_LAUNCH(bias_grad_generic<uint16_t>, dim3(nparts, d.k), dim3(256), 0, st, static_cast<const uint16_t *>(dy),
                   partial, d.y_layout, d.k, KP, P, Q, M, chunk, div_pq, div_q);
    hipError_t e = ngc::launch_result();
    if (e != hipSuccess) return e;
    NGC_LAUNCH(bias_grad_reduce, dim3((d.k + 15) / 16), dim3(256), 0, st, partial, db, nparts, d.k, KP);
    return ngc::launch_result();
}

}  // namespace ngc
