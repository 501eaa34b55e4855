// ConvolutionBackpropFilters on bf16 MFMA (gfx950), fp32 accumulate, deterministic two-stage
// reduction.
//
//   dw[k,c,r,s] = sum_{m=(n,p,q)} dy[m][k] * X[m @ tap(r,s)][c]
//
// GEMM view per tap: rows = k (output channels), columns = c (input channels), reduction over
// the N*P*Q output positions.  Both operands live in the 16-channel-blocked layout, i.e. with
// the *channel* axis contiguous, while an MFMA lane needs 8 consecutive *reduction* elements
// (positions) of one channel.  The transposition is done on the way into LDS: a thread loads
// the same 8 channels of two adjacent positions (2 x 16 bytes), interleaves them into 8 dwords
// (m, m+1) per channel, and stores those as ds_write_b32 into a [channel][position] tile whose
// rows are then read back as aligned 16-byte MFMA operands.
//
// Workgroup = 256 threads = 4 waves; grid = (splits, K/64 * C/64, taps).  A workgroup owns one
// 64(k) x 64(c) tile of one tap over one contiguous chunk of positions.  A step stages 64
// positions; wave w reduces positions 16w..16w+15 of the step into its own copy of the full
// 64x64 tile (2x2 MFMA 32x32x16 accumulators) - a wave-level split of the reduction - and the
// four copies are summed through LDS in a fixed order at the end.  The per-workgroup partial
// goes to the workspace [split][tap][k][c]; a second kernel adds the splits in index order
// and writes dw in [K][C][R][S].  No atomics: results are bit-identical run to run.
#include "common.h"

namespace ngc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int WG_PITCH = 144;                  // bytes per channel row: 64 positions * 2 B + 16 pad
constexpr int WG_TILE = 64 * WG_PITCH;         // one operand tile
constexpr int WG_STAGE = 2 * WG_TILE;          // dy tile + x tile

__device__ __forceinline__ void interleave_store(unsigned char *tile, int half, int pair, const uint4 &a, const uint4 &b)
{
    // a = 8 channels of position 2*pair, b = same channels of position 2*pair+1
    const uint32_t av[4] = {a.x, a.y, a.z, a.w};
    const uint32_t bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const uint32_t even = (av[e] & 0xFFFFu) | (bv[e] << 16);          // channel 2e
        const uint32_t odd = (av[e] >> 16) | (bv[e] & 0xFFFF0000u);       // channel 2e+1
        *reinterpret_cast<uint32_t *>(tile + (half * 8 + 2 * e) * WG_PITCH + pair * 4) = even;
        *reinterpret_cast<uint32_t *>(tile + (half * 8 + 2 * e + 1) * WG_PITCH + pair * 4) = odd;
    }
}

__global__ __launch_bounds__(256) void wgrad_bf16(const WgradParams p)
{
    preload_kernargs(p);
    __shared__ __align__(16) unsigned char smem[2 * WG_STAGE];       // 36864 B; reused for the final reduction

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l32 = lane & 31;
    const int lg = lane >> 5;

    const int split = blockIdx.x;
    const int ctiles = p.C >> 6;
    const int kt = blockIdx.y / ctiles;
    const int ct = blockIdx.y % ctiles;
    const int tap = blockIdx.z;
    const int tr = tap / p.S;
    const int ts = tap % p.S;
    const int dh_off = tr * p.dh - p.pbh;
    const int dw_off = ts * p.dw - p.pbw;

    const uint32_t m_begin = split * p.chunk;
    const uint32_t m_end = (m_begin + p.chunk < p.M) ? m_begin + p.chunk : p.M;
    const int nsteps = (m_begin < m_end) ? (int)((m_end - m_begin + 63) >> 6) : 0;

    // loader role: pair = tid % 32 (positions 2*pair, 2*pair+1 of the step), half = tid / 32
    // (channels 8*half .. 8*half+7 of the 64-channel tile)
    const int pair = tid & 31;
    const int half = tid >> 5;
    const int PQ = p.P * p.Q;
    const int HW = p.H * p.W;
    const int KB = p.K >> 4;
    const int CB = p.C >> 4;
    const int dy_cb = kt * 4 + (half >> 1);              // 16-channel block of dy this thread reads
    const int x_cb = ct * 4 + (half >> 1);
    const int sub = (half & 1) * 8;                      // element offset inside the block

    uint4 dyr[2], xr[2];

    auto load_global = [&](int step) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint32_t m = m_begin + step * 64 + 2 * pair + j;
            uint4 vdy = make_uint4(0, 0, 0, 0), vx = make_uint4(0, 0, 0, 0);
            if (m < m_end) {
                const uint32_t n = fd_div(m, p.div_pq);
                const uint32_t rem = m - n * PQ;
                const uint32_t pp = fd_div(rem, p.div_q);
                const uint32_t qq = rem - pp * p.Q;
                const size_t dblk = ((size_t)n * KB + dy_cb) * PQ + rem;
                vdy = *reinterpret_cast<const uint4 *>(p.dy + dblk * 16 + sub);
                const int ih = (int)pp * p.sh + dh_off;
                const int iw = (int)qq * p.sw + dw_off;
                if ((unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W) {
                    const size_t xblk = ((size_t)n * CB + x_cb) * HW + (size_t)ih * p.W + iw;
                    vx = *reinterpret_cast<const uint4 *>(p.x + xblk * 16 + sub);
                }
            }
            dyr[j] = vdy;
            xr[j] = vx;
        }
    };
    auto store_lds = [&](int stage) {
        unsigned char *dyt = smem + stage * WG_STAGE;
        unsigned char *xt = dyt + WG_TILE;
        interleave_store(dyt, half, pair, dyr[0], dyr[1]);
        interleave_store(xt, half, pair, xr[0], xr[1]);
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    if (nsteps > 0) {
        load_global(0);
        store_lds(0);
    }
    __syncthreads();

    for (int s = 0; s < nsteps; ++s) {
        const bool more = (s + 1 < nsteps);
        if (more) load_global(s + 1);
        const unsigned char *dyt = smem + (s & 1) * WG_STAGE;
        const unsigned char *xt = dyt + WG_TILE;
        bf16x8 fa[2], fb[2];
        const int col = (wave * 16 + lg * 8) * 2;        // byte offset of this lane's 8 positions
#pragma unroll
        for (int a = 0; a < 2; ++a) fa[a] = *reinterpret_cast<const bf16x8 *>(dyt + (a * 32 + l32) * WG_PITCH + col);
#pragma unroll
        for (int b = 0; b < 2; ++b) fb[b] = *reinterpret_cast<const bf16x8 *>(xt + (b * 32 + l32) * WG_PITCH + col);
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
        if (more) store_lds((s + 1) & 1);
        __syncthreads();
    }

    // ---- sum the four wave copies in a fixed order: (w0 + w1) + (w2 + w3), through LDS.
    // Layout of a copy in LDS: float [64 rows k][64 cols c]; lane owns column c = 32b + l32 and
    // rows k = 32a + 8*(v/4) + 4*lg + v%4.
    float *red = reinterpret_cast<float *>(smem);         // 2 copies x 16 KB = 32 KB <= 36 KB
    auto red_index = [&](int a, int b, int v) { return (a * 32 + 8 * (v >> 2) + 4 * lg + (v & 3)) * 64 + b * 32 + l32; };
    // first level: waves 1 and 3 publish, waves 0 and 2 add
    if (wave & 1) {
        float *dst = red + (wave >> 1) * 4096;
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) dst[red_index(a, b, v)] = acc[a][b][v];
    }
    __syncthreads();
    if (!(wave & 1)) {
        const float *src = red + (wave >> 1) * 4096;
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[a][b][v] += src[red_index(a, b, v)];
    }
    __syncthreads();
    // second level: wave 2 publishes, wave 0 adds and writes the partial tile
    if (wave == 2) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) red[red_index(a, b, v)] = acc[a][b][v];
    }
    __syncthreads();
    if (wave == 0) {
        float *out = p.partial + ((size_t)split * (p.R * p.S) + tap) * p.K * p.C;
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int k = kt * 64 + a * 32 + 8 * (v >> 2) + 4 * lg + (v & 3);
                    const int c = ct * 64 + b * 32 + l32;
                    out[(size_t)k * p.C + c] = acc[a][b][v] + red[red_index(a, b, v)];
                }
    }
}

// dw[k][c][r][s] = sum over splits (index order) of partial[split][tap][k][c]
__global__ __launch_bounds__(256) void wgrad_reduce(const float *__restrict__ partial, float *__restrict__ dw, int splits,
                                                    int K, int C, int RS)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;       // index into [tap][k][c]
    const size_t per = (size_t)RS * K * C;
    if (i >= per) return;
    float acc = 0.f;
    for (int sp = 0; sp < splits; ++sp) acc += partial[(size_t)sp * per + i];
    const int c = i % C;
    const size_t t = i / C;
    const int k = t % K;
    const int tap = (int)(t / K);
    dw[((size_t)k * C + c) * RS + tap] = acc;
}

hipError_t launch_wgrad(const WgradParams &p, hipStream_t st)
{
    dim3 grid(p.splits, (p.K / 64) * (p.C / 64), p.R * p.S);
    NGC_LAUNCH(wgrad_bf16, grid, dim3(256), 0, st, p);
    return ngc::launch_result();
}

hipError_t launch_wgrad_reduce(const float *partial, float *dw, int splits, int K, int C, int R, int S, hipStream_t st)
{
    const size_t per = (size_t)R * S * K * C;
    NGC_LAUNCH(wgrad_reduce, dim3((unsigned)((per + 255) / 256)), dim3(256), 0, st, partial, dw, splits, K, C,
                       R * S);
    return ngc::launch_result();
}

}  // namespace ngc
