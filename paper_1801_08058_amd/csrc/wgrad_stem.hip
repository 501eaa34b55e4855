// ConvolutionBackpropFilters of the low-channel stem (C <= 3, 7x7, stride 2, pad_w 3) on bf16
// MFMA (gfx950): x in NCHW, dy 16-channel-blocked, dw fp32 [K][C][7][7].
//
//   dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x[n,c, 2p-pad_h+r, 2q-3+s]
//
// GEMM: rows = k (64 per workgroup), columns = (c,r) pair x 8 slots (slot j>0 = tap s=j-1, slot 0
// and columns >= 8*7C are dummies) = 176 columns as 11 fragments of 16, reduction = positions.
// v_mfma_f32_16x16x32_bf16; a lane supplies 8 consecutive positions q..q+7 of one row p:
//   A (dy^T): dy tile kept in LDS in its natural [position][16 k] form (direct global->LDS
//             loads) and fetched with the LDS transpose load ds_read_b64_tr_b16;
//   B (x)   : for column (c,r,slot) the 8 elements are x[c][2p-pad+r][2q-4+slot + 2i], i = 0..7 -
//             a stride-2 run.  Input rows are therefore stored in LDS de-interleaved into an
//             even-column plane and an odd-column plane, where the run is 8 consecutive bf16 at
//             an arbitrary 2-byte offset: 5 aligned dwords + a funnel shift (v_alignbit) per lane.
// Workgroup = 8 waves = 2 column groups (6 + 5 fragments) x 4 interleaved streams of
// 32-position steps (a wave-level split of the reduction, summed through LDS in a fixed tree);
// one workgroup per strip of dy rows; partials in register order to the workspace, summed in
// index order by wgrad_stem_reduce (deterministic, no atomics).
#include "common.h"

namespace ngc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void lds_void_s;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4_s;

constexpr unsigned WST_OOB = 0x80000000u;
constexpr int WST_NF = 6;            // column fragments per wave (second group uses 5)
constexpr int WST_XCH = 3;           // 16-byte x chunks per thread per stage

__device__ __forceinline__ bf16x8 tr_frag_s(const unsigned char *lo, const unsigned char *hi)
{
    const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_s *)lo);
    const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_s *)hi);
    const s16x8 r = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

// RING: three stage buffers and every global read as a direct global->LDS load with counted waits (the input rows
// land as they are in a small staging area and the thread that requested a 16-byte piece splits it into the parity
// planes once it is there); else two stage buffers, the input rows through registers.
template <bool RING>
__global__ __launch_bounds__(512) void wgrad_stem_bf16(const WgradStemParams p)
{
    preload_kernargs(p);
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cg = wave & 1;                 // column group: fragments 6cg .. 6cg+5
    const int wh = wave >> 1;                // step stream 0..3
    const int L = lane & 15;
    const int grp = lane >> 4;               // positions +8*grp inside a 32-position step

    const int img = blockIdx.x / p.strips;
    const int strip = blockIdx.x - img * p.strips;
    const int p0 = strip * p.TP;
    const int rows_strip = (p.P - p0 < p.TP) ? (p.P - p0) : p.TP;
    const int kt = blockIdx.y;

    const int PQ = p.P * p.Q;
    const int KB = p.K >> 4;
    const int rows_in = 2 * p.SR + 5;                        // input rows per stage
    // bytes per parity plane of a row (4 + W/2 + 4 bf16 = W + 16 used) and per row; the host pads both so that the
    // 64 lanes of an operand read (2 (c,r) pairs x 2 planes x 4 position groups x 2 dwords) fall into 64 different banks
    const int PL = p.PL;
    const int RPX = p.RPX;
    const int xbytes = p.C * rows_in * RPX;
    const int stage_bytes = 4 * p.dyplane + ((xbytes + 15) & ~15);
    const int steps_full = (p.SR * p.Q) >> 5;                // SR*Q is a multiple of 32
    const int nstages = (rows_strip + p.SR - 1) / p.SR;

    __amdgpu_buffer_rsrc_t rs_dy = __builtin_amdgcn_make_buffer_rsrc((void *)p.dy, 0, (int)p.dy_bytes, 0x00020000);

    // ---- per-lane column constants: fragment f -> column 16*(6cg+f) + L -> (pair, slot)
    int colconst[WST_NF], colsh[WST_NF];
#pragma unroll
    for (int f = 0; f < WST_NF; ++f) {
        int col = 16 * (WST_NF * cg + f) + L;
        int pair = col >> 3, slot = col & 7;
        if (pair >= p.C * 7) { pair = 0; slot = 1; }        // dummy column: any valid address
        const int c = pair / 7, r = pair - c * 7;
        const int b = (c * rows_in + r) * RPX + (slot & 1) * PL + 2 * ((slot >> 1) + 2);   // byte offset of element a(q=0)
        colconst[f] = b & ~3;
        colsh[f] = (b & 2) * 8;
    }

    const int cpr = p.W >> 3;                                // 16-byte chunks per input row
    const int xchunks = p.C * rows_in * cpr;                 // <= 512 * WST_XCH (host)
    uint4 xr[WST_XCH];

    auto issue_dy = [&](int s, int buf) {
        unsigned char *base = smem + buf * stage_bytes;
        const int r0 = s * p.SR;
        int rows = rows_strip - r0;
        if (rows > p.SR) rows = p.SR;
        const int nvalid = rows * p.Q;
        for (int it = wave; it < 4 * steps_full; it += 8) {
            const int pln = it / steps_full, blk = it - pln * steps_full;
            const unsigned dy_base = (unsigned)((((img * KB + kt * 4 + pln) * PQ) + (p0 + r0) * p.Q) * 32);
            const int pos = blk * 32 + (lane >> 1);
            const unsigned off = (pos < nvalid) ? dy_base + (unsigned)(pos * 32 + (lane & 1) * 16) : WST_OOB;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_dy, (lds_void_s *)(base + pln * p.dyplane + blk * 1024), 16, (int)off,
                                                     0, 0, 0);
        }
    };
    auto load_x = [&](int s) {
        const int h0 = 2 * (p0 + s * p.SR) - p.pbh;
#pragma unroll
        for (int u = 0; u < WST_XCH; ++u) {
            const int i = tid + 512 * u;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (i < xchunks) {
                const int ch = i % cpr;
                const int rr = i / cpr;
                const int c = rr / rows_in;
                const int h = h0 + (rr - c * rows_in);
                if ((unsigned)h < (unsigned)p.H)
                    v = *reinterpret_cast<const uint4 *>(p.x + (((size_t)img * p.C + c) * p.H + h) * p.W + ch * 8);
            }
            xr[u] = v;
        }
    };
    auto store_x = [&](int buf) {
        unsigned char *xs = smem + buf * stage_bytes + 4 * p.dyplane;
#pragma unroll
        for (int u = 0; u < WST_XCH; ++u) {
            const int i = tid + 512 * u;
            if (i < xchunks) {
                const int ch = i % cpr;
                const int rr = i / cpr;
                const uint4 v = xr[u];
                unsigned char *row = xs + rr * RPX;
                const uint2 ev = make_uint2((v.x & 0xFFFFu) | (v.y << 16), (v.z & 0xFFFFu) | (v.w << 16));
                const uint2 od = make_uint2((v.x >> 16) | (v.y & 0xFFFF0000u), (v.z >> 16) | (v.w & 0xFFFF0000u));
                *reinterpret_cast<uint2 *>(row + 8 + ch * 8) = ev;
                *reinterpret_cast<uint2 *>(row + PL + 8 + ch * 8) = od;
                if (ch == 0) {
                    *reinterpret_cast<uint2 *>(row) = make_uint2(0, 0);
                    *reinterpret_cast<uint2 *>(row + PL) = make_uint2(0, 0);
                }
                if (ch == cpr - 1) {
                    *reinterpret_cast<uint2 *>(row + 8 + p.W) = make_uint2(0, 0);
                    *reinterpret_cast<uint2 *>(row + PL + 8 + p.W) = make_uint2(0, 0);
                }
            }
        }
    };

    f32x4 acc[4][WST_NF];
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int f = 0; f < WST_NF; ++f)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[kb][f][v] = 0.f;

    const int lane_col = (L & 3) * 8;
    const int nfr = cg ? WST_NF - 1 : WST_NF;               // the 12th fragment does not exist

    // ---- RING: stage s lives in buffer s % 3; raw input rows of stage s in staging area s & 1 behind the ring
    const ngc_u32x4 rw_dy = make_rsrc_words(p.dy, p.dy_bytes);
    const ngc_u32x4 rw_x = make_rsrc_words(p.x, p.x_bytes);
    unsigned char *raw0 = smem + 3 * stage_bytes;
    const int raw_bytes = ((xchunks + 63) & ~63) * 16;
    const int ndy = (4 * steps_full - wave + 7) / 8;        // this wave's dy loads per stage
    int nxw = (xchunks - wave * 64 + 511) / 512;            // and its loads of input-row pieces
    nxw = nxw < 0 ? 0 : nxw > WST_XCH ? WST_XCH : nxw;
    const int lpw = nxw + ndy;
    auto issue_stage = [&](int s) {                         // lpw loads, always
        const int h0 = 2 * (p0 + s * p.SR) - p.pbh;
        unsigned char *raw = raw0 + (s & 1) * raw_bytes;
#pragma unroll
        for (int u = 0; u < WST_XCH; ++u) {
            const int i = tid + 512 * u;
            const int ch = i % cpr;
            const int rr = i / cpr;
            const int c = rr / rows_in;
            const int h = h0 + (rr - c * rows_in);
            const bool ok = i < xchunks && (unsigned)h < (unsigned)p.H;
            const unsigned off = ok ? (unsigned)(((((img * p.C + c) * p.H + h) * p.W) + ch * 8) * 2) : WST_OOB;
            if (wave * 64 + 512 * u < xchunks)              // wave-uniform; the staging area ends at a multiple of 64 pieces
                dma_load_lds16(rw_x, raw + (wave * 64 + 512 * u) * 16, off, 0);
        }
        unsigned char *base = smem + (s % 3) * stage_bytes;
        const int r0 = s * p.SR;
        int rows = rows_strip - r0;
        if (rows > p.SR) rows = p.SR;
        const int nvalid = rows * p.Q;
        for (int it = wave; it < 4 * steps_full; it += 8) {
            const int pln = it / steps_full, blk = it - pln * steps_full;
            const unsigned dy_base = (unsigned)((((img * KB + kt * 4 + pln) * PQ) + (p0 + r0) * p.Q) * 32);
            const int pos = blk * 32 + (lane >> 1);
            const unsigned off = (pos < nvalid) ? dy_base + (unsigned)(pos * 32 + (lane & 1) * 16) : WST_OOB;
            // the quotient comes out of the vector unit: hand the (wave-uniform) destination over as a scalar
            dma_load_lds16(rw_dy, base + __builtin_amdgcn_readfirstlane(pln * p.dyplane + blk * 1024), off, 0);
        }
    };
    auto split_x = [&](int s) {                             // own pieces of stage s: staging area -> parity planes
        const unsigned char *raw = raw0 + (s & 1) * raw_bytes;
        unsigned char *xs = smem + (s % 3) * stage_bytes + 4 * p.dyplane;
#pragma unroll
        for (int u = 0; u < WST_XCH; ++u) {
            const int i = tid + 512 * u;
            if (i < xchunks) {
                const int ch = i % cpr;
                const int rr = i / cpr;
                const uint4 v = *reinterpret_cast<const uint4 *>(raw + i * 16);
                unsigned char *row = xs + rr * RPX;
                const uint2 ev = make_uint2((v.x & 0xFFFFu) | (v.y << 16), (v.z & 0xFFFFu) | (v.w << 16));
                const uint2 od = make_uint2((v.x >> 16) | (v.y & 0xFFFF0000u), (v.z >> 16) | (v.w & 0xFFFF0000u));
                *reinterpret_cast<uint2 *>(row + 8 + ch * 8) = ev;
                *reinterpret_cast<uint2 *>(row + PL + 8 + ch * 8) = od;
                if (ch == 0) {
                    *reinterpret_cast<uint2 *>(row) = make_uint2(0, 0);
                    *reinterpret_cast<uint2 *>(row + PL) = make_uint2(0, 0);
                }
                if (ch == cpr - 1) {
                    *reinterpret_cast<uint2 *>(row + 8 + p.W) = make_uint2(0, 0);
                    *reinterpret_cast<uint2 *>(row + PL + 8 + p.W) = make_uint2(0, 0);
                }
            }
        }
    };

    if constexpr (RING) {
        issue_stage(0);
        if (nstages > 1) issue_stage(1);
        wait_vmcnt(nstages > 1 ? lpw : 0);                  // stage 0 has landed (this wave's part)
        split_x(0);
    } else {
        issue_dy(0, 0);
        load_x(0);
        store_x(0);
    }
    for (int s = 0; s < nstages; ++s) {
        const bool more = s + 1 < nstages;
        if constexpr (RING) {
            // every wave has split its input pieces of stage s and seen its dy loads of stage s land; the barrier
            // makes that true for the workgroup and frees the buffer of stage s - 1 for the loads of stage s + 2
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            wg_barrier_nofence();
            if (s + 2 < nstages) issue_stage(s + 2);
        } else {
            __builtin_amdgcn_s_waitcnt(0x0F70);             // vmcnt(0): dy of stage s has landed (this wave's part)
            __syncthreads();
            if (more) {
                issue_dy(s + 1, (s + 1) & 1);
                load_x(s + 1);
            }
        }
        int rows = rows_strip - s * p.SR;
        if (rows > p.SR) rows = p.SR;
        const int nsteps = (rows * p.Q) >> 5;               // rows*Q is a multiple of 8; partial steps handled by zero dy
        const int nsteps_up = (rows * p.Q + 31) >> 5;
        (void)nsteps;
        const unsigned char *dys = smem + (RING ? s % 3 : s & 1) * stage_bytes;
        const unsigned char *xs = dys + 4 * p.dyplane;
        for (int j = (wh - (s * steps_full) % 4 + 4) % 4; j < nsteps_up; j += 4) {
            // this lane group's 8 positions: m8 .. m8+7, all in dy row pr
            int m8 = j * 32 + grp * 8;
            const int dyo0 = (m8 + (L >> 2)) * 32 + lane_col;
            if (m8 > p.SR * p.Q - 8) m8 = p.SR * p.Q - 8;   // beyond the stage: dy is zero, keep x in range
            const uint32_t pr = fd_div((uint32_t)m8, p.div_q);
            const uint32_t qa = (uint32_t)m8 - pr * p.div_q.d;
            const int pospart = (int)(2 * pr) * RPX + (int)qa * 2;
            bf16x8 a[4];
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) a[kb] = tr_frag_s(dys + kb * p.dyplane + dyo0, dys + kb * p.dyplane + dyo0 + 128);
#pragma unroll
            for (int f = 0; f < WST_NF; ++f) {
                if (f < nfr) {
                    const uint32_t *src = reinterpret_cast<const uint32_t *>(xs + colconst[f] + pospart);
                    const uint32_t w0 = src[0], w1 = src[1], w2 = src[2], w3 = src[3], w4 = src[4];
                    union { uint32_t d[4]; bf16x8 v; } u;
                    u.d[0] = __builtin_amdgcn_alignbit(w1, w0, colsh[f]);
                    u.d[1] = __builtin_amdgcn_alignbit(w2, w1, colsh[f]);
                    u.d[2] = __builtin_amdgcn_alignbit(w3, w2, colsh[f]);
                    u.d[3] = __builtin_amdgcn_alignbit(w4, w3, colsh[f]);
#pragma unroll
                    for (int kb = 0; kb < 4; ++kb)
                        acc[kb][f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[kb], u.v, acc[kb][f], 0, 0, 0);
                }
            }
        }
        if constexpr (RING) {
            if (more) {
                wait_vmcnt(s + 2 < nstages ? lpw : 0);              // stage s + 1 has landed (this wave's part)
                split_x(s + 1);
            }
        } else {
            if (more) store_x((s + 1) & 1);
        }
    }
    __syncthreads();

    // ---- fixed-order tree over the 4 step streams, then the partial in register order
    f32x4 *red = reinterpret_cast<f32x4 *>(smem);
#pragma unroll
    for (int stride = 2; stride >= 1; stride >>= 1) {
        if (wh >= stride && wh < 2 * stride) {
            f32x4 *dst = red + ((wh - stride) * 2 + cg) * (4 * WST_NF * 64);
#pragma unroll
            for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                for (int f = 0; f < WST_NF; ++f) dst[(kb * WST_NF + f) * 64 + lane] = acc[kb][f];
        }
        __syncthreads();
        if (wh < stride) {
            const f32x4 *src = red + (wh * 2 + cg) * (4 * WST_NF * 64);
#pragma unroll
            for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                for (int f = 0; f < WST_NF; ++f) acc[kb][f] += src[(kb * WST_NF + f) * 64 + lane];
        }
        __syncthreads();
    }
    if (wh == 0) {
        f32x4 *out = reinterpret_cast<f32x4 *>(p.partial) +
                     (((size_t)blockIdx.x * gridDim.y + kt) * 2 + cg) * (4 * WST_NF * 64);
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
            for (int f = 0; f < WST_NF; ++f) out[(kb * WST_NF + f) * 64 + lane] = acc[kb][f];
    }
}

// dw = sum over parts (index order); element i of a part = (((kt*2 + cg)*4 + kb)*6 + f)*64 + lane (float4)
__global__ __launch_bounds__(256) void wgrad_stem_reduce(const f32x4 *__restrict__ partial, float *__restrict__ dw,
                                                        int nparts, int K, int C)
{
    // 256 threads = 8 outputs x 32 part slices (few outputs, many parts: the slices keep enough loads in flight);
    // slice s adds parts s, s + 32, ... in index order, the slices are summed in a fixed tree
    __shared__ f32x4 sm[32][8];
    const size_t per4 = (size_t)(K / 64) * 2 * 4 * WST_NF * 64;
    const int o = threadIdx.x & 7;
    const int sl = threadIdx.x >> 3;
    const size_t i = (size_t)blockIdx.x * 8 + o;
    f32x4 t0 = {0.f, 0.f, 0.f, 0.f}, t1 = t0;
    int sp = sl;
    for (; sp + 32 < nparts; sp += 64) {
        t0 += partial[(size_t)sp * per4 + i];
        t1 += partial[(size_t)(sp + 32) * per4 + i];
    }
    if (sp < nparts) t0 += partial[(size_t)sp * per4 + i];
    sm[sl][o] = t0 + t1;
    __syncthreads();
    if (sl == 0) {
        f32x4 q[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) q[j] = (sm[4 * j][o] + sm[4 * j + 1][o]) + (sm[4 * j + 2][o] + sm[4 * j + 3][o]);
        const f32x4 r = ((q[0] + q[1]) + (q[2] + q[3])) + ((q[4] + q[5]) + (q[6] + q[7]));
        const int lane = (int)(i & 63);
        size_t u = i >> 6;
        const int f = (int)(u % WST_NF); u /= WST_NF;
        const int kb = (int)(u & 3); u >>= 2;
        const int cg = (int)(u & 1); u >>= 1;
        const int kt = (int)u;
        const int col = 16 * (WST_NF * cg + f) + (lane & 15);
        const int pair = col >> 3, slot = col & 7;
        if (slot == 0 || pair >= C * 7) return;
        const int k = kt * 64 + kb * 16 + 4 * (lane >> 4);
#pragma unroll
        for (int v = 0; v < 4; ++v) dw[((size_t)(k + v) * C * 7 + pair) * 7 + slot - 1] = r[v];
    }
}

hipError_t launch_wgrad_stem(const WgradStemParams &p, size_t lds_bytes, hipStream_t st)
{
    dim3 grid(p.N * p.strips, p.K / 64);
    if (p.ring) {
        static LdsLimitOnce lds_limit;              // per template instantiation
        const hipError_t e = lds_limit.raise(reinterpret_cast<const void *>(&wgrad_stem_bf16<true>));
        if (e != hipSuccess) return e;
        NGC_LAUNCH(wgrad_stem_bf16<true>, grid, dim3(512), lds_bytes, st, p);
    } else {
        static LdsLimitOnce lds_limit;
        const hipError_t e = lds_limit.raise(reinterpret_cast<const void *>(&wgrad_stem_bf16<false>));
        if (e != hipSuccess) return e;
        NGC_LAUNCH(wgrad_stem_bf16<false>, grid, dim3(512), lds_bytes, st, p);
    }
    hipError_t e = ngc::launch_result();
    if (e != hipSuccess) return e;
    const size_t per4 = (size_t)(p.K / 64) * 2 * 4 * WST_NF * 64;
    NGC_LAUNCH(wgrad_stem_reduce, dim3((unsigned)(per4 / 8)), dim3(256), 0, st,
               reinterpret_cast<const f32x4 *>(p.partial), p.dw, p.N * p.strips, p.K, p.C);
    return ngc::launch_result();
}

}  // namespace ngc
