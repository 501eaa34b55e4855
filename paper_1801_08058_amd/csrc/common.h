// Internal declarations shared by the translation units of libngconv (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/ngconv.h"

// Launch wrapper: the HIP "last error" is per-thread state shared with every other user of the
// runtime in the process (a pending hipEventQuery of the caller's allocator leaves
// hipErrorNotReady there), so it is cleared before the launch and read right after it.
#define NGC_LAUNCH(...)            \
    do {                           \
        if (ngc::dry_run()) break; \
        (void)hipGetLastError();   \
        hipLaunchKernelGGL(__VA_ARGS__); \
    } while (0)

// Cache policy of the stores of result tensors (buffer-store aux bits / non-temporal flag).  A result is written once
// and not read again by the kernel that writes it; where a kernel's stores cover whole cache lines (every pixel of the
// tensor, i.e. output pixel stride 1) they are marked as streaming, so they leave the L2 as they are written instead of
// when the kernel ends (headline 3x3 layer: forward 18.9 -> 17.4 us).  Strided backprop-data writes every other pixel
// per launch or per store instruction and keeps ordinary stores (streaming partial lines doubles its time).
// The buffer stores also carry the system-scope bit (aux 16: written through; another 2-4 % on the strip and stem
// kernels).  NGC_ST_AUX = 0: ordinary stores everywhere.
#ifndef NGC_ST_AUX
#define NGC_ST_AUX 18
#endif
namespace ngc {

// 16-byte store of a result element group; stream (wave-uniform): see NGC_ST_AUX
__device__ __forceinline__ void store16_result(void *dst, uint4 v, bool stream)
{
    typedef unsigned ngc_st_u32x4 __attribute__((ext_vector_type(4)));
    const ngc_st_u32x4 w = {v.x, v.y, v.z, v.w};
    if (NGC_ST_AUX != 0 && stream) {
        asm volatile("" ::: "memory");      // keeps the two stores apart: hoisted or sunk into one, they lose the flag
        __builtin_nontemporal_store(w, reinterpret_cast<ngc_st_u32x4 *>(dst));
        asm volatile("" ::: "memory");
    } else {
        *reinterpret_cast<ngc_st_u32x4 *>(dst) = w;
    }
}

// ---- environment switches (tests and experiments only; the default build path reads none of them per call) ----
// The NGC_* variables are read once per process, at the first use, into a table; env_switch(SW_X) returns the value of
// NGC_X or nullptr.  ngc_reload_switches() (exported for the test suite) reads them again and bumps the epoch, which
// also drops every cached plan.
enum Switch { SW_CONV3D_RANK2, SW_CONV3D_STRIP, SW_DB_FUSE, SW_G1_NCHW, SW_G1_VARIANT, SW_GEMM1X1, SW_STEM_BH, SW_STEM_TP, SW_STRIP_BW, SW_STRIP_MERGE, SW_STRIP_NF, SW_STRIP_ROWS, SW_STRIP_STRIDED, SW_STRIP_XCD, SW_WGG3_PARTS, SW_WGG_SLOTS, SW_WGG_SP, SW_WGG_TILE, SW_WGG_XCD, SW_WGRAD_G1, SW_WGRAD_GEMM, SW_WGRAD_LATE, SW_WGRAD_NCQ, SW_WGRAD_RING, SW_WGRAD_STRIP, SW_WSTEM_POS, SW_WSTEM_RING, SW_ROWS, SW_ROWS_LATE, SW_STAGED, SW_STRIP_TAIL, SW_STRIP_SPLIT, SW_WGRAD_NT, SW_STRIP_CPS, SW_DRY_RUN, SW_COUNT };
const char *env_switch(Switch s);
uint32_t sw_epoch();
// NGC_DRY_RUN=1: every launch is skipped after the host-side planning (host-path timing without a GPU)
bool dry_run();
// what a launcher returns right after NGC_LAUNCH
inline hipError_t launch_result() { return dry_run() ? hipSuccess : hipGetLastError(); }

// ---- exact unsigned division by a runtime constant (round-up multiplier method) ----
// q = n / d for every 32-bit n: t = mulhi(mul, n); q = (t + ((n - t) >> sh1)) >> sh2.
struct FastDiv {
    uint32_t mul, sh1, sh2, d;
};

inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;                       // l = ceil(log2 d)
    f.mul = (uint32_t)((((1ull << l) - d) << 32) / d + 1);
    f.sh1 = l < 1 ? l : 1;
    f.sh2 = l - f.sh1;
    f.d = d;
    return f;
}

__host__ __device__ inline uint32_t fd_mulhi(uint32_t a, uint32_t b)
{
    return (uint32_t)(((uint64_t)a * b) >> 32);      // v_mul_hi_u32 on the device
}

__host__ __device__ inline uint32_t fd_div(uint32_t n, const FastDiv &f)
{
    uint32_t t = fd_mulhi(f.mul, n);
    return (t + ((n - t) >> f.sh1)) >> f.sh2;
}

// ---- bf16 bit helpers ----
__host__ __device__ inline float bf16_bits_to_float(uint16_t b)
{
    union { uint32_t u; float f; } v;
    v.u = (uint32_t)b << 16;
    return v.f;
}

// round-to-nearest-even on the 16 dropped bits (finite inputs; canonical NaN stays NaN)
__host__ __device__ inline uint32_t float_to_bf16_bits(float x)
{
    union { uint32_t u; float f; } v;
    v.f = x;
    uint32_t u = v.u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

__host__ __device__ inline uint32_t pack_bf16x2(float lo, float hi)
{
    return float_to_bf16_bits(lo) | (float_to_bf16_bits(hi) << 16);
}

// two fp32 -> packed bf16x2 with the hardware conversion (v_cvt_pk_bf16_f32, round-to-nearest-even)
__device__ __forceinline__ uint32_t pack_bf16x2_hw(float lo, float hi)
{
    // as one vector conversion: two scalar casts become two conversions and a byte permute
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// ReLU of two rounded bf16 values at once (or of neither: on = false).  As 16-bit integers the negative bf16 values
// (and -0) are the negative numbers, so a signed maximum with 0 is max(v, 0) of both halves in one instruction, and
// rounding to nearest even keeps the sign, so it commutes with ReLU for every finite value and the infinities; a
// maximum with the most negative integer changes nothing.  (A NaN, which finite inputs cannot produce, stays a NaN here
// where an fp32 maximum would give 0.)
__device__ __forceinline__ uint32_t relu_bf16x2(uint32_t w, bool on)
{
    typedef short ngc_s16x2 __attribute__((ext_vector_type(2)));
    const short fl = on ? (short)0 : (short)-32768;
    const ngc_s16x2 v = __builtin_bit_cast(ngc_s16x2, w), f = {fl, fl};
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(v, f));
}

// A kernel's by-value argument struct lives in the kernel-argument segment and is read with scalar loads where a
// field is first used; every 64-byte line of it that is touched for the first time costs a round trip to memory, and
// left to the compiler these come one after the other all through the set-up code.  Reading one word of every line
// at the top of the kernel brings the whole segment into the scalar cache in one batch of loads under one wait.
template <class P>
__device__ __forceinline__ void preload_kernargs(const P &p)
{
    const uint32_t *w = reinterpret_cast<const uint32_t *>(&p);
    constexpr unsigned n = sizeof(P) / 4;
#pragma unroll
    for (unsigned b = 0; b < n; b += 256) {               // 16 lines per statement: one clause of loads, one wait
#define NGC_KARG_LINE(k) w[b + 16 * (k) < n ? b + 16 * (k) : 0]
        asm volatile("" ::"s"(NGC_KARG_LINE(0)), "s"(NGC_KARG_LINE(1)), "s"(NGC_KARG_LINE(2)), "s"(NGC_KARG_LINE(3)),
                     "s"(NGC_KARG_LINE(4)), "s"(NGC_KARG_LINE(5)), "s"(NGC_KARG_LINE(6)), "s"(NGC_KARG_LINE(7)),
                     "s"(NGC_KARG_LINE(8)), "s"(NGC_KARG_LINE(9)), "s"(NGC_KARG_LINE(10)), "s"(NGC_KARG_LINE(11)),
                     "s"(NGC_KARG_LINE(12)), "s"(NGC_KARG_LINE(13)), "s"(NGC_KARG_LINE(14)), "s"(NGC_KARG_LINE(15)));
#undef NGC_KARG_LINE
    }
}

// s_waitcnt vmcnt(n) for a wave-uniform run-time n; waiting for fewer outstanding loads than
// necessary is always correct, so counts beyond the table fall back to vmcnt(0).
__device__ __forceinline__ void wait_vmcnt(int n)
{
    // the count is a 6-bit field split over bits 3:0 and 15:14 of the immediate; the other counters stay unconstrained
#define NGC_VMCNT_CASE(N) case N: __builtin_amdgcn_s_waitcnt(0x0F70 | ((N) & 15) | (((N) >> 4) << 14)); break;
    switch (n) {
        NGC_VMCNT_CASE(1) NGC_VMCNT_CASE(2) NGC_VMCNT_CASE(3) NGC_VMCNT_CASE(4) NGC_VMCNT_CASE(5) NGC_VMCNT_CASE(6)
        NGC_VMCNT_CASE(7) NGC_VMCNT_CASE(8) NGC_VMCNT_CASE(9) NGC_VMCNT_CASE(10) NGC_VMCNT_CASE(11) NGC_VMCNT_CASE(12)
        NGC_VMCNT_CASE(13) NGC_VMCNT_CASE(14) NGC_VMCNT_CASE(15) NGC_VMCNT_CASE(16) NGC_VMCNT_CASE(17) NGC_VMCNT_CASE(18)
        NGC_VMCNT_CASE(19) NGC_VMCNT_CASE(20) NGC_VMCNT_CASE(21) NGC_VMCNT_CASE(22) NGC_VMCNT_CASE(23) NGC_VMCNT_CASE(24)
        NGC_VMCNT_CASE(25) NGC_VMCNT_CASE(26) NGC_VMCNT_CASE(27) NGC_VMCNT_CASE(28) NGC_VMCNT_CASE(29) NGC_VMCNT_CASE(30)
        NGC_VMCNT_CASE(31)
    default: __builtin_amdgcn_s_waitcnt(0x0F70); break;
    }
#undef NGC_VMCNT_CASE
}

// Each lane of a 32-lane half-wave holds v[0..31]; returns, in lane l (l = lane % 32), the sum over the 32
// lanes of v[j(l)], j(l) = ((l % 16) << 1) | (l / 16).  A butterfly that halves the values a lane carries
// at every step (16 + 8 + 4 + 2 + 1 exchanges instead of 32 x 5), in a fixed order.  The four large steps
// are DPP lane permutations inside a row of 16 (mirror, half mirror, quad swaps: one VALU operation each;
// LDS-based shuffles here cost a 1x1 layer more than a second pass over its output); the mirrored partners
// come first because they also flip the lower lane bits, which no step has used by then.
template <int CTRL>
__device__ __forceinline__ float dpp_perm_f32(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float half_wave_transpose_sum32(float (&v)[32], int l32)
{
    constexpr int ROW_MIRROR = 0x140, ROW_HALF_MIRROR = 0x141, QUAD_XOR2 = 0x4E, QUAD_XOR1 = 0xB1;
    bool up = (l32 & 8) != 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = (up ? v[i + 16] : v[i]) + dpp_perm_f32<ROW_MIRROR>(up ? v[i] : v[i + 16]);
    up = (l32 & 4) != 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (up ? v[i + 8] : v[i]) + dpp_perm_f32<ROW_HALF_MIRROR>(up ? v[i] : v[i + 8]);
    up = (l32 & 2) != 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = (up ? v[i + 4] : v[i]) + dpp_perm_f32<QUAD_XOR2>(up ? v[i] : v[i + 4]);
    up = (l32 & 1) != 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) v[i] = (up ? v[i + 2] : v[i]) + dpp_perm_f32<QUAD_XOR1>(up ? v[i] : v[i + 2]);
    up = (l32 & 16) != 0;
    return (up ? v[1] : v[0]) + __shfl_xor(up ? v[0] : v[1], 16, 64);
}

// Lanes l and l + 32 of a 32x32 MFMA accumulator hold, for one position, the two 4-channel halves of two
// 8-channel groups: (q0, q1) of group 0 and (q2, q3) of group 1, each 2 packed bf16.  After the exchange
// lane l has all 8 channels of group 0 and lane l + 32 those of group 1 (16 bytes to store).
// v_permlane32_swap (gfx950) swaps the upper 32 lanes of one register with the lower 32 of another: two
// VALU operations instead of two LDS-based shuffles and four selects.
__device__ __forceinline__ uint4 lane_pair_exchange(uint32_t q0, uint32_t q1, uint32_t q2, uint32_t q3)
{
    const auto a = __builtin_amdgcn_permlane32_swap(q0, q2, false, false);
    const auto b = __builtin_amdgcn_permlane32_swap(q1, q3, false, false);
    return make_uint4(a[0], b[0], a[1], b[1]);
}

// ---- element index functions for the public layouts ----
// ReLU backprop on packed bf16: keep the halves of v whose counterpart in m is > 0 (as a float
// comparison: +0, -0, negatives and NaN block), zero the others.
__device__ __forceinline__ uint32_t relu_keep2(uint32_t v, uint32_t m)
{
    // As 16-bit integers the bf16 values greater than zero are 1 .. 0x7F80 (+inf); the NaNs lie above, zero and the
    // negative values (-0 is the most negative integer) below.  Two saturating differences have their sign bit set
    // exactly for m > 0 and for m < 0x7F81; their conjunction, shifted down arithmetically, is the 16-bit keep mask:
    // five packed instructions per pair.
    typedef short ngc_s16x2 __attribute__((ext_vector_type(2)));
    const ngc_s16x2 mm = __builtin_bit_cast(ngc_s16x2, m), zero = {0, 0}, lim = {0x7F81, 0x7F81};
    const ngc_s16x2 a = __builtin_elementwise_sub_sat(zero, mm);
    const ngc_s16x2 b = __builtin_elementwise_sub_sat(mm, lim);
    const ngc_s16x2 k = (a & b) >> 15;
    return v & __builtin_bit_cast(uint32_t, k);
}
__device__ __forceinline__ uint4 relu_keep8(uint4 v, uint4 m)
{
    return make_uint4(relu_keep2(v.x, m.x), relu_keep2(v.y, m.y), relu_keep2(v.z, m.z), relu_keep2(v.w, m.w));
}

__host__ __device__ inline size_t data_index(int layout, int C, int H, int W, int n, int c, int h, int w)
{
    if (layout == NGC_NCHW) return (((size_t)n * C + c) * H + h) * W + w;
    const int CB = (C + 15) >> 4;
    return ((((size_t)n * CB + (c >> 4)) * H + h) * W + w) * 16 + (c & 15);
}

__host__ __device__ inline size_t filter_index(int layout, int K, int C, int R, int S, int k, int c, int r, int s)
{
    if (layout == NGC_KCRS) return (((size_t)k * C + c) * R + r) * S + s;
    if (layout == NGC_BLOCKED_FWD) {                    // [r][s][cb][k][ci]
        const int CB = (C + 15) >> 4;
        return ((((size_t)(r * S + s)) * CB + (c >> 4)) * K + k) * 16 + (c & 15);
    }
    const int KB = (K + 15) >> 4;                       // [r][s][kb][c][ki]
    return ((((size_t)(r * S + s)) * KB + (k >> 4)) * C + c) * 16 + (k & 15);
}

// Raises a kernel's dynamic-LDS limit to the 160 KB of a gfx950 compute unit, once per device (the
// attribute belongs to the device the kernel's module is loaded on; the library runs on whatever device is
// current).  One object per kernel (template instantiation).
struct LdsLimitOnce {
    bool done[16] = {};
    hipError_t raise(const void *kernel)
    {
        if (dry_run()) return hipSuccess;
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 16 && done[dev]) return hipSuccess;
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e == hipSuccess && dev >= 0 && dev < 16) done[dev] = true;
        return e;
    }
};

// ---- implicit-GEMM (MFMA) forward / backprop-data: generalised gather convolution ----
// out[n, co, i*os_h+oa_h, j*os_w+oa_w] = sum_{tap t in class} sum_ci
//        in[n, ci, i*is_h + t.dh, j*is_w + t.dw] * wt[t.slab][ci/16][co][ci%16]
// Rank-3 spatial tensors [N][C/16][D][H][W][16] add a depth coordinate to every term (template flag R3 of the
// kernel): input slice o*is_d + t.dd, output slice o*os_d + oa_d; rank-2 launches leave those fields 0 / 1.
constexpr int IGEMM_MAX_TAPS = 64;
constexpr int IGEMM_MAX_CLASSES = 16;

struct IgemmTap {
    int32_t dh, dw, slab, dd;
};

struct IgemmClass {
    int32_t oa_h, oa_w;        // output offset of the class inside the output-stride lattice
    int32_t OP, OQ;            // lattice extents of the class
    int32_t tap_begin, tap_count;
    uint32_t M;                // N*OP*OQ (rank 3: N*OD*OP*OQ)
    FastDiv div_pq, div_q;     // divide by OP*OQ and by OQ
    int32_t oa_d, OD;          // rank 3: depth offset and lattice extent of the class
    FastDiv div_opq;           // rank 3: divide by OD*OP*OQ
};

struct IgemmParams {
    const uint16_t *in;
    const uint16_t *wt;
    uint16_t *out;
    const float *bias;         // may be null
    const uint16_t *mask;      // may be null; else same shape / layout as out: out = (mask > 0) ? out : 0
    int32_t N, Cin, Hin, Win, Cout, Hout, Wout;
    int32_t os_h, os_w, is_h, is_w;
    int32_t Din, Dout, os_d, is_d;     // rank 3 only
    int32_t relu;
    int32_t ncls;
    IgemmClass cls[IGEMM_MAX_CLASSES];
    IgemmTap taps[IGEMM_MAX_TAPS];
};

// ---- output-stationary strip kernel (stride-1 forward / backprop-data) ----
constexpr int STRIP_MAX_TAPS = 25;
constexpr int STRIP_MAX_DT = 7;       // depth taps of a rank-3 launch

struct StripParams {
    const uint16_t *in;
    const uint16_t *wt;
    uint16_t *out;
    const float *bias;         // may be null
    const uint16_t *mask;      // may be null; else same shape / layout as out: out = (mask > 0) ? out : 0
    float *dbp;                // may be null; else [rows][dbp_ld] fp32: channel sums of what each workgroup stored
                               // (row dbp_row0 + blockIdx.x): partials of a bias gradient of the stored tensor
    int32_t dbp_row0, dbp_ld;  // first row of this launch, row pitch in floats
    int32_t N, Cin, Hin, Win, Cout, Hout, Wout;
    int32_t TN, TP;            // images and output rows per workgroup
    int32_t groups, strips;    // ceil(N/TN), ceil(Hout/TP)
    int32_t PR, PC;            // patch rows / columns per image
    int32_t min_dh, min_dw;    // input row/col of patch (0,0) relative to output (p0, 0)
    int32_t npix, npatch;      // TN*TP*Wout, TN*PR*PC
    int32_t xpitch;            // bytes per X plane in LDS
    int32_t relu;
    int32_t ntaps;
    int32_t tap_off[STRIP_MAX_TAPS];    // patch-pixel offset of the tap
    int32_t tap_slab[STRIP_MAX_TAPS];
    uint32_t in_bytes, wt_bytes;
    uint32_t out_bytes;        // out_mode 0, rank 2: bytes of the stored tensor if below 2 GiB (stores then take 32-bit
                               // offsets into a buffer descriptor), else 0
    // out_mode 0: 16-channel-blocked [N][Cout/16][Hout][Wout][16].
    // out_mode 1: "sub-pixel" NCHW: output channel col = (a*sub_BW + b)*sub_C + c of position (i,j) is
    //             pixel (sub_BH*i + a, sub_BW*j + b) of channel c of an [N][sub_C][sub_H][sub_W] tensor.
    int32_t out_mode, sub_C, sub_H, sub_W, sub_BH, sub_BW;
    int32_t sub_stage;         // out_mode 1: assemble the strip's pixels in LDS and store whole rows
    int32_t sub_off[64];       // sub_stage: element offset of column col inside the staged [c][row][WP] block of
                               // a position, (c*ROWS + a)*WP + b, or -1 for padding columns
    FastDiv div_chunks, div_rows, div_subc;   // sub_stage row copy: 16-byte pieces per row, rows per channel, channels
    int32_t half_cols;         // only output columns 0..31 of the tile are in use (out_mode 1 with few columns)
    // Positions form a lattice of Hout x Wout per image.  Position (i, j) reads the patch at input
    // pixel (i*sh, j*sw) + tap and is stored at pixel (i*os_h + oa_h, j*os_w + oa_w) of an output
    // tensor of Hfull x Wfull pixels (forward: sh/sw = stride, os = 1; backprop-data: sh = sw = 1,
    // one launch per residue class (oa_h, oa_w) of the stride os).
    int32_t sh, sw, os_h, os_w, oa_h, oa_w, Hfull, Wfull;
    FastDiv div_tpq, div_q, div_prpc, div_pc;
    // Rank-3 spatial tensors (r3 != 0; template flag R3 of the kernel): an "image" of the fields above is a pair
    // (n, o) of a batch element and a slice of the depth lattice, N = batch * OD; the reduction runs over
    // (depth tap, 16-channel chunk) pairs.  Image (n, o) reads input slice o*is_d + dt_off[td] (zeros outside
    // [0, Din)) with filter slab dt_slab[td] + tap_slab[t], and is stored to slice o*os_d + oa_d of Dfull.
    int32_t r3, Din, Dfull, OD, is_d, os_d, oa_d, ndt;
    int32_t dt_off[STRIP_MAX_DT], dt_slab[STRIP_MAX_DT];
    FastDiv div_od;
    int32_t xcd_order;         // single launches: one-dimensional grid, the output-channel tiles of a strip on one XCD
    int32_t tail_fuse;         // blocked rank-2 output through the buffer descriptor: the last chunk runs fragment after
                               // fragment with each fragment's epilogue behind its taps
    int32_t frag_split;        // same path: a last fragment that only wave 0 would hold is shared by waves 0 and 1
    int32_t cps;               // chunks per LDS stage: 2 = two (rank 2, small strips), anything else = one
    // Column tiles (rows wider than a strip holds): a strip covers BW of the Wout lattice columns; `strips` counts
    // (row strip, column tile) pairs, column tile fastest; the geometry fields and divisors above are those of a
    // BW-wide lattice.  ncolt = 1: BW = Wout.
    int32_t ncolt, BW;
    FastDiv div_ncolt;
};

// ---- filter-resident strip kernel (stride-1 forward / backprop-data with a filter that fits the LDS) ----
struct RowsParams {
    const uint16_t *in;
    const uint16_t *wt;
    uint16_t *out;
    const float *bias;         // may be null
    const uint16_t *mask;      // may be null; else same shape / layout as out: out = (mask > 0) ? out : 0
    int32_t N, Cin, Hin, Win, Cout, Hout, Wout;
    int32_t TP, strips;        // output rows per workgroup, workgroups per image
    int32_t SRB;               // output rows per sub-strip (SRB * Wout <= 512 positions)
    int32_t PC;                // patch columns (Wout + window span in w)
    int32_t min_dh, min_dw, span_h;
    int32_t nblocks;           // 64-pixel blocks of the input patch of a full sub-strip
    int32_t xpitch;            // bytes per 8-channel plane of a stage buffer
    int32_t relu;
    int32_t ntaps;
    int32_t tap_off[STRIP_MAX_TAPS];    // patch-pixel offset of the tap
    int32_t tap_slab[STRIP_MAX_TAPS];   // filter slab (r * S + s) the tap reads
    uint32_t in_bytes, wt_bytes, out_bytes;
    int32_t late_mask;         // bit w: wave w issues the loads of a later stage after its MFMAs instead of before
    FastDiv div_q, div_pc;
};
constexpr int ROWS_NBUF = 3;             // stage buffers of the input patch (prefetch two stages ahead)
hipError_t launch_rows(const RowsParams &p, size_t lds_bytes, hipStream_t st);

// ---- MFMA backprop-filters ----
struct WgradParams {
    const uint16_t *x;         // blocked [N][C/16][H][W][16]
    const uint16_t *dy;        // blocked [N][K/16][P][Q][16]
    float *partial;            // [split][tap][K][C]
    int32_t N, C, H, W, K, P, Q, R, S;
    int32_t sh, sw, dh, dw, pbh, pbw;
    uint32_t M;                // N*P*Q
    uint32_t chunk;            // positions per split (multiple of 64)
    int32_t splits;
    FastDiv div_pq, div_q;
};

// ---- backprop-filters, all taps per pass (stride-1, 9 taps) ----
struct WgradStripParams {
    const uint16_t *x;         // blocked [N][C/16][H][W][16]
    const uint16_t *dy;        // blocked [N][K/16][P][Q][16]
    float *partial;            // [nparts][tap][K][C]
    float *dw;                 // [K][C][R][S]
    int32_t N, C, H, W, K, P, Q;
    int32_t NI;                // images per workgroup
    int32_t TP, strips;        // dy rows per workgroup, row strips per image
    int32_t SR, nstages;       // rows per LDS stage, stages per (image, strip)
    int32_t nparts;            // ceil(N/NI) * strips
    int32_t PRS, PC;           // x patch rows per stage, patch columns
    int32_t min_dh, min_dw;
    int32_t tap_off[9];        // patch-pixel offset of the tap
    int32_t dyplane, xplane;   // bytes per 16-channel plane of a stage
    int32_t ncq;               // 16-channel groups of c per workgroup (4, 2 or 1)
    int32_t nring;             // LDS stage buffers (2 or 3)
    int32_t G;                 // whole images per stage (small images; 1 = row blocks of one image)
    int32_t late_mask;         // bit w: wave w issues the loads of a later stage after its MFMAs instead of before
    int32_t ctiles;            // C / (16 * ncq)
    int32_t stream_partials;   // the partials leave with non-temporal stores
    uint32_t x_bytes, dy_bytes;
    FastDiv div_q, div_pc, div_pq, div_patch;
};

// ---- low-channel stem forward (C <= 3, 7x7 stride 2, NCHW in, blocked out) ----
struct StemFwdParams {
    const uint16_t *x;         // NCHW
    const uint16_t *w;         // KCRS
    const float *bias;         // may be null
    uint16_t *y;               // blocked
    int32_t N, C, H, W, K, P, Q;
    int32_t pbh;
    int32_t relu;
    int32_t TP, tiles_per_img;
    uint32_t y_bytes;          // bytes of y if below 2 GiB (stores then take 32-bit offsets into a buffer descriptor), else 0
    FastDiv div_q;
    FastDiv div_cpr, div_rows; // patch loader: 16-byte chunks per input row (W / 8), input rows per channel (2 TP + 5)
};

// ---- low-channel stem backprop-filters ----
struct WgradStemParams {
    const uint16_t *x;         // NCHW
    const uint16_t *dy;        // blocked
    float *partial;
    float *dw;                 // [K][C][7][7]
    int32_t N, C, H, W, K, P, Q;
    int32_t pbh;
    int32_t TP, strips;        // dy rows per workgroup (multiple of SR), strips per image
    int32_t SR;                // dy rows per LDS stage (SR*Q multiple of 32)
    int32_t dyplane;           // bytes per 16-channel dy plane of a stage
    uint32_t dy_bytes, x_bytes;
    int32_t ring;              // three stage buffers + staging area for the raw input rows (else two buffers)
    int32_t PL, RPX;           // LDS bytes per parity plane of an input row (>= W + 16) and per row (>= 2 PL)
    FastDiv div_q;
};

// ---- backprop-filters as a GEMM over positions, one tap per workgroup ----
struct WgradGemmParams {
    const uint16_t *x;
    const uint16_t *dy;
    float *partial;            // [part][tap][tile][sub][kb][cq][lane][4]
    float *dw;                 // [K][C][R][S]
    int32_t N, C, H, W, K, P, Q, R, S;
    int32_t sh, sw, dil_h, dil_w, pbh, pbw;
    int32_t wk, wc;            // 64-wide sub-tiles of k and c per workgroup
    int32_t sp;                // positions per LDS stage (128 or 64)
    int32_t x_nchw, dy_nchw;   // operand read from an NCHW tensor (1x1, stride 1, no padding, H*W % 8 == 0)
    int32_t ktiles, ctiles;    // tiles of 64 wk output and 64 wc input channels (the last of each may be partial)
    int32_t nparts;
    uint32_t M, chunk;         // N*P*Q, positions per part (multiple of 128)
    uint32_t x_bytes, dy_bytes;
    FastDiv div_pq, div_q;
    // rank-3 spatial tensors (r3 != 0): x [N][C/16][D][H][W][16], dy [N][K/16][O][P][Q][16], dw [K][C][T][R][S],
    // M = N*O*P*Q, taps = T*R*S
    int32_t r3, D, O, T, sd, dil_d, pbd;
    FastDiv div_opq;           // divide by O*P*Q
    int32_t xcd_order;         // rank 2, blocked operands: one-dimensional grid with the workgroups of a position chunk on one XCD
};

// ---- both derivative ops of a 1x1 stride-1 node in one pass over dy ----
struct Bwd1x1FusedParams {
    const uint16_t *x;         // blocked [N][C/16][HW][16]
    const uint16_t *dy;        // blocked [N][K/16][HW][16]
    const uint16_t *w;         // [K/16][C][16]: the backprop-data filter layout
    uint16_t *dx;              // blocked, same shape as x
    float *partial;            // [part][K][C]
    float *dw;                 // [K][C]
    int32_t N, C, K, HW;
    uint32_t M;                // N * HW positions
    int32_t nstages;           // stages of 64 positions
    int32_t stages_per_part, nparts;
    int32_t relu_mask;         // dx = (x > 0) ? dx : 0
    uint32_t x_bytes, dy_bytes;
    FastDiv div_hw;
};
hipError_t launch_bwd1x1_fused(const Bwd1x1FusedParams &p, hipStream_t st);

// ---- one-tap (1x1) forward / backprop-data as a pipelined GEMM ----
struct Gemm1x1Params {
    const uint16_t *in;
    const uint16_t *wt;        // [Cin/16][Cout][16]
    uint16_t *out;
    const float *bias;         // may be null
    const uint16_t *mask;      // may be null; else same shape / layout as out: out = (mask > 0) ? out : 0
    int32_t Cin, Hin, Win, Cout, Hout, Wout;
    float *dbp;                        // may be null; else [rows][dbp_ld] fp32: channel sums of what each workgroup stored
    int32_t dbp_row0, dbp_ld;          // row of m-tile t: dbp_row0 + t; row pitch in floats
    int32_t in_nchw, out_nchw;         // activations read from / result written to NCHW (stride 1, no padding, H*W % 8 == 0)
    int32_t is_h, is_w, dh, dw;        // input pixel of lattice position (i,j): (i*is_h + dh, j*is_w + dw)
    int32_t os_h, os_w, oa_h, oa_w;    // output pixel: (i*os_h + oa_h, j*os_w + oa_w)
    int32_t relu;
    int32_t zero_sib;          // also store zeros to the other pixels of the position's os_h x os_w block (oa = 0)
    uint32_t M;                // N * OP * OQ lattice positions
    uint32_t in_bytes, wt_bytes;
    uint32_t out_bytes;        // blocked result: bytes of the stored tensor if below 2 GiB (stores then take 32-bit offsets
                               // into a buffer descriptor), else 0
    FastDiv div_pq, div_q;
};

// Direct global->LDS load of 16 bytes per lane (lane l lands at lds_dst + 16 l, lanes whose offset is out of range
// deliver zeros), written as an instruction sequence the compiler does not interpret.  With the builtin form the
// compiler knows that an LDS write is in flight and makes every later LDS read of the wave it cannot tell apart from
// it (the transpose loads, for one) wait for vmcnt(0), i.e. for every stage the wave has prefetched: a ring of
// stage buffers then runs as a single buffer.  Callers order their accesses themselves, as they do anyway:
// wait_vmcnt(n) for the stage about to be read, then the workgroup barrier.
// rsrc: buffer descriptor words {base[31:0], base[47:32], bytes, 0x00020000}.
typedef unsigned ngc_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ ngc_u32x4 make_rsrc_words(const void *base, unsigned bytes)
{
    const unsigned long long b = reinterpret_cast<unsigned long long>(base);
    ngc_u32x4 r = {(unsigned)b, (unsigned)(b >> 32) & 0xFFFFu, bytes, 0x00020000u};
    return r;
}
__device__ __forceinline__ void dma_load_lds16(ngc_u32x4 rsrc, const void *lds_dst_uniform, unsigned voff, unsigned soff)
{
    typedef __attribute__((address_space(3))) const void lds_cvoid;
    const unsigned m0v = (unsigned)reinterpret_cast<unsigned long long>((lds_cvoid *)lds_dst_uniform) ;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(m0v), "v"(voff), "s"(rsrc), "s"(soff)
                 : "memory", "m0");
}

// Workgroup barrier without the memory fence of __syncthreads().  The fence waits for every
// outstanding global->LDS load of the wave (s_waitcnt vmcnt(0)), which would serialise a
// multi-stage prefetch ring.  Callers order their LDS traffic themselves: s_waitcnt vmcnt(n) for
// the stage they are about to read before the barrier (and lgkmcnt(0) if they have LDS writes
// pending); LDS reads of a buffer have returned to registers before the wave reaches the barrier
// after which that buffer is refilled.
__device__ __forceinline__ void wg_barrier_nofence()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// launchers (each returns launch_result() after the launch)
hipError_t launch_gemm1x1(const Gemm1x1Params &p, hipStream_t st);
hipError_t launch_zero_fill(void *dst, size_t bytes, hipStream_t st);
hipError_t launch_igemm(const IgemmParams &p, int bn, uint32_t max_m, hipStream_t st);
hipError_t launch_igemm3(const IgemmParams &p, int bn, uint32_t max_m, hipStream_t st);    // rank-3 spatial
hipError_t launch_strip(const StripParams &p, int nf, size_t lds_bytes, hipStream_t st);

// up to 4 launches of the strip kernel (blocked output, same Cout) in one grid
constexpr int STRIP_MULTI_MAX = 4;
struct StripMulti {
    int32_t n;
    int32_t wg_end[STRIP_MULTI_MAX];   // prefix sums of groups * strips
    StripParams c[STRIP_MULTI_MAX];
};
static_assert(sizeof(StripMulti) <= 4096, "kernel arguments are passed by value: at most 4 KB");
hipError_t launch_strip_multi(const StripMulti &mp, int nf, size_t lds_bytes, hipStream_t st);
// plan of the strip kernel for forward (op 0) or residue class (ca, cb) of backprop-data (op 1) of a rank-2
// node (csrc/api.hip); false if the kernel does not take it, *empty if the class has nothing to launch
bool strip_plan_for_class(const ngc_conv_desc *d, int op, int ca, int cb, int P, int Q, StripParams *sp, int *nf_out,
                          size_t *lds_out, bool *empty);
hipError_t launch_stem_fwd(const StemFwdParams &p, size_t lds_bytes, hipStream_t st);
hipError_t launch_wgrad_stem(const WgradStemParams &p, size_t lds_bytes, hipStream_t st);
hipError_t launch_wgrad_gemm(const WgradGemmParams &p, hipStream_t st);
hipError_t launch_wgrad(const WgradParams &p, hipStream_t st);
hipError_t launch_wgrad_strip(const WgradStripParams &p, size_t lds_bytes, hipStream_t st);
hipError_t launch_wgrad_reduce(const float *partial, float *dw, int splits, int K, int C, int R, int S,
                               hipStream_t st);
hipError_t launch_direct_fwd(const ngc_conv_desc &d, int P, int Q, const void *x, const void *w,
                             const float *bias, void *y, hipStream_t st);
hipError_t launch_direct_bwd_data(const ngc_conv_desc &d, int P, int Q, const void *dy, const void *w,
                                  const void *mask, void *dx, hipStream_t st);
hipError_t launch_direct3_fwd(const ngc_conv3d_desc &d, int O, int P, int Q, const void *x, const void *w, const float *bias,
                              void *y, hipStream_t st);
hipError_t launch_direct3_bwd_data(const ngc_conv3d_desc &d, int O, int P, int Q, const void *dy, const void *w, const void *mask,
                                   void *dx, hipStream_t st);
hipError_t launch_direct3_bwd_filters(const ngc_conv3d_desc &d, int O, int P, int Q, const void *x, const void *dy, float *dw,
                                      hipStream_t st);
int gemm1x1_dbp_tile_m(const Gemm1x1Params &p);
int softmax_vectors(int dtype, int cols, bool bwd, bool aligned);
hipError_t launch_softmax(int dtype, bool bwd, const void *a, const void *b, void *out, uint32_t rows, int cols, int V,
                          hipStream_t st);
hipError_t launch_bias_grad(const ngc_conv_desc &d, int P, int Q, const void *dy, float *db, float *partial, int nparts,
                            hipStream_t st);
int bias_grad_parts(const ngc_conv_desc &d, int P, int Q);
hipError_t launch_bias_grad_reduce(const float *partial, float *db, int nparts, int K, int KP, hipStream_t st);
hipError_t launch_direct_bwd_filters(const ngc_conv_desc &d, int P, int Q, const void *x, const void *dy,
                                     float *dw, hipStream_t st);
hipError_t launch_layout_convert(int elem_bytes, int n, int c, int h, int w, const void *src, int src_layout,
                                 void *dst, int dst_layout, hipStream_t st);
hipError_t launch_subpixel_filter(int K, int C, int R, int S, int pbh, int pbw, int dr_min, int ndr, int ds_min, int nds,
                                  int BH, int BW, int sh, int sw, const uint16_t *w_kcrs, uint16_t *wu, hipStream_t st);
hipError_t launch_filter_convert(int elem_bytes, int K, int C, int R, int S, const void *w_kcrs, void *dst,
                                 int dst_layout, hipStream_t st);

}  // namespace ngc
