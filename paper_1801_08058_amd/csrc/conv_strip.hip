// Rank-2 instantiations and launchers of the strip convolution kernels (see conv_strip_kernels.h).
#include "conv_strip_kernels.h"

namespace ngc {

#ifdef NGC_TIMELINE
extern "C" int ngc_debug_strip_timeline(unsigned *host_dst, size_t count)
{
    return (int)hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(g_strip_timeline), count * sizeof(unsigned));
}
#endif

template <int NF, int NW, int SUB = 0>
static hipError_t launch_strip_nf(const StripParams &p, size_t lds_bytes, hipStream_t st)
{
    if constexpr (SUB == 0 && NW == 8) {
        if (p.ncolt > 1 && p.dbp) return hipErrorInvalidValue;
        if (p.ncolt > 1) return launch_strip_d<NF, NW, SUB, false, false, true>(p, lds_bytes, st);
        if (p.dbp) return launch_strip_d<NF, NW, SUB, true>(p, lds_bytes, st);
    }
    // column tiles exist for the blocked-output 8-wave kernels only
    if (p.r3 || p.ncolt > 1) return hipErrorInvalidValue;
    if (p.dbp) return hipErrorInvalidValue;          // channel sums exist for the blocked-output 8-wave kernels only
    return launch_strip_d<NF, NW, SUB, false>(p, lds_bytes, st);
}

// nf = 32-position fragments per SIMD (7, 4 or 2); the fragments of a SIMD are spread over two
// waves so that one wave's LDS latency hides behind the other's MFMAs
hipError_t launch_strip(const StripParams &p_in, int nf, size_t lds_bytes, hipStream_t st)
{
    StripParams p = p_in;
    // several output-channel tiles: XCD-ordered grid, so that the tiles of a strip read its input through one L2
    // (strided forward layers of the ResNet-50 stack 58 -> 55 us, others 0-2 %; NGC_STRIP_XCD=0: two-dimensional grid)
    const char *xo = env_switch(SW_STRIP_XCD);
    const int gx = p.groups * p.strips;                  // strips per XCD must come out even: a multiple of 8, or many
    if (p.Cout > 64 && (gx % 8 == 0 || gx >= 64) && !(xo && atoi(xo) == 0)) p.xcd_order = 1;
    {
        const char *tf = env_switch(SW_STRIP_TAIL);      // NGC_STRIP_TAIL=0: epilogues behind the last chunk, not in it
        p.tail_fuse = (tf && atoi(tf) == 0) ? 0 : 1;
        const char *fs = env_switch(SW_STRIP_SPLIT);     // NGC_STRIP_SPLIT=0: the odd last fragment stays with wave 0
        p.frag_split = (fs && atoi(fs) == 0) ? 0 : 1;
    }
    // Small strips (two or four fragments per SIMD) of a launch that leaves no room for a second workgroup per compute
    // unit anyway take two chunks per LDS stage when that fits: half as many barriers (NGC_STRIP_CPS=1: never).
    {
        const char *fc = env_switch(SW_STRIP_CPS);
        const long wgs = (long)p.groups * p.strips * ((p.Cout + 63) / 64);
        p.cps = 1;
        if (!p.r3 && p.out_mode == 0 && nf <= 4 && (p.Cin >> 4) >= 4 && 2 * lds_bytes <= 160 * 1024 &&
            wgs <= 256 && !(fc && atoi(fc) == 1)) {
            p.cps = 2;
            lds_bytes *= 2;
        }
    }
    if (p.r3) {                                          // blocked output, two waves per SIMD; a code object of its own
        if (p.out_mode != 0) return hipErrorInvalidValue;
        return launch_strip_r3(p, nf, lds_bytes, st);
    }
    if (p.out_mode == 1 && p.half_cols) {
        switch (nf) {
        case 7: return launch_strip_nf<4, 8, 1>(p, lds_bytes, st);
        case 4: return launch_strip_nf<2, 8, 1>(p, lds_bytes, st);
        case 2: return launch_strip_nf<1, 8, 1>(p, lds_bytes, st);
        default: return hipErrorInvalidValue;
        }
    }
    if (p.out_mode == 1) {
        switch (nf) {
        case 7: return launch_strip_nf<4, 8, 2>(p, lds_bytes, st);
        case 4: return launch_strip_nf<2, 8, 2>(p, lds_bytes, st);
        case 2: return launch_strip_nf<1, 8, 2>(p, lds_bytes, st);
        default: return hipErrorInvalidValue;
        }
    }
    switch (nf) {
    case 7: return launch_strip_nf<4, 8>(p, lds_bytes, st);
    case 4: return launch_strip_nf<2, 8>(p, lds_bytes, st);
    case 2: return launch_strip_nf<1, 8>(p, lds_bytes, st);
    default: return hipErrorInvalidValue;
    }
}

// nf = the largest strip size (7, 4 or 2) among the launches, lds_bytes the largest stage buffers; blocked output
hipError_t launch_strip_multi(const StripMulti &mp, int nf, size_t lds_bytes, hipStream_t st)
{
    const bool db = mp.c[0].dbp != nullptr;
    for (int i = 0; i < mp.n; ++i)
        if (mp.c[i].ncolt > 1) return hipErrorInvalidValue;          // column tiles: single launches only
    if (mp.c[0].r3) {                                // all launches of a grid are of one rank
        if (db) return hipErrorInvalidValue;
        return launch_strip_multi_r3(mp, nf, lds_bytes, st);
    }
    switch (nf) {
    case 7: return db ? launch_strip_multi_t<4, true>(mp, lds_bytes, st) : launch_strip_multi_t<4, false>(mp, lds_bytes, st);
    case 4: return db ? launch_strip_multi_t<2, true>(mp, lds_bytes, st) : launch_strip_multi_t<2, false>(mp, lds_bytes, st);
    case 2: return db ? launch_strip_multi_t<1, true>(mp, lds_bytes, st) : launch_strip_multi_t<1, false>(mp, lds_bytes, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace ngc
