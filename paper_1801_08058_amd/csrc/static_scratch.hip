// ConvolutionBackpropFilters for callers that cannot allocate: the split-reduction partials live in a
// file-scope device array instead of a caller-provided workspace.  Host code only (plus the array).
#include "common.h"

#include <mutex>
#include <stdio.h>

// Every GPU the library runs on holds its own copy of this array, at its own address, until the process ends.
static __device__ __align__(256) unsigned char scratch[NGC_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex g_lock;
void *g_ptr[MAX_DEVICES] = {};          // device address of `scratch` on device i (0 = not looked up yet)

// Device address of the array on the current device.  In host code the array's name is only a handle for the
// runtime; the address a kernel can use comes from hipGetSymbolAddress, once per device with that device current.
int scratch_address(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return NGC_LAUNCH_FAILED;
    std::lock_guard<std::mutex> g(g_lock);
    if (!g_ptr[dev]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            fprintf(stderr, "ngconv: hipGetSymbolAddress(scratch) failed on device %d: %s\n", dev, hipGetErrorString(e));
            return NGC_LAUNCH_FAILED;
        }
        g_ptr[dev] = p;
    }
    *out = g_ptr[dev];
    return NGC_OK;
}

}  // namespace

extern "C" {

size_t ngc_static_scratch_bytes(void) { return NGC_STATIC_SCRATCH_BYTES; }

int ngc_conv_bwd_filters_noalloc(const ngc_conv_desc *desc, const void *x, const void *dy, float *dw, void *hip_stream)
{
    int32_t P, Q;
    const int vs = ngc_conv_out_shape(desc, &P, &Q);
    if (vs != NGC_OK) return vs;
    if (!x || !dy || !dw) return NGC_BAD_ARG;
    // sizes beyond the array are refused before anything touches the GPU
    const size_t need = ngc_conv_workspace_bytes(desc, NGC_OP_BWD_FILTERS);
    if (need > NGC_STATIC_SCRATCH_BYTES) return NGC_SCRATCH_EXCEEDED;
    void *ptr = nullptr;
    const int rc = scratch_address(&ptr);
    if (rc != NGC_OK) return rc;
    // Same kernels as ngc_conv_bwd_filters, the array's device address in place of the workspace.  Every partial a
    // launch reads it has written before (nothing has to start at zero), so the contents the previous call left behind
    // do not matter; two calls in flight on one GPU at once would share the array and race.
    return ngc_conv_bwd_filters(desc, x, dy, dw, ptr, NGC_STATIC_SCRATCH_BYTES, hip_stream);
}

}  // extern "C"
