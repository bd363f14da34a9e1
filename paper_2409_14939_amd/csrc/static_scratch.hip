// fastgl_block_aggregate_fwd_static: the forward aggregation for callers that may
// not allocate device memory and have no workspace to pass (code under HIP graph
// capture, serving loops, harnesses that forbid hipMalloc).  Its scratch - the
// forward bookkeeping of the block and the partial sums of long rows, which
// fastgl_block_aggregate_fwd keeps in the caller's workspace - lives in a
// file-scope device array of fixed size.  Every GPU the library runs on holds its
// own copy of the array from the moment the code object is loaded until the
// process ends.
#include <mutex>

#include "internal.h"

namespace {

static __device__ __align__(256) unsigned char scratch[FASTGL_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, looked up once

// In host code the array's name is only a handle for the symbol lookup; the
// address kernels may use is the one hipGetSymbolAddress returns for the device
// that is current, and it differs from GPU to GPU.
fastgl_status scratch_of_current_device(void **out)
{
    int dev = -1;
    FASTGL_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) {
        fastgl::set_error("device ordinal %d is outside the supported range [0, %d)", dev, kMaxDevices);
        return FASTGL_ERR_UNSUPPORTED;
    }
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        FASTGL_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || ((uintptr_t)p & 255)) {
            fastgl::set_error("symbol lookup of the static scratch array gave an unusable address");
            return FASTGL_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return FASTGL_OK;
}

}  // namespace

extern "C" fastgl_status fastgl_block_aggregate_fwd_static(
    const int32_t *indptr, const int32_t *indices, const float *edge_w, int64_t num_dst, int64_t num_src,
    int64_t num_edges, int64_t feat, fastgl_agg_mode mode, fastgl_dtype dtype, const void *X, void *out,
    void *stream)
{
    // every host-side check first, so that a refused call touches neither the GPU nor the runtime
    size_t need = 0;
    fastgl_status st = fastgl::aggregate_check(false, indptr, indices, edge_w, num_dst, num_src, num_edges, feat,
                                               mode, dtype, X, out, nullptr, &need);
    if (st != FASTGL_OK) return st;
    if (need > (size_t)FASTGL_STATIC_SCRATCH_BYTES) {
        fastgl::set_error("block too large for the static scratch array: it needs %zu bytes, the array holds %zu",
                          need, (size_t)FASTGL_STATIC_SCRATCH_BYTES);
        return FASTGL_ERR_WORKSPACE;
    }
    void *ws = nullptr;
    st = scratch_of_current_device(&ws);
    if (st != FASTGL_OK) return st;
    // Same bookkeeping kernels and aggregation kernels as the entry point with a
    // workspace; they get the array's device address as their workspace.  Nothing
    // in the array has to start at zero: every counter, degree and partial sum is
    // written (by a kernel of this call) before it is read.
    return fastgl::aggregate_run(false, indptr, indices, edge_w, num_dst, num_src, num_edges, feat, mode, dtype, X,
                                 out, nullptr, ws, stream);
}
