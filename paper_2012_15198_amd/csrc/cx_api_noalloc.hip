// C-ABI entry point cx_gossip_mix_noalloc: cx_gossip_mix for callers that cannot allocate (see
// include/cx_mix.h).  Its only scratch -- the row-order table that order_kernel writes and
// gather_kernel reads -- is a file-scope device array of a fixed size; the kernels receive its
// device address as an argument.
#include "cx_launch.hpp"

namespace {

// One table per GPU, held until the process ends.  Nothing in it has to start at zero: a call
// rewrites every word it later reads (one word per cluster and row of its own geometry) and
// reads no other, so the leftovers of an earlier, larger call are never looked at.
static __device__ __align__(256) unsigned scratch[CX_NOALLOC_ORDER_WORDS];

// In host code `scratch` is only a handle for the runtime: the array's device address comes from
// hipGetSymbolAddress, asked once per device with that device current, and kept.
unsigned *scratch_on_current_device()
{
    static std::mutex mu;
    static unsigned *ptr[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return nullptr; }
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return nullptr; }
        ptr[dev] = static_cast<unsigned *>(p);
    }
    return ptr[dev];
}

}  // namespace

extern "C" {

int cx_gossip_mix_noalloc(const float *x_in, float *x_out, int64_t ld, int32_t W, int64_t P, int32_t S,
                          const int64_t *seg_off_dev, const int32_t *peers_dev, uint32_t flags,
                          void *stream)
{
    if (!seg_off_dev || !peers_dev) return CX_ERR_NULL;
    if (W < 2 || W > CX_MAX_ROWS) return (!x_in || !x_out) ? CX_ERR_NULL : CX_ERR_SHAPE;
    const int rc = check_matrix_args(x_in, x_out, ld, W, P, S, flags);
    if (rc != CX_OK) return rc;
    if (x_in == x_out) return CX_ERR_ALIAS;          // the in-place kernel has no scratch to place
    const MeanOp<1> op{x_in, x_out, ld};
    MixArgs a{W, P, S, seg_off_dev, peers_dev, 0, 0, static_cast<hipStream_t>(stream), true, 1};
    a.order_provider = scratch_on_current_device;
    a.order_entries = CX_NOALLOC_ORDER_WORDS;
    return launch_mix<MeanOp<1>>(op, a);
}

}  // extern "C"
