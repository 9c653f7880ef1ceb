// ddp_partial_average_static: the averaging entry point for callers that cannot allocate device memory.  Its
// reduction scratch (one pair of partial sums per chunk, then 64 slice sums per layer) is a fixed array in the
// library's device image instead of memory the context allocated.
#include <hip/hip_runtime.h>

#include <mutex>
#include <string>

#include "ddp_internal.h"

namespace {

// One copy per GPU the library runs on, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress: kernels and memsets get the device address resolved below, never the name.
static __device__ __align__(256) unsigned char scratch[DDP_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
double *g_scratch_ptr[kMaxDevices];  // per device: address of its copy of `scratch`, nullptr until resolved

}  // namespace

namespace ddp {

int static_scratch_for(const ddp_ctx *ctx, int device, double **ptr) {
    *ptr = nullptr;
    if (device < 0 || device >= kMaxDevices)
        return fail(ctx, DDP_EINVAL, "device ordinal " + std::to_string(device) + " is beyond the " + std::to_string(kMaxDevices) + " the library keeps scratch for");
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch_ptr[device]) {
        int cur = -1;
        hipError_t e = hipGetDevice(&cur);
        if (e != hipSuccess) return fail(ctx, DDP_EHIP, std::string("hipGetDevice: ") + hipGetErrorString(e));
        if (cur != device) return fail(ctx, DDP_ESTATE, "the fixed scratch of device " + std::to_string(device) + " must be resolved with that device current");
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(ctx, DDP_EHIP, std::string("hipGetSymbolAddress of the fixed scratch: ") + hipGetErrorString(e));
        g_scratch_ptr[device] = static_cast<double *>(p);
    }
    *ptr = g_scratch_ptr[device];
    return DDP_OK;
}

}  // namespace ddp

extern "C" int ddp_partial_average_static(ddp_ctx *ctx, int slot, const float *flat_local, const float *const *peers, int N,
                                          int local_rank, float *flat_out, double *layer_stats, void *stream) {
    return ddp::guarded(ctx, [&]() -> int {
        if (!ctx) return ddp::fail(nullptr, DDP_EINVAL, "ddp_partial_average_static: ctx is NULL");
        if (!ctx->static_scratch)
            return ddp::fail(ctx, DDP_ESTATE, "ddp_partial_average_static: the fixed scratch could not be resolved when the context was created: " + ctx->static_scratch_err);
        return ddp::partial_average_impl(ctx, "ddp_partial_average_static", false, slot, flat_local,
                                         reinterpret_cast<const void *const *>(peers), N, local_rank, flat_out, layer_stats, stream,
                                         ctx->static_scratch, (int64_t)DDP_STATIC_SCRATCH_BYTES);
    });
}
