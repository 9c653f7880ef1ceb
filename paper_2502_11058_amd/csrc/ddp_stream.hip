// Streams restricted to a subset of the GPU's compute units, for running the synchronisation + update of a layer beside
// the backward pass of the layers below it (Sec. 3.2 of the paper) without the two fighting for the same CUs.
#include <hip/hip_runtime.h>

#include <string>
#include <vector>

#include "ddp_internal.h"

extern "C" int ddp_device_cu_count(int device, int *out_cus) {
    using namespace ddp;
    return guarded(nullptr, [&]() -> int {
        if (!out_cus) return fail(nullptr, DDP_EINVAL, "ddp_device_cu_count: out_cus is NULL");
        hipDeviceProp_t prop;
        hipError_t e = hipGetDeviceProperties(&prop, device);
        if (e != hipSuccess) return fail(nullptr, DDP_EHIP, std::string("ddp_device_cu_count: ") + hipGetErrorString(e));
        *out_cus = prop.multiProcessorCount;
        return DDP_OK;
    });
}

extern "C" int ddp_stream_create_cu_range(int device, int cu_first, int cu_count, void **out_stream) {
    using namespace ddp;
    return guarded(nullptr, [&]() -> int {
        if (!out_stream) return fail(nullptr, DDP_EINVAL, "ddp_stream_create_cu_range: out_stream is NULL");
        *out_stream = nullptr;
        int cur = -1;
        hipError_t e = hipGetDevice(&cur);
        if (e != hipSuccess) return fail(nullptr, DDP_EHIP, std::string("ddp_stream_create_cu_range: hipGetDevice: ") + hipGetErrorString(e));
        if (cur != device) return fail(nullptr, DDP_ESTATE, "ddp_stream_create_cu_range: `device` must be the current device");
        hipDeviceProp_t prop;
        e = hipGetDeviceProperties(&prop, device);
        if (e != hipSuccess) return fail(nullptr, DDP_EHIP, std::string("ddp_stream_create_cu_range: ") + hipGetErrorString(e));
        const int n = prop.multiProcessorCount;
        if (cu_first < 0 || cu_count < 1 || cu_first > n || cu_count > n - cu_first)
            return fail(nullptr, DDP_EINVAL, "ddp_stream_create_cu_range: range outside the device's " + std::to_string(n) + " compute units");
        std::vector<uint32_t> mask((size_t)(n + 31) / 32, 0u);
        for (int i = cu_first; i < cu_first + cu_count; ++i) mask[(size_t)i / 32] |= 1u << (i % 32);
        hipStream_t s = nullptr;
        e = hipExtStreamCreateWithCUMask(&s, (uint32_t)mask.size(), mask.data());  // default priority, like every stream here
        if (e != hipSuccess) return fail(nullptr, DDP_EHIP, std::string("ddp_stream_create_cu_range: hipExtStreamCreateWithCUMask: ") + hipGetErrorString(e));
        *out_stream = s;
        return DDP_OK;
    });
}

extern "C" int ddp_stream_destroy(void *stream) {
    using namespace ddp;
    return guarded(nullptr, [&]() -> int {
        if (!stream) return DDP_OK;
        hipError_t e = hipStreamDestroy((hipStream_t)stream);
        if (e != hipSuccess) return fail(nullptr, DDP_EHIP, std::string("ddp_stream_destroy: ") + hipGetErrorString(e));
        return DDP_OK;
    });
}
