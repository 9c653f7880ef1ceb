// ddp_stream_probe: a measurement aid.  One kernel in the launch shape of the library's streaming kernels (256-thread
// workgroups, one chunk per workgroup, buffer accesses with the streaming hint, optional unused-LDS residency cap) that
// does nothing but read R streams and write W streams.  Timing it tells what the memory system gives a kernel with that
// mix of streams: the practical ceiling the averaging kernel (N reads : 1 write) and the update kernel (4 reads : 4
// writes) are compared with.
#include "ddp_device.h"

namespace ddp {
namespace {

struct ProbeArgs {
    const void *rd[16];
    void *wr[4];
    int64_t bytes;    // per stream, a multiple of 16
    int chunk_bytes;  // per workgroup and stream, a multiple of 4096
};

template <int NR, int NW>
__global__ __launch_bounds__(kThreads) void probe_kernel(const ProbeArgs a) {
    constexpr int AUX = 2;  // nt
    const int64_t b0 = (int64_t)blockIdx.x * a.chunk_bytes;
    const int64_t left = a.bytes - b0;
    const int nb = left < (int64_t)a.chunk_bytes ? (int)left : a.chunk_bytes;
    const int nv = nb >> 4;
    __amdgpu_buffer_rsrc_t rr[NR > 0 ? NR : 1], rw[NW > 0 ? NW : 1];
#pragma unroll
    for (int k = 0; k < NR; ++k) rr[k] = make_rsrc(static_cast<const char *>(a.rd[k]) + b0, nb);
#pragma unroll
    for (int k = 0; k < NW; ++k) rw[k] = make_rsrc(static_cast<char *>(a.wr[k]) + b0, nb);
    f32x4 keep{0.0f, 0.0f, 0.0f, 0.0f};
    for (int v = threadIdx.x; v < nv; v += 2 * kThreads) {  // two vectors per thread and stream in flight, like the real kernels
        const int w = v + kThreads;
        f32x4 x0[NR > 0 ? NR : 1], x1[NR > 0 ? NR : 1];
#pragma unroll
        for (int k = 0; k < NR; ++k) {
            x0[k] = bld<AUX, f32x4>(rr[k], v * 16);
            x1[k] = bld<AUX, f32x4>(rr[k], w * 16);  // past the extent: reads zero
        }
        f32x4 s0{1.0f, 1.0f, 1.0f, 1.0f}, s1 = s0;
#pragma unroll
        for (int k = 0; k < NR; ++k) {
            s0 = s0 + x0[k];
            s1 = s1 + x1[k];
        }
#pragma unroll
        for (int k = 0; k < NW; ++k) {
            bst<AUX>(rw[k], v * 16, s0);
            bst<AUX>(rw[k], w * 16, s1);  // past the extent: dropped
        }
        if constexpr (NW == 0) keep = keep + s0 + s1;
    }
    if constexpr (NW == 0) {
        // a read-only probe has no result to store: hand the accumulated sum to an empty asm statement so that the loads
        // that feed it cannot be removed
        asm volatile("" : : "v"(keep.x), "v"(keep.y), "v"(keep.z), "v"(keep.w));
    }
}

template <int NR>
int launch_probe_w(int nw, const ProbeArgs &a, int64_t grid, int lds_pad, void *stream) {
    switch (nw) {
        case 0:
            if constexpr (NR > 0) return launch(probe_kernel<NR, 0>, grid, stream, lds_pad, a);
            return (int)hipErrorInvalidValue;
        case 1: return launch(probe_kernel<NR, 1>, grid, stream, lds_pad, a);
        case 2: return launch(probe_kernel<NR, 2>, grid, stream, lds_pad, a);
        case 3: return launch(probe_kernel<NR, 3>, grid, stream, lds_pad, a);
        case 4: return launch(probe_kernel<NR, 4>, grid, stream, lds_pad, a);
        default: return (int)hipErrorInvalidValue;
    }
}

}  // namespace
}  // namespace ddp

extern "C" int ddp_stream_probe(int n_read, int n_write, int64_t bytes, const void *const *read_ptrs, void *const *write_ptrs,
                                int chunk_bytes, int lds_pad, void *stream) {
    using namespace ddp;
    return guarded(nullptr, [&]() -> int {
        const bool nr_ok = n_read == 0 || n_read == 1 || n_read == 2 || n_read == 3 || n_read == 4 || n_read == 8 || n_read == 16;
        if (!nr_ok || n_write < 0 || n_write > 4 || n_read + n_write == 0)
            return fail(nullptr, DDP_EINVAL, "ddp_stream_probe: n_read must be one of 0, 1, 2, 3, 4, 8, 16 and n_write in [0, 4], not both 0");
        if (bytes <= 0 || bytes % 16 != 0) return fail(nullptr, DDP_EINVAL, "ddp_stream_probe: bytes must be a positive multiple of 16");
        if (chunk_bytes < 4096 || chunk_bytes > (1 << 22) || chunk_bytes % 4096 != 0)
            return fail(nullptr, DDP_EINVAL, "ddp_stream_probe: chunk_bytes must be a multiple of 4096 in [4096, 4194304]");
        if (lds_pad < 0 || lds_pad > 65536) return fail(nullptr, DDP_EINVAL, "ddp_stream_probe: lds_pad must be in [0, 65536]");
        if ((n_read > 0 && !read_ptrs) || (n_write > 0 && !write_ptrs)) return fail(nullptr, DDP_EINVAL, "ddp_stream_probe: NULL pointer array");
        ProbeArgs a{};
        for (int k = 0; k < n_read; ++k) {
            if (!read_ptrs[k] || (reinterpret_cast<uintptr_t>(read_ptrs[k]) & 15u)) return fail(nullptr, DDP_EALIGN, "ddp_stream_probe: read stream NULL or not 16-byte aligned");
            a.rd[k] = read_ptrs[k];
        }
        for (int k = 0; k < n_write; ++k) {
            if (!write_ptrs[k] || (reinterpret_cast<uintptr_t>(write_ptrs[k]) & 15u)) return fail(nullptr, DDP_EALIGN, "ddp_stream_probe: write stream NULL or not 16-byte aligned");
            a.wr[k] = write_ptrs[k];
        }
        a.bytes = bytes;
        a.chunk_bytes = chunk_bytes;
        const int64_t grid = (bytes + chunk_bytes - 1) / chunk_bytes;
        int rc;
        switch (n_read) {
            case 0: rc = launch_probe_w<0>(n_write, a, grid, lds_pad, stream); break;
            case 1: rc = launch_probe_w<1>(n_write, a, grid, lds_pad, stream); break;
            case 2: rc = launch_probe_w<2>(n_write, a, grid, lds_pad, stream); break;
            case 3: rc = launch_probe_w<3>(n_write, a, grid, lds_pad, stream); break;
            case 4: rc = launch_probe_w<4>(n_write, a, grid, lds_pad, stream); break;
            case 8: rc = launch_probe_w<8>(n_write, a, grid, lds_pad, stream); break;
            default: rc = launch_probe_w<16>(n_write, a, grid, lds_pad, stream); break;
        }
        if (rc != 0) return fail(nullptr, DDP_EHIP, std::string("ddp_stream_probe: kernel launch failed: ") + hipGetErrorString((hipError_t)rc));
        return DDP_OK;
    });
}
