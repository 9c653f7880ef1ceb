// pack / unpack kernels (Algorithm 1: the operand of the average, and writing the average back).
#include "ddp_device.h"

namespace ddp {
namespace {

// Elements [4 - d .. 7 - d] of the 8-element window (a, b): the 4 source elements that start d elements after a.
__device__ __forceinline__ f32x4 window(f32x4 a, f32x4 b, int d) {
    switch (d) {
        case 1: return f32x4{a.y, a.z, a.w, b.x};
        case 2: return f32x4{a.z, a.w, b.x, b.y};
        case 3: return f32x4{a.w, b.x, b.y, b.z};
        default: return a;
    }
}

// UNPACK = false: flat[flat_begin + i] = sync[t_begin + i]           (Algorithm 1: operand of the average)
// UNPACK = true : sync[t_begin + i] = flat[flat_begin + i], and the bf16 model copy = RNE of the same value.
// Stores are always 16-byte aligned.  When source and destination differ in their offset within a 16-byte
// granule, each lane loads the two aligned source granules that cover its 4 elements (the second is the next
// lane's first: it comes from the cache, not from HBM) and picks its window.  Every granule that is loaded
// holds at least one element of the chunk, so no access leaves the allocation's pages.
template <bool UNPACK, bool MODEL, bool NT>
__global__ __launch_bounds__(kThreads) void copy_kernel(const TensorDesc *__restrict__ tensors, const CopyChunk *__restrict__ chunks,
                                                        float *__restrict__ flat) {
    const CopyChunk ch = chunks[blockIdx.x];
    const TensorDesc td = tensors[ch.tensor];
    float *tptr = td.sync + ch.t_begin;
    float *fptr = flat + ch.flat_begin;
    const float *src = UNPACK ? fptr : tptr;
    float *dst = UNPACK ? tptr : fptr;
    unsigned short *mdl = MODEL ? td.model + ch.t_begin : reinterpret_cast<unsigned short *>(dst);  // unused without MODEL
    const int n = ch.count;
    const int tid = threadIdx.x;

    const int h = head_to_16B(dst, n);
    if (tid < h) {
        float v = src[tid];
        dst[tid] = v;
        if constexpr (MODEL) mdl[tid] = bf16_rne(v);
    }
    const int nv = (n - h) >> 2;
    const int tail0 = h + 4 * nv;
    if (tid < n - tail0) {
        float v = src[tail0 + tid];
        dst[tail0 + tid] = v;
        if constexpr (MODEL) mdl[tail0 + tid] = bf16_rne(v);
    }
    if (nv == 0) return;

    f32x4 *d4 = reinterpret_cast<f32x4 *>(dst + h);
    const int delta = (int)((reinterpret_cast<uintptr_t>(src + h) >> 2) & 3u);
    const bool mdl_vec = MODEL && ((reinterpret_cast<uintptr_t>(mdl + h) & 7u) == 0);
    u16x4 *m4 = reinterpret_cast<u16x4 *>(mdl + h);

    auto put = [&](int v, f32x4 val) {
        st<NT>(d4 + v, val);
        if constexpr (MODEL) {
            u16x4 b = bf16_rne4(val);
            if (mdl_vec) {
                st<NT>(m4 + v, b);
            } else {
                unsigned short *m = mdl + h + 4 * v;
                m[0] = b.x;
                m[1] = b.y;
                m[2] = b.z;
                m[3] = b.w;
            }
        }
    };

    if (delta == 0) {
        const f32x4 *s4 = reinterpret_cast<const f32x4 *>(src + h);
        int v = tid;
        for (; v + 3 * kThreads < nv; v += 4 * kThreads) {
            f32x4 a0 = ld<NT>(s4 + v);
            f32x4 a1 = ld<NT>(s4 + v + kThreads);
            f32x4 a2 = ld<NT>(s4 + v + 2 * kThreads);
            f32x4 a3 = ld<NT>(s4 + v + 3 * kThreads);
            put(v, a0);
            put(v + kThreads, a1);
            put(v + 2 * kThreads, a2);
            put(v + 3 * kThreads, a3);
        }
        for (; v < nv; v += kThreads) put(v, ld<NT>(s4 + v));
    } else {
        // aligned granule that holds the first source element of the body
        const f32x4 *s4 = reinterpret_cast<const f32x4 *>(src + h - delta);
        // the last vector's second granule would start past the chunk's last element only if it held none of
        // the 4 wanted elements, which cannot happen for delta != 0
        int v = tid;
        for (; v + kThreads < nv; v += 2 * kThreads) {
            f32x4 a0 = s4[v], b0 = s4[v + 1];
            f32x4 a1 = s4[v + kThreads], b1 = s4[v + kThreads + 1];
            put(v, window(a0, b0, delta));
            put(v + kThreads, window(a1, b1, delta));
        }
        for (; v < nv; v += kThreads) put(v, window(s4[v], s4[v + 1], delta));
    }
}

// Pack for a bf16 wire: flat16[flat_begin + i] = bf16_rne(sync[t_begin + i]).  Stores are 8-byte aligned groups of
// four; the source side uses the same two-granule window as copy_kernel when its alignment differs.
template <bool NT>
__global__ __launch_bounds__(kThreads) void pack16_kernel(const TensorDesc *__restrict__ tensors, const CopyChunk *__restrict__ chunks,
                                                          unsigned short *__restrict__ flat16) {
    const CopyChunk ch = chunks[blockIdx.x];
    const TensorDesc td = tensors[ch.tensor];
    const float *src = td.sync + ch.t_begin;
    unsigned short *dst = flat16 + ch.flat_begin;
    const int n = ch.count;
    const int tid = threadIdx.x;
    int h = (int)((4 - (ch.flat_begin & 3)) & 3);  // the flat buffer is 16-byte aligned at element 0
    if (h > n) h = n;
    if (tid < h) dst[tid] = bf16_rne(src[tid]);
    const int nv = (n - h) >> 2;
    const int tail0 = h + 4 * nv;
    if (tid < n - tail0) dst[tail0 + tid] = bf16_rne(src[tail0 + tid]);
    if (nv == 0) return;
    u16x4 *d4 = reinterpret_cast<u16x4 *>(dst + h);
    const int delta = (int)((reinterpret_cast<uintptr_t>(src + h) >> 2) & 3u);
    if (delta == 0) {
        const f32x4 *s4 = reinterpret_cast<const f32x4 *>(src + h);
        for (int v = tid; v < nv; v += kThreads) st<NT>(d4 + v, bf16_rne4(ld<NT>(s4 + v)));
    } else {
        const f32x4 *s4 = reinterpret_cast<const f32x4 *>(src + h - delta);
        for (int v = tid; v < nv; v += kThreads) st<NT>(d4 + v, bf16_rne4(window(s4[v], s4[v + 1], delta)));
    }
}

}  // namespace

int launch_copy(bool unpack, const TensorDesc *tensors, const CopyChunk *chunks, int64_t n_chunks, float *flat, bool with_model,
                bool nontemporal, int lds_pad, void *stream) {
    if (!unpack) return nontemporal ? launch(copy_kernel<false, false, true>, n_chunks, stream, lds_pad, tensors, chunks, flat)
                                    : launch(copy_kernel<false, false, false>, n_chunks, stream, lds_pad, tensors, chunks, flat);
    if (with_model) return nontemporal ? launch(copy_kernel<true, true, true>, n_chunks, stream, lds_pad, tensors, chunks, flat)
                                       : launch(copy_kernel<true, true, false>, n_chunks, stream, lds_pad, tensors, chunks, flat);
    return nontemporal ? launch(copy_kernel<true, false, true>, n_chunks, stream, lds_pad, tensors, chunks, flat)
                       : launch(copy_kernel<true, false, false>, n_chunks, stream, lds_pad, tensors, chunks, flat);
}

int launch_pack16(const TensorDesc *tensors, const CopyChunk *chunks, int64_t n_chunks, uint16_t *flat16, bool nontemporal, int lds_pad,
                  void *stream) {
    return nontemporal ? launch(pack16_kernel<true>, n_chunks, stream, lds_pad, tensors, chunks, flat16)
                       : launch(pack16_kernel<false>, n_chunks, stream, lds_pad, tensors, chunks, flat16);
}

}  // namespace ddp
