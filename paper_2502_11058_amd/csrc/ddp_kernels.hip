// gfx950 kernels of the partial-synchronisation + local-update step (Algorithm 1 / Eq. (5) of the paper).
//
// All kernels are HBM streaming kernels (well under 1 flop per byte): no MFMA, no data reuse.  The design
// rules are the same everywhere:
//   - one workgroup (256 threads = 4 wavefronts of 64) per table entry ("chunk"), a run of elements inside one
//     tensor or one layer, so the ragged boundaries of tensors and layers are handled by the table, not by
//     per-element searches; where the registered tensors form dense arenas the update and the fused step need no
//     table at all (the *_dense_kernel variants: addresses from the block index, buffer accesses);
//   - inside a chunk: a scalar head of < 4 elements up to the next 16-byte boundary of the destination, a body
//     of 128-bit accesses (lane i of a wavefront touches bytes [16i, 16i+16) of a 1 KiB line, fully coalesced),
//     and a scalar tail of < 4 elements;
//   - several independent 128-bit loads are issued before the first use, to keep enough bytes in flight per CU;
//   - streaming (nontemporal) cache hints, since nothing is read twice;
//   - floating-point contraction is off: every product and sum below is its own IEEE fp32 operation, and
//     division and square root are the correctly rounded ones, so results do not depend on instruction selection.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "ddp_internal.h"

#pragma clang fp contract(off)

namespace ddp {
namespace {

constexpr int kThreads = 256;
constexpr int kWave = 64;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));

template <bool NT, class T>
__device__ __forceinline__ T ld(const T *p) {
    if constexpr (NT)
        return __builtin_nontemporal_load(p);
    else
        return *p;
}

template <bool NT, class T>
__device__ __forceinline__ void st(T *p, T v) {
    if constexpr (NT)
        __builtin_nontemporal_store(v, p);
    else
        *p = v;
}

// fp32 -> bf16, round to nearest, ties to even (add 0x7fff plus the lowest kept bit, then truncate); NaN -> quiet NaN.
__device__ __forceinline__ unsigned short bf16_rne(float f) {
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

__device__ __forceinline__ float bf16_widen(unsigned short h) { return __uint_as_float(((unsigned int)h) << 16); }

__device__ __forceinline__ u16x4 bf16_rne4(f32x4 v) {
    u16x4 r;
    r.x = bf16_rne(v.x);
    r.y = bf16_rne(v.y);
    r.z = bf16_rne(v.z);
    r.w = bf16_rne(v.w);
    return r;
}

__device__ __forceinline__ f32x4 bf16_widen4(u16x4 h) {
    return f32x4{bf16_widen(h.x), bf16_widen(h.y), bf16_widen(h.z), bf16_widen(h.w)};
}

// One replica's flat buffer as it arrives: fp32 (W16 = false) or bf16 bit patterns (W16 = true, widened exactly).
// Element index i, or index v of a group of 4 elements (16 bytes of fp32, 8 bytes of bf16).
template <bool W16>
__device__ __forceinline__ float wire1(const void *base, int64_t i) {
    if constexpr (W16)
        return bf16_widen(reinterpret_cast<const unsigned short *>(base)[i]);
    else
        return reinterpret_cast<const float *>(base)[i];
}
template <bool W16, bool NT>
__device__ __forceinline__ f32x4 wire4(const void *base, int64_t v) {
    if constexpr (W16)
        return bf16_widen4(ld<NT>(reinterpret_cast<const u16x4 *>(base) + v));
    else
        return ld<NT>(reinterpret_cast<const f32x4 *>(base) + v);
}

// Buffer (MUBUF) accesses: a per-workgroup descriptor (base in SGPRs, extent = the workgroup's part of the stream)
// plus a 32-bit byte offset per lane.  Accesses past the extent read zero / are dropped by the hardware.
// AUX: cache policy bits of the instruction (2 = nt, the streaming hint; 0 = default).
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, int bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);  // raw dword format
}

template <int AUX, class T>
__device__ __forceinline__ T bld(__amdgpu_buffer_rsrc_t r, int byte_off) {
    static_assert(sizeof(T) == 16 || sizeof(T) == 8, "128- or 64-bit access");
    if constexpr (sizeof(T) == 16)
        return __builtin_bit_cast(T, __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, AUX));
    else
        return __builtin_bit_cast(T, __builtin_amdgcn_raw_buffer_load_b64(r, byte_off, 0, AUX));
}

template <int AUX, class T>
__device__ __forceinline__ void bst(__amdgpu_buffer_rsrc_t r, int byte_off, T v) {
    static_assert(sizeof(T) == 16 || sizeof(T) == 8, "128- or 64-bit access");
    if constexpr (sizeof(T) == 16)
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, byte_off, 0, AUX);
    else
        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, v), r, byte_off, 0, AUX);
}

__device__ __forceinline__ int head_to_16B(const void *p, int n) {  // fp32 elements until p is 16-byte aligned
    int h = (int)((4u - (unsigned)((reinterpret_cast<uintptr_t>(p) >> 2) & 3u)) & 3u);
    return h < n ? h : n;
}

// ---------------------------------------------------------------------------------------------------------------
// pack / unpack
// ---------------------------------------------------------------------------------------------------------------

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

// ---------------------------------------------------------------------------------------------------------------
// partial average
// ---------------------------------------------------------------------------------------------------------------

struct MeanArgs {
    const void *x[DDP_MAX_REPLICAS];  // fp32 or bf16 flat buffers, rank order
    float *out;
    const MeanChunk *chunks;
    double *partials;
    float inv_n;
    int n;
};

// Sum of a double over the workgroup in a fixed order: butterfly-free shuffle-down tree inside each wavefront,
// then the four wavefront sums added in wavefront order by thread 0.  Result valid in thread 0.
__device__ __forceinline__ double block_sum(double v, double *lds) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_down(v, off, kWave);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    if (lane == 0) lds[wave] = v;
    __syncthreads();
    double r = 0.0;
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 0; w < kThreads / kWave; ++w) r += lds[w];
    }
    __syncthreads();
    return r;
}

// Eq. (5), second case.  NREP > 0: replica count known at compile time (pointer loads and the sum fully
// unrolled); NREP == 0: run-time count.  The sum runs left to right over replicas in rank order, in fp32, then
// one multiply by 1/N.  STATS adds, per chunk, sum_k sum_i (out_i - x_k,i)^2 and sum_i out_i^2 in fp64.
template <int NREP, bool STATS, bool NT, bool W16 = false>
__global__ __launch_bounds__(kThreads) void mean_kernel(const MeanArgs a) {
    __shared__ double lds[2][kThreads / kWave];
    const MeanChunk ch = a.chunks[blockIdx.x];
    const int n = ch.count;
    const int tid = threadIdx.x;
    const int nrep = NREP > 0 ? NREP : a.n;
    const float inv_n = a.inv_n;
    const int64_t base = ch.begin;
    double gsum = 0.0, msum = 0.0;

    auto one = [&](int64_t i) {
        float acc = wire1<W16>(a.x[0], i);
        for (int k = 1; k < nrep; ++k) acc = acc + wire1<W16>(a.x[k], i);
        const float m = acc * inv_n;
        if constexpr (STATS) {
            for (int k = 0; k < nrep; ++k) {
                const float d = m - wire1<W16>(a.x[k], i);
                gsum += (double)d * (double)d;
            }
            msum += (double)m * (double)m;
        }
        a.out[i] = m;
    };

    // all buffers are 16-byte aligned at element 0, so the flat index decides the alignment
    int h = (int)((4 - (base & 3)) & 3);
    if (h > n) h = n;
    if (tid < h) one(base + tid);
    const int nv = (n - h) >> 2;
    const int tail0 = h + 4 * nv;
    if (tid < n - tail0) one(base + tail0 + tid);

    const int64_t vbase = (base + h) >> 2;  // index in 16-byte units
    f32x4 *o4 = reinterpret_cast<f32x4 *>(a.out) + vbase;

    auto stats4 = [&](f32x4 m, f32x4 x) {
        const f32x4 d = m - x;
        gsum += (double)d.x * (double)d.x;
        gsum += (double)d.y * (double)d.y;
        gsum += (double)d.z * (double)d.z;
        gsum += (double)d.w * (double)d.w;
    };
    auto msq4 = [&](f32x4 m) {
        msum += (double)m.x * (double)m.x;
        msum += (double)m.y * (double)m.y;
        msum += (double)m.z * (double)m.z;
        msum += (double)m.w * (double)m.w;
    };

    if constexpr (NREP > 0) {
        constexpr int B = 2;  // vectors per thread in flight: 2 * NREP loads (a 2048-element chunk is 2 vectors per thread)
        auto rep4 = [&](int k, int idx) -> f32x4 { return wire4<W16, NT>(a.x[k], vbase + idx); };
        auto put4 = [&](int idx, f32x4 m) { st<NT>(o4 + idx, m); };
        int v = tid;
        for (; v + (B - 1) * kThreads < nv; v += B * kThreads) {
            f32x4 x[B][NREP];
#pragma unroll
            for (int b = 0; b < B; ++b)
#pragma unroll
                for (int k = 0; k < NREP; ++k) x[b][k] = rep4(k, v + b * kThreads);
#pragma unroll
            for (int b = 0; b < B; ++b) {
                f32x4 acc = x[b][0];
#pragma unroll
                for (int k = 1; k < NREP; ++k) acc = acc + x[b][k];
                const f32x4 m = acc * inv_n;
                if constexpr (STATS) {
#pragma unroll
                    for (int k = 0; k < NREP; ++k) stats4(m, x[b][k]);
                    msq4(m);
                }
                put4(v + b * kThreads, m);
            }
        }
        for (; v < nv; v += kThreads) {
            f32x4 x[NREP];
#pragma unroll
            for (int k = 0; k < NREP; ++k) x[k] = rep4(k, v);
            f32x4 acc = x[0];
#pragma unroll
            for (int k = 1; k < NREP; ++k) acc = acc + x[k];
            const f32x4 m = acc * inv_n;
            if constexpr (STATS) {
#pragma unroll
                for (int k = 0; k < NREP; ++k) stats4(m, x[k]);
                msq4(m);
            }
            put4(v, m);
        }
    } else {
        for (int v = tid; v < nv; v += kThreads) {
            f32x4 acc = wire4<W16, NT>(a.x[0], vbase + v);
            for (int k = 1; k < nrep; ++k) acc = acc + wire4<W16, NT>(a.x[k], vbase + v);
            const f32x4 m = acc * inv_n;
            if constexpr (STATS) {
                for (int k = 0; k < nrep; ++k) stats4(m, wire4<W16, false>(a.x[k], vbase + v));
                msq4(m);
            }
            st<NT>(o4 + v, m);
        }
    }

    if constexpr (STATS) {
        const double g = block_sum(gsum, lds[0]);
        const double m = block_sum(msum, lds[1]);
        if (tid == 0) {
            a.partials[2 * (int64_t)ch.partial] = g;
            a.partials[2 * (int64_t)ch.partial + 1] = m;
        }
    }
}

// Per-layer statistics from the per-chunk partials, in two fixed-order stages so that a layer with 10^5 chunks does
// not hang on one workgroup: stage 1 cuts layer l's partials [ranges[2l], ranges[2l+1]) into kStatSlices contiguous
// slices, one workgroup each (thread-strided sums, then the workgroup tree); stage 2 adds the slice sums of a layer
// in slice order and scales the divergence by 1/N (Sec. 3.4: Gamma = 1/K sum_k ||wbar - w^k||^2, per layer).
__global__ __launch_bounds__(kThreads) void stats_slices_kernel(const double *__restrict__ partials,
                                                                const int32_t *__restrict__ ranges, double *__restrict__ slice_sums) {
    __shared__ double lds[2][kThreads / kWave];
    const int l = blockIdx.y, j = blockIdx.x;
    const int64_t c0 = ranges[2 * l], c1 = ranges[2 * l + 1];
    const int64_t lo = c0 + (c1 - c0) * j / kStatSlices, hi = c0 + (c1 - c0) * (j + 1) / kStatSlices;
    double g = 0.0, m = 0.0;
    for (int64_t c = lo + (int64_t)threadIdx.x; c < hi; c += kThreads) {
        g += partials[2 * c];
        m += partials[2 * c + 1];
    }
    g = block_sum(g, lds[0]);
    m = block_sum(m, lds[1]);
    if (threadIdx.x == 0) {
        slice_sums[2 * ((int64_t)l * kStatSlices + j)] = g;
        slice_sums[2 * ((int64_t)l * kStatSlices + j) + 1] = m;
    }
}

__global__ __launch_bounds__(kWave) void stats_finalize_kernel(const double *__restrict__ slice_sums, int n_replicas,
                                                               double *__restrict__ stats) {
    const int l = blockIdx.x;
    if (threadIdx.x == 0) {
        double g = 0.0, m = 0.0;
        for (int j = 0; j < kStatSlices; ++j) {
            g += slice_sums[2 * ((int64_t)l * kStatSlices + j)];
            m += slice_sums[2 * ((int64_t)l * kStatSlices + j) + 1];
        }
        stats[2 * l] = g / (double)n_replicas;
        stats[2 * l + 1] = m;
    }
}

// The same reduction in one launch, for layers with few partials (launch-bound slots): one workgroup per layer adds the
// layer's partials thread-strided, then the workgroup tree.  Fixed order as well.
__global__ __launch_bounds__(kThreads) void stats_single_kernel(const double *__restrict__ partials, const int32_t *__restrict__ ranges,
                                                                int n_replicas, double *__restrict__ stats) {
    __shared__ double lds[2][kThreads / kWave];
    const int l = blockIdx.x;
    const int64_t c0 = ranges[2 * l], c1 = ranges[2 * l + 1];
    double g = 0.0, m = 0.0;
    for (int64_t c = c0 + (int64_t)threadIdx.x; c < c1; c += kThreads) {
        g += partials[2 * c];
        m += partials[2 * c + 1];
    }
    g = block_sum(g, lds[0]);
    m = block_sum(m, lds[1]);
    if (threadIdx.x == 0) {
        stats[2 * l] = g / (double)n_replicas;
        stats[2 * l + 1] = m;
    }
}

// ---------------------------------------------------------------------------------------------------------------
// local update
// ---------------------------------------------------------------------------------------------------------------

// buf = mu*buf + g;  p = p - lr*buf
__device__ __forceinline__ void sgdm_one(float g, float &p, float &buf, const UpdateScalars &s) {
    float b = s.mu * buf;
    b = b + g;
    buf = b;
    const float u = s.lr * b;
    p = p - u;
}

// m = beta1*m + (1-beta1)*g;  v = beta2*v + ((1-beta2)*g)*g;  p = p*decay;  p = p - step_size*(m / (sqrt(v)*rsqrt_bc2 + eps))
__device__ __forceinline__ void adamw_one(float g, float &p, float &m, float &v, const UpdateScalars &s) {
    const float a = s.beta1 * m;
    const float b = s.omb1 * g;
    const float mi = a + b;
    const float c = s.beta2 * v;
    const float d = s.omb2 * g;
    const float e = d * g;
    const float vi = c + e;
    float pi = p * s.decay;
    const float r = __builtin_sqrtf(vi);  // correctly rounded (hipcc default -fhip-fp32-correctly-rounded-divide-sqrt)
    float den = r * s.rsqrt_bc2;
    den = den + s.eps;
    const float q = mi / den;  // IEEE division, correctly rounded
    const float u = s.step_size * q;
    pi = pi - u;
    m = mi;
    v = vi;
    p = pi;
}

template <bool BF16>
struct GradVec;
template <>
struct GradVec<false> {
    typedef float elem;
    typedef f32x4 vec;
    static __device__ __forceinline__ f32x4 widen(f32x4 g) { return g; }
    static __device__ __forceinline__ float widen1(float g) { return g; }
};
template <>
struct GradVec<true> {
    typedef unsigned short elem;
    typedef u16x4 vec;
    static __device__ __forceinline__ f32x4 widen(u16x4 g) {
        return f32x4{bf16_widen(g.x), bf16_widen(g.y), bf16_widen(g.z), bf16_widen(g.w)};
    }
    static __device__ __forceinline__ float widen1(unsigned short g) { return bf16_widen(g); }
};

// Eq. (5), first case, fused: one pass reads gradient, parameter and optimizer state and writes parameter,
// state and (if present) the bf16 model copy.  ADAM selects AdamW, else SGD with momentum.
template <bool ADAM, bool GBF16, bool MODEL, bool NT>
__device__ __forceinline__ void update_chunk_body(const TensorDesc &td, const UpdateChunk &ch, const UpdateScalars &s) {
    typedef GradVec<GBF16> G;
    typedef typename G::elem gelem;
    typedef typename G::vec gvec;
    float *p = td.sync + ch.begin;
    float *s0 = td.state0 + ch.begin;
    float *s1 = ADAM ? td.state1 + ch.begin : s0;  // unused without ADAM
    const gelem *g = reinterpret_cast<const gelem *>(td.grad) + ch.begin;
    unsigned short *mdl = MODEL ? td.model + ch.begin : reinterpret_cast<unsigned short *>(p);  // unused without MODEL
    const int n = ch.count;
    const int tid = threadIdx.x;

    auto one = [&](int i) {
        float pi = p[i], a = s0[i];
        const float gi = G::widen1(g[i]);
        if constexpr (ADAM) {
            float b = s1[i];
            adamw_one(gi, pi, a, b, s);
            s1[i] = b;
        } else {
            sgdm_one(gi, pi, a, s);
        }
        p[i] = pi;
        s0[i] = a;
        if constexpr (MODEL) mdl[i] = bf16_rne(pi);
    };

    // 128-bit path needs every stream to reach its vector alignment after the same head
    const int h = head_to_16B(p, n);
    bool vec_ok = (reinterpret_cast<uintptr_t>(s0 + h) & 15u) == 0;
    if constexpr (ADAM) vec_ok = vec_ok && (reinterpret_cast<uintptr_t>(s1 + h) & 15u) == 0;
    vec_ok = vec_ok && (reinterpret_cast<uintptr_t>(g + h) & (sizeof(gvec) - 1)) == 0;
    if constexpr (MODEL) vec_ok = vec_ok && (reinterpret_cast<uintptr_t>(mdl + h) & 7u) == 0;
    if (!vec_ok) {
        for (int i = tid; i < n; i += kThreads) one(i);
        return;
    }

    if (tid < h) one(tid);
    const int nv = (n - h) >> 2;
    const int tail0 = h + 4 * nv;
    if (tid < n - tail0) one(tail0 + tid);

    f32x4 *p4 = reinterpret_cast<f32x4 *>(p + h);
    f32x4 *a4 = reinterpret_cast<f32x4 *>(s0 + h);
    f32x4 *b4 = reinterpret_cast<f32x4 *>(s1 + h);
    const gvec *g4 = reinterpret_cast<const gvec *>(g + h);
    u16x4 *m4 = reinterpret_cast<u16x4 *>(mdl + h);

    auto compute_store = [&](int v, gvec gv, f32x4 pv, f32x4 av, f32x4 bv) {
        const f32x4 gw = G::widen(gv);
        float G4[4] = {gw.x, gw.y, gw.z, gw.w};
        float P4[4] = {pv.x, pv.y, pv.z, pv.w};
        float A4[4] = {av.x, av.y, av.z, av.w};
        float B4[4] = {bv.x, bv.y, bv.z, bv.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (ADAM)
                adamw_one(G4[j], P4[j], A4[j], B4[j], s);
            else
                sgdm_one(G4[j], P4[j], A4[j], s);
        }
        const f32x4 pn{P4[0], P4[1], P4[2], P4[3]};
        st<NT>(p4 + v, pn);
        st<NT>(a4 + v, f32x4{A4[0], A4[1], A4[2], A4[3]});
        if constexpr (ADAM) st<NT>(b4 + v, f32x4{B4[0], B4[1], B4[2], B4[3]});
        if constexpr (MODEL) st<NT>(m4 + v, bf16_rne4(pn));
    };

    int v = tid;
    for (; v + kThreads < nv; v += 2 * kThreads) {
        const int w = v + kThreads;
        gvec g0 = ld<NT>(g4 + v), g1 = ld<NT>(g4 + w);
        f32x4 p0 = ld<NT>(p4 + v), p1 = ld<NT>(p4 + w);
        f32x4 a0 = ld<NT>(a4 + v), a1 = ld<NT>(a4 + w);
        f32x4 b0{}, b1{};
        if constexpr (ADAM) {
            b0 = ld<NT>(b4 + v);
            b1 = ld<NT>(b4 + w);
        }
        compute_store(v, g0, p0, a0, b0);
        compute_store(w, g1, p1, a1, b1);
    }
    for (; v < nv; v += kThreads) {
        gvec g0 = ld<NT>(g4 + v);
        f32x4 p0 = ld<NT>(p4 + v);
        f32x4 a0 = ld<NT>(a4 + v);
        f32x4 b0{};
        if constexpr (ADAM) b0 = ld<NT>(b4 + v);
        compute_store(v, g0, p0, a0, b0);
    }
}

template <bool ADAM, bool GBF16, bool MODEL, bool NT>
__global__ __launch_bounds__(kThreads) void update_kernel(const TensorDesc *__restrict__ tensors, const UpdateChunk *__restrict__ chunks,
                                                          const UpdateScalars s) {
    const UpdateChunk ch = chunks[blockIdx.x];
    const TensorDesc td = tensors[ch.tensor];
    update_chunk_body<ADAM, GBF16, MODEL, NT>(td, ch, s);
}

// ---------------------------------------------------------------------------------------------------------------
// local update over dense arenas
// ---------------------------------------------------------------------------------------------------------------

struct DenseArgs {
    const void *g;  // the five streams at the first element of the range, each aligned for 128-bit (bf16: 64-bit) access
    float *p;
    float *s0;
    float *s1;
    unsigned short *mdl;
    int64_t n;  // elements in the range
    int chunk;  // elements per workgroup, a multiple of 1024
    UpdateScalars s;
};

// The update when the registered tensors lie back to back in every stream (one arena per stream): workgroup b takes
// elements [b * chunk, (b + 1) * chunk) of the range, addresses follow from the block index alone (no table), and
// every chunk starts aligned, so there is no head; only the last workgroup has a tail of fewer than four elements.
// Same operations per element as update_kernel, hence the same bits.
template <bool ADAM, bool GBF16, bool MODEL, int AUX>
__global__ __launch_bounds__(kThreads) void update_dense_kernel(const DenseArgs a) {
    typedef GradVec<GBF16> G;
    typedef typename G::elem gelem;
    typedef typename G::vec gvec;
    const int64_t b = (int64_t)blockIdx.x * a.chunk;
    const int64_t left = a.n - b;
    const int count = left < (int64_t)a.chunk ? (int)left : a.chunk;
    const UpdateScalars &s = a.s;
    float *p = a.p + b;
    float *s0 = a.s0 + b;
    float *s1 = ADAM ? a.s1 + b : s0;
    const gelem *g = reinterpret_cast<const gelem *>(a.g) + b;
    unsigned short *mdl = MODEL ? a.mdl + b : reinterpret_cast<unsigned short *>(p);
    const int tid = threadIdx.x;
    const int nv = count >> 2;
    const __amdgpu_buffer_rsrc_t rp = make_rsrc(p, nv * 16), ra = make_rsrc(s0, nv * 16), rb = make_rsrc(s1, nv * 16),
                                 rg = make_rsrc(g, nv * (int)sizeof(gvec)), rm = make_rsrc(mdl, nv * 8);

    auto finish = [&](int v, gvec gv, f32x4 pv, f32x4 av, f32x4 bv) {
        const f32x4 gw = G::widen(gv);
        float G4[4] = {gw.x, gw.y, gw.z, gw.w};
        float P4[4] = {pv.x, pv.y, pv.z, pv.w};
        float A4[4] = {av.x, av.y, av.z, av.w};
        float B4[4] = {bv.x, bv.y, bv.z, bv.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (ADAM)
                adamw_one(G4[j], P4[j], A4[j], B4[j], s);
            else
                sgdm_one(G4[j], P4[j], A4[j], s);
        }
        const f32x4 pn{P4[0], P4[1], P4[2], P4[3]};
        bst<AUX>(rp, v * 16, pn);
        bst<AUX>(ra, v * 16, f32x4{A4[0], A4[1], A4[2], A4[3]});
        if constexpr (ADAM) bst<AUX>(rb, v * 16, f32x4{B4[0], B4[1], B4[2], B4[3]});
        if constexpr (MODEL) bst<AUX>(rm, v * 8, bf16_rne4(pn));
    };

    int v = tid;
    for (; v + kThreads < nv; v += 2 * kThreads) {
        const int w = v + kThreads;
        const gvec g0 = bld<AUX, gvec>(rg, v * (int)sizeof(gvec)), g1 = bld<AUX, gvec>(rg, w * (int)sizeof(gvec));
        const f32x4 p0 = bld<AUX, f32x4>(rp, v * 16), p1 = bld<AUX, f32x4>(rp, w * 16);
        const f32x4 a0 = bld<AUX, f32x4>(ra, v * 16), a1 = bld<AUX, f32x4>(ra, w * 16);
        f32x4 b0{}, b1{};
        if constexpr (ADAM) {
            b0 = bld<AUX, f32x4>(rb, v * 16);
            b1 = bld<AUX, f32x4>(rb, w * 16);
        }
        finish(v, g0, p0, a0, b0);
        finish(w, g1, p1, a1, b1);
    }
    for (; v < nv; v += kThreads) {
        const gvec g0 = bld<AUX, gvec>(rg, v * (int)sizeof(gvec));
        const f32x4 p0 = bld<AUX, f32x4>(rp, v * 16);
        const f32x4 a0 = bld<AUX, f32x4>(ra, v * 16);
        f32x4 b0{};
        if constexpr (ADAM) b0 = bld<AUX, f32x4>(rb, v * 16);
        finish(v, g0, p0, a0, b0);
    }
    const int i = 4 * nv + tid;  // fewer than four elements, last workgroup of the range only
    if (i < count) {
        float pi = p[i], av = s0[i];
        const float gi = G::widen1(g[i]);
        if constexpr (ADAM) {
            float bv = s1[i];
            adamw_one(gi, pi, av, bv, s);
            s1[i] = bv;
        } else {
            sgdm_one(gi, pi, av, s);
        }
        p[i] = pi;
        s0[i] = av;
        if constexpr (MODEL) mdl[i] = bf16_rne(pi);
    }
}

// ---------------------------------------------------------------------------------------------------------------
// fused synchronisation + update
// ---------------------------------------------------------------------------------------------------------------

// One group of four elements of a scheduled tensor, N known at compile time: pv = the N-1 peers' values (rank order,
// local rank left out), x = the local parameter on entry and the value to store on return, av / bv = optimizer state
// (updated in place).  The local contribution (x, stepped first if UTS, rounded to bf16 if W16) is put at position
// lr with register selects (lr is wave-uniform); rank-order fp32 sum, one multiply by 1/N; statistics in fp64.
template <bool ADAM, bool GBF16, int NREP, bool STATS, bool W16, bool UTS>
__device__ __forceinline__ void fused_math4(const f32x4 (&pv)[NREP - 1], typename GradVec<GBF16>::vec gv, f32x4 &x, f32x4 &av, f32x4 &bv,
                                            int lr, float inv_n, const UpdateScalars &s, double &gsum, double &msum) {
    auto step4 = [&](f32x4 &q) {
        const f32x4 gw = GradVec<GBF16>::widen(gv);
        float G4[4] = {gw.x, gw.y, gw.z, gw.w};
        float P4[4] = {q.x, q.y, q.z, q.w};
        float A4[4] = {av.x, av.y, av.z, av.w};
        float B4[4] = {bv.x, bv.y, bv.z, bv.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (ADAM)
                adamw_one(G4[j], P4[j], A4[j], B4[j], s);
            else
                sgdm_one(G4[j], P4[j], A4[j], s);
        }
        q = f32x4{P4[0], P4[1], P4[2], P4[3]};
        av = f32x4{A4[0], A4[1], A4[2], A4[3]};
        bv = f32x4{B4[0], B4[1], B4[2], B4[3]};
    };
    if constexpr (UTS) step4(x);
    f32x4 loc = x;
    if constexpr (W16) loc = bf16_widen4(bf16_rne4(x));
    f32x4 r[NREP];
#pragma unroll
    for (int k = 0; k < NREP; ++k) {
        const f32x4 before = pv[k < NREP - 1 ? k : NREP - 2], after = pv[k > 0 ? k - 1 : 0];
        r[k] = k == lr ? loc : (k < lr ? before : after);
    }
    f32x4 acc = r[0];
#pragma unroll
    for (int k = 1; k < NREP; ++k) acc = acc + r[k];
    f32x4 m = acc * inv_n;
    if constexpr (STATS) {
#pragma unroll
        for (int k = 0; k < NREP; ++k) {
            const f32x4 d = m - r[k];
            gsum += (double)d.x * (double)d.x;
            gsum += (double)d.y * (double)d.y;
            gsum += (double)d.z * (double)d.z;
            gsum += (double)d.w * (double)d.w;
        }
        msum += (double)m.x * (double)m.x;
        msum += (double)m.y * (double)m.y;
        msum += (double)m.z * (double)m.z;
        msum += (double)m.w * (double)m.w;
    }
    if constexpr (!UTS) step4(m);
    x = m;
}

struct FusedArgs {
    const void *x[DDP_MAX_REPLICAS];  // peers' flat buffers (fp32 or bf16) in rank order; entry local_rank is unused
    const TensorDesc *tensors;
    const UpdateChunk *chunks;
    const int64_t *tensor_flat_off;     // per tensor: first flat index in this slot, or -1 if not scheduled
    const int32_t *tensor_chunk_base;   // per tensor: index of its first chunk in registration order
    double *partials;                   // [n_chunks][2], only touched for scheduled chunks
    UpdateScalars s;
    float inv_n;
    int n;
    int local_rank;
    int chunk_elems;
};

// Both cases of Eq. (5) in one pass.  For a chunk of a scheduled tensor the average over the N replicas is formed from
// the local tensor and the peers' flat buffers (read at the tensor's flat offset; same rank-ordered fp32 sum and 1/N
// multiply as mean_kernel) and the optimizer step is applied; every other chunk gets the optimizer step only.
//   UTS = false: average, then update the average (the bits of pack -> partial average -> unpack -> local update);
//   UTS = true:  update the local value, then average it with the peers (Eq. (5) and Algorithm 1 as printed: the
//                replicas that are averaged have taken this iteration's step; the bits of local update -> pack ->
//                partial average -> unpack).
// W16: peers are bf16 and the local replica contributes its bf16 rounding.  NREP > 0: replica count known at compile
// time; 0: run-time loop.
template <bool ADAM, bool GBF16, bool MODEL, int NREP, bool STATS, bool W16 = false, bool UTS = false>
__global__ __launch_bounds__(kThreads) void fused_kernel(const FusedArgs a) {
    typedef GradVec<GBF16> G;
    typedef typename G::elem gelem;
    typedef typename G::vec gvec;
    constexpr bool NT = true;
    __shared__ double lds[2][kThreads / kWave];
    const UpdateChunk ch = a.chunks[blockIdx.x];
    const TensorDesc td = a.tensors[ch.tensor];
    const int64_t toff = a.tensor_flat_off[ch.tensor];
    if (toff < 0) {  // uniform for the workgroup
        update_chunk_body<ADAM, GBF16, MODEL, NT>(td, ch, a.s);
        return;
    }
    const UpdateScalars &s = a.s;
    const int64_t fo = toff + ch.begin;
    float *p = td.sync + ch.begin;
    float *s0 = td.state0 + ch.begin;
    float *s1 = ADAM ? td.state1 + ch.begin : s0;
    const gelem *g = reinterpret_cast<const gelem *>(td.grad) + ch.begin;
    unsigned short *mdl = MODEL ? td.model + ch.begin : reinterpret_cast<unsigned short *>(p);
    const int n = ch.count;
    const int tid = threadIdx.x;
    const int nrep = NREP > 0 ? NREP : a.n;
    const int lr = a.local_rank;
    const float inv_n = a.inv_n;
    double gsum = 0.0, msum = 0.0;

    auto step1 = [&](float gi, float &x, float &av, float &bv) {
        if constexpr (ADAM)
            adamw_one(gi, x, av, bv, s);
        else
            sgdm_one(gi, x, av, s);
    };

    // one element: scalar head and tail, and chunks whose streams are not mutually aligned
    auto one = [&](int i) {
        float pl = p[i], av = s0[i], bv = ADAM ? s1[i] : 0.0f;
        const float gi = G::widen1(g[i]);
        if constexpr (UTS) step1(gi, pl, av, bv);
        // what this worker contributes: its value, rounded to bf16 first if that is what its peers received
        const float loc = W16 ? bf16_widen(bf16_rne(pl)) : pl;
        auto term = [&](int k) -> float { return k == lr ? loc : wire1<W16>(a.x[k], fo + i); };
        float acc = term(0);
        for (int k = 1; k < nrep; ++k) acc = acc + term(k);
        const float m = acc * inv_n;
        if constexpr (STATS) {
            for (int k = 0; k < nrep; ++k) {
                const float d = m - term(k);
                gsum += (double)d * (double)d;
            }
            msum += (double)m * (double)m;
        }
        float res = m;
        if constexpr (!UTS) step1(gi, res, av, bv);
        p[i] = res;
        s0[i] = av;
        if constexpr (ADAM) s1[i] = bv;
        if constexpr (MODEL) mdl[i] = bf16_rne(res);
    };

    const int h = head_to_16B(p, n);
    bool vec_ok = (reinterpret_cast<uintptr_t>(s0 + h) & 15u) == 0 && ((fo + h) & 3) == 0;
    if constexpr (ADAM) vec_ok = vec_ok && (reinterpret_cast<uintptr_t>(s1 + h) & 15u) == 0;
    vec_ok = vec_ok && (reinterpret_cast<uintptr_t>(g + h) & (sizeof(gvec) - 1)) == 0;
    if constexpr (MODEL) vec_ok = vec_ok && (reinterpret_cast<uintptr_t>(mdl + h) & 7u) == 0;
    if (!vec_ok) {
        for (int i = tid; i < n; i += kThreads) one(i);
    } else {
        if (tid < h) one(tid);
        const int nv = (n - h) >> 2;
        const int tail0 = h + 4 * nv;
        if (tid < n - tail0) one(tail0 + tid);
        f32x4 *p4 = reinterpret_cast<f32x4 *>(p + h);
        f32x4 *a4 = reinterpret_cast<f32x4 *>(s0 + h);
        f32x4 *b4 = reinterpret_cast<f32x4 *>(s1 + h);
        const gvec *g4 = reinterpret_cast<const gvec *>(g + h);
        u16x4 *m4 = reinterpret_cast<u16x4 *>(mdl + h);
        const int64_t vfo = (fo + h) >> 2;  // peers' index of the body's first group of four
        auto stats4 = [&](f32x4 m, f32x4 x) {
            const f32x4 d = m - x;
            gsum += (double)d.x * (double)d.x;
            gsum += (double)d.y * (double)d.y;
            gsum += (double)d.z * (double)d.z;
            gsum += (double)d.w * (double)d.w;
        };
        auto msq4 = [&](f32x4 m) {
            msum += (double)m.x * (double)m.x;
            msum += (double)m.y * (double)m.y;
            msum += (double)m.z * (double)m.z;
            msum += (double)m.w * (double)m.w;
        };
        auto step4 = [&](gvec gv, f32x4 &x, f32x4 &av, f32x4 &bv) {
            const f32x4 gw = G::widen(gv);
            float G4[4] = {gw.x, gw.y, gw.z, gw.w};
            float P4[4] = {x.x, x.y, x.z, x.w};
            float A4[4] = {av.x, av.y, av.z, av.w};
            float B4[4] = {bv.x, bv.y, bv.z, bv.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) step1(G4[j], P4[j], A4[j], B4[j]);
            x = f32x4{P4[0], P4[1], P4[2], P4[3]};
            av = f32x4{A4[0], A4[1], A4[2], A4[3]};
            bv = f32x4{B4[0], B4[1], B4[2], B4[3]};
        };
        auto store4 = [&](int v, f32x4 res, f32x4 av, f32x4 bv) {
            st<NT>(p4 + v, res);
            st<NT>(a4 + v, av);
            if constexpr (ADAM) st<NT>(b4 + v, bv);
            if constexpr (MODEL) st<NT>(m4 + v, bf16_rne4(res));
        };
        if constexpr (NREP > 1) {
            // The local contribution may be computed (updated and / or rounded) and a branch per replica would
            // serialise the loads: load the N-1 peers unconditionally, all in flight before the first use.
            for (int v = tid; v < nv; v += kThreads) {
                f32x4 pv[NREP - 1];
#pragma unroll
                for (int j = 0; j < NREP - 1; ++j) pv[j] = wire4<W16, NT>(a.x[j + (j >= lr ? 1 : 0)], vfo + v);
                f32x4 pl = ld<NT>(p4 + v);
                const gvec gv = ld<NT>(g4 + v);
                f32x4 av = ld<NT>(a4 + v);
                f32x4 bv{};
                if constexpr (ADAM) bv = ld<NT>(b4 + v);
                fused_math4<ADAM, GBF16, NREP, STATS, W16, UTS>(pv, gv, pl, av, bv, lr, inv_n, s, gsum, msum);
                store4(v, pl, av, bv);
            }
        } else {
            for (int v = tid; v < nv; v += kThreads) {
                f32x4 pl = ld<NT>(p4 + v);
                const gvec gv = ld<NT>(g4 + v);
                f32x4 av = ld<NT>(a4 + v);
                f32x4 bv{};
                if constexpr (ADAM) bv = ld<NT>(b4 + v);
                if constexpr (UTS) step4(gv, pl, av, bv);
                f32x4 loc = pl;
                if constexpr (W16) loc = bf16_widen4(bf16_rne4(pl));
                auto term = [&](int k) -> f32x4 { return k == lr ? loc : wire4<W16, NT>(a.x[k], vfo + v); };
                f32x4 acc = term(0);
                for (int k = 1; k < nrep; ++k) acc = acc + term(k);
                f32x4 m = acc * inv_n;
                if constexpr (STATS) {
                    for (int k = 0; k < nrep; ++k) stats4(m, term(k));
                    msq4(m);
                }
                if constexpr (!UTS) step4(gv, m, av, bv);
                store4(v, m, av, bv);
            }
        }
    }
    if constexpr (STATS) {
        const double gt = block_sum(gsum, lds[0]);
        const double mt = block_sum(msum, lds[1]);
        if (tid == 0) {
            const int64_t pi = (int64_t)a.tensor_chunk_base[ch.tensor] + ch.begin / a.chunk_elems;
            a.partials[2 * pi] = gt;
            a.partials[2 * pi + 1] = mt;
        }
    }
}

struct FusedDenseArgs {
    DenseArgs d;                       // the scheduled layer's local streams; d.n is a multiple of 4
    const void *x[DDP_MAX_REPLICAS];   // peers' whole flat buffers in rank order; entry local_rank is unused
    int64_t fo0;                       // flat index of the layer's first element (a multiple of 4)
    double *partials;                  // workgroup b writes its pair at partials[2 * (pbase + b)]
    int64_t pbase;
    float inv_n;
    int local_rank;
};

// fused_kernel for one scheduled layer of a model registered as dense arenas: table-free addressing, buffer accesses
// for all streams, the arithmetic of fused_math4.  Launched once per scheduled layer; the layers in between take
// update_dense_kernel.
template <bool ADAM, bool GBF16, bool MODEL, int NREP, bool STATS, bool W16, bool UTS>
__global__ __launch_bounds__(kThreads) void fused_dense_kernel(const FusedDenseArgs a) {
    typedef GradVec<GBF16> G;
    typedef typename G::elem gelem;
    typedef typename G::vec gvec;
    static_assert(NREP > 1, "compile-time replica count");
    constexpr int AUX = 2;                  // nt
    constexpr int XB = W16 ? 8 : 16;        // bytes of one peer's group of four
    __shared__ double lds[2][kThreads / kWave];
    const int64_t b = (int64_t)blockIdx.x * a.d.chunk;
    const int64_t left = a.d.n - b;
    const int count = left < (int64_t)a.d.chunk ? (int)left : a.d.chunk;
    const int nv = count >> 2;
    const int tid = threadIdx.x;
    const int lr = a.local_rank;
    float *p = a.d.p + b;
    float *s0 = a.d.s0 + b;
    float *s1 = ADAM ? a.d.s1 + b : s0;
    const gelem *g = reinterpret_cast<const gelem *>(a.d.g) + b;
    unsigned short *mdl = MODEL ? a.d.mdl + b : reinterpret_cast<unsigned short *>(p);
    const __amdgpu_buffer_rsrc_t rp = make_rsrc(p, nv * 16), ra = make_rsrc(s0, nv * 16), rb = make_rsrc(s1, nv * 16),
                                 rg = make_rsrc(g, nv * (int)sizeof(gvec)), rm = make_rsrc(mdl, nv * 8);
    __amdgpu_buffer_rsrc_t rx[NREP - 1];
#pragma unroll
    for (int j = 0; j < NREP - 1; ++j)
        rx[j] = make_rsrc(reinterpret_cast<const char *>(a.x[j + (j >= lr ? 1 : 0)]) + (a.fo0 + b) * (XB / 4), nv * XB);
    double gsum = 0.0, msum = 0.0;
    for (int v = tid; v < nv; v += kThreads) {
        f32x4 pv[NREP - 1];
#pragma unroll
        for (int j = 0; j < NREP - 1; ++j) {
            if constexpr (W16)
                pv[j] = bf16_widen4(bld<AUX, u16x4>(rx[j], v * XB));
            else
                pv[j] = bld<AUX, f32x4>(rx[j], v * XB);
        }
        f32x4 x = bld<AUX, f32x4>(rp, v * 16);
        const gvec gv = bld<AUX, gvec>(rg, v * (int)sizeof(gvec));
        f32x4 av = bld<AUX, f32x4>(ra, v * 16);
        f32x4 bv{};
        if constexpr (ADAM) bv = bld<AUX, f32x4>(rb, v * 16);
        fused_math4<ADAM, GBF16, NREP, STATS, W16, UTS>(pv, gv, x, av, bv, lr, a.inv_n, a.d.s, gsum, msum);
        bst<AUX>(rp, v * 16, x);
        bst<AUX>(ra, v * 16, av);
        if constexpr (ADAM) bst<AUX>(rb, v * 16, bv);
        if constexpr (MODEL) bst<AUX>(rm, v * 8, bf16_rne4(x));
    }
    if constexpr (STATS) {
        const double gt = block_sum(gsum, lds[0]);
        const double mt = block_sum(msum, lds[1]);
        if (tid == 0) {
            a.partials[2 * (a.pbase + blockIdx.x)] = gt;
            a.partials[2 * (a.pbase + blockIdx.x) + 1] = mt;
        }
    }
}

// lds_pad: bytes of dynamic LDS requested per workgroup although no kernel uses them.  A CU has 160 KiB, so the pad
// caps how many workgroups are resident per CU, i.e. how wide the window of addresses in flight is.
template <class K, class... Args>
int launch(K kernel, int64_t grid, void *stream, int lds_pad, Args... args) {
    if (grid <= 0) return 0;
    if (grid > 0x7fffffff) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(kThreads), (size_t)lds_pad, (hipStream_t)stream, args...);
    return (int)hipGetLastError();
}


template <int NREP>
int launch_mean16_n(const MeanArgs &ma, const MeanLaunch &a, void *stream) {
    if (a.partials) return launch(mean_kernel<NREP, true, true, true>, a.n_chunks, stream, a.lds_pad, ma);
    return launch(mean_kernel<NREP, false, true, true>, a.n_chunks, stream, a.lds_pad, ma);
}

template <int NREP>
int launch_mean_n(const MeanArgs &ma, const MeanLaunch &a, void *stream) {
    if (a.partials) return a.nontemporal ? launch(mean_kernel<NREP, true, true>, a.n_chunks, stream, a.lds_pad, ma) : launch(mean_kernel<NREP, true, false>, a.n_chunks, stream, a.lds_pad, ma);
    return a.nontemporal ? launch(mean_kernel<NREP, false, true>, a.n_chunks, stream, a.lds_pad, ma) : launch(mean_kernel<NREP, false, false>, a.n_chunks, stream, a.lds_pad, ma);
}

}  // namespace

int launch_stats(const double *partials, double *slice_sums, const int32_t *ranges, int n_layers, int n_replicas, double *stats,
                 int64_t max_partials_per_layer, void *stream) {
    if (n_layers <= 0) return 0;
    if (max_partials_per_layer <= kStatSingleMax) {
        hipLaunchKernelGGL(stats_single_kernel, dim3((unsigned)n_layers), dim3(kThreads), 0, (hipStream_t)stream, partials, ranges,
                           n_replicas, stats);
        return (int)hipGetLastError();
    }
    hipLaunchKernelGGL(stats_slices_kernel, dim3(kStatSlices, (unsigned)n_layers), dim3(kThreads), 0, (hipStream_t)stream, partials,
                       ranges, slice_sums);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
    hipLaunchKernelGGL(stats_finalize_kernel, dim3((unsigned)n_layers), dim3(kWave), 0, (hipStream_t)stream,
                       (const double *)slice_sums, n_replicas, stats);
    return (int)hipGetLastError();
}

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

int launch_mean(const MeanLaunch &a, void *stream) {
    MeanArgs ma{};
    for (int k = 0; k < a.n_replicas; ++k) ma.x[k] = a.x[k];
    ma.out = a.out;
    ma.chunks = a.chunks;
    ma.partials = a.partials;
    ma.inv_n = a.inv_n;
    ma.n = a.n_replicas;
    int rc;
    if (a.wire16) {
        switch (a.n_replicas) {
            case 4: rc = launch_mean16_n<4>(ma, a, stream); break;
            case 8: rc = launch_mean16_n<8>(ma, a, stream); break;
            case 16: rc = launch_mean16_n<16>(ma, a, stream); break;
            default: rc = launch_mean16_n<0>(ma, a, stream); break;
        }
    } else {
        switch (a.n_replicas) {
            case 1: rc = launch_mean_n<1>(ma, a, stream); break;
            case 2: rc = launch_mean_n<2>(ma, a, stream); break;
            case 3: rc = launch_mean_n<3>(ma, a, stream); break;
            case 4: rc = launch_mean_n<4>(ma, a, stream); break;
            case 5: rc = launch_mean_n<5>(ma, a, stream); break;
            case 6: rc = launch_mean_n<6>(ma, a, stream); break;
            case 7: rc = launch_mean_n<7>(ma, a, stream); break;
            case 8: rc = launch_mean_n<8>(ma, a, stream); break;
            case 16: rc = launch_mean_n<16>(ma, a, stream); break;
            default: rc = launch_mean_n<0>(ma, a, stream); break;
        }
    }
    if (rc != 0 || !a.partials) return rc;
    return launch_stats(a.partials, a.slice_sums, a.layer_ranges, a.n_layers, a.n_replicas, a.stats, a.max_partials_per_layer, stream);
}

int launch_update(int kind, int grad_dtype, bool with_model, const TensorDesc *tensors, const UpdateChunk *chunks, int64_t n_chunks,
                  const UpdateScalars &s, bool nontemporal, int lds_pad, void *stream) {
    const bool adam = kind == DDP_OPT_ADAMW, gb = grad_dtype == DDP_BF16;
#define DDP_UPD(A, G, M)                                                                               \
    if (adam == A && gb == G && with_model == M)                                                       \
        return nontemporal ? launch(update_kernel<A, G, M, true>, n_chunks, stream, lds_pad, tensors, chunks, s) \
                           : launch(update_kernel<A, G, M, false>, n_chunks, stream, lds_pad, tensors, chunks, s);
    DDP_UPD(false, false, false)
    DDP_UPD(false, false, true)
    DDP_UPD(false, true, false)
    DDP_UPD(false, true, true)
    DDP_UPD(true, false, false)
    DDP_UPD(true, false, true)
    DDP_UPD(true, true, false)
    DDP_UPD(true, true, true)
#undef DDP_UPD
    return (int)hipErrorInvalidValue;
}

int launch_update_dense(int kind, int grad_dtype, bool with_model, const DenseLaunch &d, const UpdateScalars &s, bool nontemporal,
                        int lds_pad, void *stream) {
    if (d.n <= 0) return 0;
    DenseArgs a{};
    a.g = d.g;
    a.p = d.p;
    a.s0 = d.s0;
    a.s1 = d.s1;
    a.mdl = d.mdl;
    a.n = d.n;
    a.chunk = d.chunk;
    a.s = s;
    const int64_t grid = (d.n + d.chunk - 1) / d.chunk;
    const bool adam = kind == DDP_OPT_ADAMW, gb = grad_dtype == DDP_BF16;
#define DDP_UPD(A, G, M)                                                                                \
    if (adam == A && gb == G && with_model == M)                                                        \
        return nontemporal ? launch(update_dense_kernel<A, G, M, 2>, grid, stream, lds_pad, a)          \
                           : launch(update_dense_kernel<A, G, M, 0>, grid, stream, lds_pad, a);
    DDP_UPD(false, false, false)
    DDP_UPD(false, false, true)
    DDP_UPD(false, true, false)
    DDP_UPD(false, true, true)
    DDP_UPD(true, false, false)
    DDP_UPD(true, false, true)
    DDP_UPD(true, true, false)
    DDP_UPD(true, true, true)
#undef DDP_UPD
    return (int)hipErrorInvalidValue;
}

template <bool A, bool G, bool M, int NR>
static int launch_fused_dense_n(const FusedDenseLaunch &f, const FusedDenseArgs &fa, int64_t grid, void *stream) {
    const bool st = f.partials != nullptr;
#define DDP_FUSED(W, U)                                                                             \
    return st ? launch(fused_dense_kernel<A, G, M, NR, true, W, U>, grid, stream, f.lds_pad, fa)    \
              : launch(fused_dense_kernel<A, G, M, NR, false, W, U>, grid, stream, f.lds_pad, fa);
    if (f.wire16) {
        if (f.update_first) { DDP_FUSED(true, true) }
        DDP_FUSED(true, false)
    }
    if (f.update_first) { DDP_FUSED(false, true) }
    DDP_FUSED(false, false)
#undef DDP_FUSED
}

bool fused_dense_supports(int n_replicas) { return n_replicas == 4 || n_replicas == 8 || n_replicas == 16; }

int launch_fused_dense(const FusedDenseLaunch &f, void *stream) {
    if (f.d.n <= 0) return 0;
    FusedDenseArgs fa{};
    fa.d.g = f.d.g;
    fa.d.p = f.d.p;
    fa.d.s0 = f.d.s0;
    fa.d.s1 = f.d.s1;
    fa.d.mdl = f.d.mdl;
    fa.d.n = f.d.n;
    fa.d.chunk = f.d.chunk;
    fa.d.s = f.s;
    for (int k = 0; k < f.n_replicas; ++k) fa.x[k] = f.x[k];
    fa.fo0 = f.fo0;
    fa.partials = f.partials;
    fa.pbase = f.pbase;
    fa.inv_n = f.inv_n;
    fa.local_rank = f.local_rank;
    const int64_t grid = (f.d.n + f.d.chunk - 1) / f.d.chunk;
    const bool adam = f.kind == DDP_OPT_ADAMW, gb = f.grad_dtype == DDP_BF16, md = f.with_model;
#define DDP_F(A, G, M)                                                                                  \
    if (adam == A && gb == G && md == M) switch (f.n_replicas) {                                        \
            case 4: return launch_fused_dense_n<A, G, M, 4>(f, fa, grid, stream);                       \
            case 8: return launch_fused_dense_n<A, G, M, 8>(f, fa, grid, stream);                       \
            case 16: return launch_fused_dense_n<A, G, M, 16>(f, fa, grid, stream);                     \
            default: return (int)hipErrorInvalidValue;                                                  \
        }
    DDP_F(false, false, false)
    DDP_F(false, false, true)
    DDP_F(false, true, false)
    DDP_F(false, true, true)
    DDP_F(true, false, false)
    DDP_F(true, false, true)
    DDP_F(true, true, false)
    DDP_F(true, true, true)
#undef DDP_F
    return (int)hipErrorInvalidValue;
}

template <bool A, bool G, bool M, int NR>
static int launch_fused_n(const FusedLaunch &f, const FusedArgs &fa, void *stream) {
    const bool st = f.partials != nullptr;
#define DDP_FUSED(W, U)                                                                                \
    return st ? launch(fused_kernel<A, G, M, NR, true, W, U>, f.n_chunks, stream, f.lds_pad, fa)       \
              : launch(fused_kernel<A, G, M, NR, false, W, U>, f.n_chunks, stream, f.lds_pad, fa);
    if (f.wire16) {
        if (f.update_first) { DDP_FUSED(true, true) }
        DDP_FUSED(true, false)
    }
    if (f.update_first) { DDP_FUSED(false, true) }
    DDP_FUSED(false, false)
#undef DDP_FUSED
}

template <bool A, bool G, bool M>
static int launch_fused_t(const FusedLaunch &f, const FusedArgs &fa, void *stream) {
    switch (f.n_replicas) {
        case 4: return launch_fused_n<A, G, M, 4>(f, fa, stream);
        case 8: return launch_fused_n<A, G, M, 8>(f, fa, stream);
        case 16: return launch_fused_n<A, G, M, 16>(f, fa, stream);
        default: return launch_fused_n<A, G, M, 0>(f, fa, stream);
    }
}

int launch_fused(const FusedLaunch &f, void *stream) {
    FusedArgs fa{};
    for (int k = 0; k < f.n_replicas; ++k) fa.x[k] = f.x[k];
    fa.tensors = f.tensors;
    fa.chunks = f.chunks;
    fa.tensor_flat_off = f.tensor_flat_off;
    fa.tensor_chunk_base = f.tensor_chunk_base;
    fa.partials = f.partials;
    fa.s = f.s;
    fa.inv_n = f.inv_n;
    fa.n = f.n_replicas;
    fa.local_rank = f.local_rank;
    fa.chunk_elems = f.chunk_elems;
    const bool adam = f.kind == DDP_OPT_ADAMW, gb = f.grad_dtype == DDP_BF16, md = f.with_model;
    int rc = (int)hipErrorInvalidValue;
#define DDP_F(A, G, M) \
    if (adam == A && gb == G && md == M) rc = launch_fused_t<A, G, M>(f, fa, stream);
    DDP_F(false, false, false)
    DDP_F(false, false, true)
    DDP_F(false, true, false)
    DDP_F(false, true, true)
    DDP_F(true, false, false)
    DDP_F(true, false, true)
    DDP_F(true, true, false)
    DDP_F(true, true, true)
#undef DDP_F
    if (rc != 0 || !f.partials) return rc;
    return launch_stats(f.partials, f.slice_sums, f.layer_ranges, f.n_layers, f.n_replicas, f.stats, f.max_partials_per_layer, stream);
}

}  // namespace ddp
