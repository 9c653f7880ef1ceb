// Device-side helpers shared by the kernel files of the library (gfx950).
//
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
#ifndef DDP_DEVICE_H
#define DDP_DEVICE_H

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

// A group of four elements of a replica as it sits in memory, and its exact widening to fp32.
template <bool W16>
struct WireVec;
template <>
struct WireVec<false> {
    typedef f32x4 type;
    static __device__ __forceinline__ f32x4 widen(f32x4 v) { return v; }
};
template <>
struct WireVec<true> {
    typedef u16x4 type;
    static __device__ __forceinline__ f32x4 widen(u16x4 v) { return bf16_widen4(v); }
};

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

// Run-time replica counts (the kernels compiled for a fixed count keep all replicas in registers): a thread parks
// each vector it loads in LDS while it forms the rank-order sum, and reads the vectors back for the statistics, so every
// replica is fetched from memory once (the averaging kernel keeps the first kRegReps replicas in registers and parks only
// the rest).  The staging area is dynamic LDS laid out [replica][thread] (each thread only
// ever touches its own column: no barrier needed, no bank conflicts); with kStageBytes of it, stage_threads(N) threads
// of the workgroup (whole wavefronts) take part in the vector loop.
constexpr int kStageBytes = 65536;
constexpr int kRegReps = 16;  // averaging kernel, run-time count: replicas of a vector that stay in registers
inline int stage_threads(int n_replicas) {
    int t = kStageBytes / 16 / (n_replicas > 0 ? n_replicas : 1) / kWave * kWave;
    return t > kThreads ? kThreads : t;  // at least one wavefront up to DDP_MAX_REPLICAS = 64
}
static_assert(kStageBytes / 16 / DDP_MAX_REPLICAS >= kWave, "the staging area must hold one wavefront at the largest replica count");

// lds_pad: bytes of dynamic LDS requested per workgroup although no kernel uses them.  A CU has 160 KiB, so the pad
// caps how many workgroups are resident per CU, i.e. how wide the window of addresses in flight is.
template <class K, class... Args>
int launch(K kernel, int64_t grid, void *stream, int lds_pad, Args... args) {
    if (grid <= 0) return 0;
    if (grid > 0x7fffffff) return (int)hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(kThreads), (size_t)lds_pad, (hipStream_t)stream, args...);
    return (int)hipGetLastError();
}

}  // namespace
}  // namespace ddp

#endif
