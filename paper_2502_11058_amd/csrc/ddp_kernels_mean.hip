// partial average (Eq. (5), second case) and the per-layer statistics (Sec. 3.4).
#include "ddp_device.h"

namespace ddp {
namespace {

struct MeanArgs {
    const void *x[DDP_MAX_REPLICAS];  // fp32 or bf16 flat buffers, rank order
    float *out;
    const MeanChunk *chunks;
    double *partials;
    float inv_n;
    int n;
    int stage_threads;  // run-time replica count with statistics: threads that take part in the vector loop
};

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
        // vectors per thread in flight: 2 * NREP loads (a 2048-element chunk is 2 vectors per thread); beyond 16 replicas one
        // vector, so that the loads still fit the register file
        constexpr int B = NREP > 16 ? 1 : 2;
        // a replica's vector as it sits in memory: kept in that form (bf16: half the registers) until it is used
        typedef typename WireVec<W16>::type raw4;
        auto rep4 = [&](int k, int idx) -> raw4 { return ld<NT>(reinterpret_cast<const raw4 *>(a.x[k]) + vbase + idx); };
        auto put4 = [&](int idx, f32x4 m) { st<NT>(o4 + idx, m); };
        int v = tid;
        for (; v + (B - 1) * kThreads < nv; v += B * kThreads) {
            raw4 x[B][NREP];
#pragma unroll
            for (int b = 0; b < B; ++b)
#pragma unroll
                for (int k = 0; k < NREP; ++k) x[b][k] = rep4(k, v + b * kThreads);
#pragma unroll
            for (int b = 0; b < B; ++b) {
                f32x4 acc = WireVec<W16>::widen(x[b][0]);
#pragma unroll
                for (int k = 1; k < NREP; ++k) acc = acc + WireVec<W16>::widen(x[b][k]);
                const f32x4 m = acc * inv_n;
                if constexpr (STATS) {
#pragma unroll
                    for (int k = 0; k < NREP; ++k) stats4(m, WireVec<W16>::widen(x[b][k]));
                    msq4(m);
                }
                put4(v + b * kThreads, m);
            }
        }
        for (; v < nv; v += kThreads) {
            raw4 x[NREP];
#pragma unroll
            for (int k = 0; k < NREP; ++k) x[k] = rep4(k, v);
            f32x4 acc = WireVec<W16>::widen(x[0]);
#pragma unroll
            for (int k = 1; k < NREP; ++k) acc = acc + WireVec<W16>::widen(x[k]);
            const f32x4 m = acc * inv_n;
            if constexpr (STATS) {
#pragma unroll
                for (int k = 0; k < NREP; ++k) stats4(m, WireVec<W16>::widen(x[k]));
                msq4(m);
            }
            put4(v, m);
        }
    } else if constexpr (STATS) {
        // Run-time replica count with statistics: the first kRegReps replicas of a vector stay in registers, the rest are
        // parked in LDS (one column per thread), so every replica is fetched from memory once and, up to 32 replicas,
        // every thread takes part.
        extern __shared__ __align__(16) unsigned char dyn_lds[];
        f32x4 *stage = reinterpret_cast<f32x4 *>(dyn_lds);
        const int vt = a.stage_threads;
        if (tid < vt) {
            for (int v = tid; v < nv; v += vt) {
                f32x4 r[kRegReps];
#pragma unroll
                for (int k = 0; k < kRegReps; ++k)
                    if (k < nrep) r[k] = wire4<W16, NT>(a.x[k], vbase + v);
                f32x4 acc = r[0];
#pragma unroll
                for (int k = 1; k < kRegReps; ++k)
                    if (k < nrep) acc = acc + r[k];
                for (int k0 = kRegReps; k0 < nrep; k0 += 4) {  // four more loads in flight, then park and add them in rank order
                    f32x4 x[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (k0 + j < nrep) x[j] = wire4<W16, NT>(a.x[k0 + j], vbase + v);
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (k0 + j < nrep) {
                            stage[(k0 + j - kRegReps) * vt + tid] = x[j];
                            acc = acc + x[j];
                        }
                }
                const f32x4 m = acc * inv_n;
#pragma unroll
                for (int k = 0; k < kRegReps; ++k)
                    if (k < nrep) stats4(m, r[k]);
                for (int k = kRegReps; k < nrep; ++k) stats4(m, stage[(k - kRegReps) * vt + tid]);
                msq4(m);
                st<NT>(o4 + v, m);
            }
        }
    } else {
        for (int v = tid; v < nv; v += kThreads) {
            f32x4 acc = wire4<W16, NT>(a.x[0], vbase + v);
            for (int k = 1; k < nrep; ++k) acc = acc + wire4<W16, NT>(a.x[k], vbase + v);
            st<NT>(o4 + v, acc * inv_n);
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

// Dynamic LDS of a launch: the residency pad, or the staging area of the run-time replica count if that is larger.
template <int NREP>
int mean_lds(const MeanLaunch &a) {
    const int staged = a.n_replicas > kRegReps ? a.n_replicas - kRegReps : 0;
    const int need = NREP == 0 && a.partials ? staged * stage_threads(staged) * 16 : 0;
    return a.lds_pad > need ? a.lds_pad : need;
}

template <int NREP>
int launch_mean16_n(const MeanArgs &ma, const MeanLaunch &a, void *stream) {
    if (a.partials) return launch(mean_kernel<NREP, true, true, true>, a.n_chunks, stream, mean_lds<NREP>(a), ma);
    return launch(mean_kernel<NREP, false, true, true>, a.n_chunks, stream, a.lds_pad, ma);
}

template <int NREP>
int launch_mean_n(const MeanArgs &ma, const MeanLaunch &a, void *stream) {
    if (a.partials) return a.nontemporal ? launch(mean_kernel<NREP, true, true>, a.n_chunks, stream, mean_lds<NREP>(a), ma) : launch(mean_kernel<NREP, true, false>, a.n_chunks, stream, mean_lds<NREP>(a), ma);
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

int launch_mean(const MeanLaunch &a, void *stream) {
    MeanArgs ma{};
    for (int k = 0; k < a.n_replicas; ++k) ma.x[k] = a.x[k];
    ma.out = a.out;
    ma.chunks = a.chunks;
    ma.partials = a.partials;
    ma.inv_n = a.inv_n;
    ma.n = a.n_replicas;
    ma.stage_threads = stage_threads(a.n_replicas > kRegReps ? a.n_replicas - kRegReps : 0);   // the replicas beyond the registers are staged
    int rc;
    if (a.wire16) {
        switch (a.n_replicas) {
            case 2: rc = launch_mean16_n<2>(ma, a, stream); break;
            case 4: rc = launch_mean16_n<4>(ma, a, stream); break;
            case 8: rc = launch_mean16_n<8>(ma, a, stream); break;
            case 16: rc = launch_mean16_n<16>(ma, a, stream); break;
            case 32: rc = launch_mean16_n<32>(ma, a, stream); break;
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
            case 9: rc = launch_mean_n<9>(ma, a, stream); break;
            case 10: rc = launch_mean_n<10>(ma, a, stream); break;
            case 11: rc = launch_mean_n<11>(ma, a, stream); break;
            case 12: rc = launch_mean_n<12>(ma, a, stream); break;
            case 13: rc = launch_mean_n<13>(ma, a, stream); break;
            case 14: rc = launch_mean_n<14>(ma, a, stream); break;
            case 15: rc = launch_mean_n<15>(ma, a, stream); break;
            case 16: rc = launch_mean_n<16>(ma, a, stream); break;
            case 32: rc = launch_mean_n<32>(ma, a, stream); break;
            default: rc = launch_mean_n<0>(ma, a, stream); break;
        }
    }
    if (rc != 0 || !a.partials) return rc;
    return launch_stats(a.partials, a.slice_sums, a.layer_ranges, a.n_layers, a.n_replicas, a.stats, a.max_partials_per_layer, stream);
}

}  // namespace ddp
