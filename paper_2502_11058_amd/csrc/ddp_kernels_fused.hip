// fused synchronisation + update, table-driven (both cases of Eq. (5) in one pass).
//
// Compiled twice, once per optimizer (-DDDP_FUSED_ADAM=0: SGD with momentum, =1: AdamW), so that the two halves of the
// kernel's instantiations build in parallel; the first half also holds the dispatcher.
#include "ddp_device.h"

#ifndef DDP_FUSED_ADAM
#error "compile with -DDDP_FUSED_ADAM=0 or -DDDP_FUSED_ADAM=1"
#endif

namespace ddp {
namespace {

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
    int stage_threads;  // run-time replica count with statistics: threads that take part in the vector loop
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
            // run-time replica count; with statistics the terms beyond the first kRegReps are parked in LDS (see
            // stage_threads) so that the peers are fetched once; only the first `vt` threads take part (all of them
            // up to 32 replicas)
            extern __shared__ __align__(16) unsigned char dyn_lds[];
            f32x4 *stage = reinterpret_cast<f32x4 *>(dyn_lds);
            const int vt = STATS ? a.stage_threads : kThreads;
            for (int v = tid; v < nv && tid < vt; v += vt) {
                f32x4 pl = ld<NT>(p4 + v);
                const gvec gv = ld<NT>(g4 + v);
                f32x4 av = ld<NT>(a4 + v);
                f32x4 bv{};
                if constexpr (ADAM) bv = ld<NT>(b4 + v);
                if constexpr (UTS) step4(gv, pl, av, bv);
                f32x4 loc = pl;
                if constexpr (W16) loc = bf16_widen4(bf16_rne4(pl));
                auto term = [&](int k) -> f32x4 { return k == lr ? loc : wire4<W16, NT>(a.x[k], vfo + v); };
                // the first kRegReps terms of the rank-order sum stay in registers, the rest are parked in LDS
                f32x4 r[kRegReps];
#pragma unroll
                for (int k = 0; k < kRegReps; ++k)
                    if (k < nrep) r[k] = term(k);
                f32x4 acc = r[0];
#pragma unroll
                for (int k = 1; k < kRegReps; ++k)
                    if (k < nrep) acc = acc + r[k];
                for (int k0 = kRegReps; k0 < nrep; k0 += 8) {  // eight more peers in flight, then park and add them in rank order
                    f32x4 x[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (k0 + j < nrep) x[j] = term(k0 + j);
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (k0 + j < nrep) {
                            if constexpr (STATS) stage[(k0 + j - kRegReps) * vt + tid] = x[j];
                            acc = acc + x[j];
                        }
                }
                f32x4 m = acc * inv_n;
                if constexpr (STATS) {
#pragma unroll
                    for (int k = 0; k < kRegReps; ++k)
                        if (k < nrep) stats4(m, r[k]);
                    for (int k = kRegReps; k < nrep; ++k) stats4(m, stage[(k - kRegReps) * vt + tid]);
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

}  // namespace

template <bool A, bool G, bool M, int NR>
static int launch_fused_n(const FusedLaunch &f, const FusedArgs &fa, void *stream) {
    const bool st = f.partials != nullptr;
    // dynamic LDS: the residency pad, or the staging area of the run-time replica count if that is larger
    const int staged = f.n_replicas > kRegReps ? f.n_replicas - kRegReps : 0;
    const int need = NR == 0 && st ? staged * stage_threads(staged) * 16 : 0;
    const int lds = f.lds_pad > need ? f.lds_pad : need;
#define DDP_FUSED(W, U)                                                                                \
    return st ? launch(fused_kernel<A, G, M, NR, true, W, U>, f.n_chunks, stream, lds, fa)             \
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
        case 2: return launch_fused_n<A, G, M, 2>(f, fa, stream);
        case 4: return launch_fused_n<A, G, M, 4>(f, fa, stream);
        case 8: return launch_fused_n<A, G, M, 8>(f, fa, stream);
        case 16: return launch_fused_n<A, G, M, 16>(f, fa, stream);
        case 32: return launch_fused_n<A, G, M, 32>(f, fa, stream);
        default: return launch_fused_n<A, G, M, 0>(f, fa, stream);
    }
}

#if DDP_FUSED_ADAM
#define DDP_FUSED_HALF launch_fused_adamw
#else
#define DDP_FUSED_HALF launch_fused_sgdm
#endif

// The kernel launch of this file's optimizer (no statistics reduction).
int DDP_FUSED_HALF(const FusedLaunch &f, void *stream) {
    constexpr bool A = DDP_FUSED_ADAM != 0;
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
    fa.stage_threads = stage_threads(f.n_replicas > kRegReps ? f.n_replicas - kRegReps : 0);   // only the terms beyond the registers are staged
    const bool gb = f.grad_dtype == DDP_BF16, md = f.with_model;
    if (!gb && !md) return launch_fused_t<A, false, false>(f, fa, stream);
    if (!gb && md) return launch_fused_t<A, false, true>(f, fa, stream);
    if (gb && !md) return launch_fused_t<A, true, false>(f, fa, stream);
    return launch_fused_t<A, true, true>(f, fa, stream);
}

#if !DDP_FUSED_ADAM
int launch_fused_adamw(const FusedLaunch &f, void *stream);

int launch_fused(const FusedLaunch &f, void *stream) {
    const int rc = f.kind == DDP_OPT_ADAMW ? launch_fused_adamw(f, stream) : launch_fused_sgdm(f, stream);
    if (rc != 0 || !f.partials) return rc;
    return launch_stats(f.partials, f.slice_sums, f.layer_ranges, f.n_layers, f.n_replicas, f.stats, f.max_partials_per_layer, stream);
}
#endif

}  // namespace ddp
