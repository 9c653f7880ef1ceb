// local update (Eq. (5), first case): table-driven and table-free kernels.
#include "ddp_device.h"

namespace ddp {
namespace {

template <bool ADAM, bool GBF16, bool MODEL, bool NT>
__global__ __launch_bounds__(kThreads) void update_kernel(const TensorDesc *__restrict__ tensors, const UpdateChunk *__restrict__ chunks,
                                                          const UpdateScalars s) {
    const UpdateChunk ch = chunks[blockIdx.x];
    const TensorDesc td = tensors[ch.tensor];
    update_chunk_body<ADAM, GBF16, MODEL, NT>(td, ch, s);
}

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

}  // namespace

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

}  // namespace ddp
