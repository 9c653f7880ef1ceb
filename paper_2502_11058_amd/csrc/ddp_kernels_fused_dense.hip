// fused synchronisation + update over dense arenas (table-free).
#include "ddp_device.h"

namespace ddp {
namespace {

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

}  // namespace

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

bool fused_dense_supports(int n_replicas) { return n_replicas == 2 || n_replicas == 4 || n_replicas == 8 || n_replicas == 16 || n_replicas == 32; }

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
            case 2: return launch_fused_dense_n<A, G, M, 2>(f, fa, grid, stream);                       \
            case 4: return launch_fused_dense_n<A, G, M, 4>(f, fa, grid, stream);                       \
            case 8: return launch_fused_dense_n<A, G, M, 8>(f, fa, grid, stream);                       \
            case 16: return launch_fused_dense_n<A, G, M, 16>(f, fa, grid, stream);                     \
            case 32: return launch_fused_dense_n<A, G, M, 32>(f, fa, grid, stream);                     \
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

}  // namespace ddp
