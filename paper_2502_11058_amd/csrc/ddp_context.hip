// Host side of the library: context, model registration, per-slot offset tables, argument checks and the four
// per-iteration entry points (Algorithm 1 of the paper, one worker).  Kernels live in ddp_kernels.hip.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <exception>
#include <new>
#include <string>
#include <vector>

#include "ddp_internal.h"

namespace ddp {

static thread_local std::string g_err;

int fail(const ddp_ctx *ctx, int code, const std::string &msg) {
    if (ctx)
        ctx->err = msg;
    else
        g_err = msg;
    return code;
}

static int hip_fail(const ddp_ctx *ctx, hipError_t e, const char *what) {
    return fail(ctx, DDP_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

template <class T>
static int upload(const ddp_ctx *ctx, const std::vector<T> &host, T **dev) {
    *dev = nullptr;
    if (host.empty()) return DDP_OK;
    hipError_t e = hipMalloc((void **)dev, host.size() * sizeof(T));
    if (e != hipSuccess) {
        *dev = nullptr;
        return fail(ctx, DDP_ENOMEM, std::string("hipMalloc of a table failed: ") + hipGetErrorString(e));
    }
    e = hipMemcpy(*dev, host.data(), host.size() * sizeof(T), hipMemcpyHostToDevice);
    if (e != hipSuccess) return hip_fail(ctx, e, "hipMemcpy of a table");
    return DDP_OK;
}

static void free_slot(SlotTables &s) {
    if (s.d_copy) (void)hipFree(s.d_copy);
    if (s.d_mean) (void)hipFree(s.d_mean);
    if (s.d_layer_ranges) (void)hipFree(s.d_layer_ranges);
    if (s.d_tensor_flat_off) (void)hipFree(s.d_tensor_flat_off);
    if (s.d_fused_ranges) (void)hipFree(s.d_fused_ranges);
    if (s.d_dense_ranges) (void)hipFree(s.d_dense_ranges);
    s.d_dense_ranges = nullptr;
    s.d_copy = nullptr;
    s.d_mean = nullptr;
    s.d_layer_ranges = nullptr;
    s.d_tensor_flat_off = nullptr;
    s.d_fused_ranges = nullptr;
}

static void drop_schedule(ddp_ctx *c) {
    for (auto &s : c->slots) free_slot(s);
    c->slots.clear();
    c->H = 0;
    if (c->d_partials) (void)hipFree(c->d_partials);
    c->d_partials = nullptr;
    c->d_slice_sums = nullptr;
    c->partials_cap = 0;
}

static void drop_model(ddp_ctx *c) {
    drop_schedule(c);
    if (c->d_tensors) (void)hipFree(c->d_tensors);
    if (c->d_update) (void)hipFree(c->d_update);
    if (c->d_tensor_chunk_base) (void)hipFree(c->d_tensor_chunk_base);
    c->d_tensor_chunk_base = nullptr;
    c->d_tensors = nullptr;
    c->d_update = nullptr;
    c->n_update = 0;
    c->registered = false;
}

static int check_device(const ddp_ctx *c, const char *who) {
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return hip_fail(c, e, "hipGetDevice");
    if (cur != c->device)
        return fail(c, DDP_ESTATE, std::string(who) + ": current device " + std::to_string(cur) + " is not the context's device " +
                                       std::to_string(c->device));
    return DDP_OK;
}

// Launchers hand back the hipError_t of the launch (0 = success).
static int after_launch(const ddp_ctx *c, const char *who, int hip_rc) {
    if (hip_rc == 0) return DDP_OK;
    return fail(c, DDP_EHIP, std::string(who) + ": kernel launch failed: " + hipGetErrorString((hipError_t)hip_rc));
}

// Dispatch order of a chunk table.  Workgroups are handed to the 8 XCDs round-robin in launch order, and the
// resident workgroups of a launch form a moving window over the table.  With `ways` > 1 the table is cut into
// `ways` contiguous segments and launch position j takes entry j / ways of segment j % ways: the window then
// covers `ways` far-apart regions of every stream at once instead of one contiguous region, and with ways a
// multiple of 8 each XCD walks its own segments front to back.
template <class T>
static void interleave_segments(std::vector<T> &v, int ways) {
    const size_t n = v.size();
    if (ways <= 1 || n < (size_t)ways * 2) return;
    const size_t seg = (n + (size_t)ways - 1) / (size_t)ways;
    std::vector<T> out;
    out.reserve(n);
    for (size_t i = 0; i < seg; ++i)
        for (size_t s = 0; s < (size_t)ways; ++s) {
            const size_t idx = s * seg + i;
            if (idx < n) out.push_back(v[idx]);
        }
    v.swap(out);
}

// Bytes of dynamic LDS a workgroup has to request (without using them) so that at most `wg_per_cu` workgroups of a
// kernel with a few hundred bytes of static LDS are resident on a CU; 0 = no cap.  A request cannot exceed the
// per-workgroup limit, so the smallest residency that can be enforced is ceil(LDS per CU / that limit).
static int residency_pad(const ddp_ctx *c, int wg_per_cu) {
    if (wg_per_cu <= 0) return 0;
    int pad = c->lds_per_cu / wg_per_cu - 1024;      // room for the kernels' own static LDS and allocation granularity
    pad = pad / 512 * 512;
    const int cap = (c->lds_per_wg_max < 65536 ? c->lds_per_wg_max : 65536) - 1024;  // requests beyond 64 KiB are never made
    if (pad > cap) pad = cap / 512 * 512;
    return pad > 0 ? pad : 0;
}

static bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

}  // namespace ddp

using namespace ddp;

extern "C" const char *ddp_last_error(const ddp_ctx *ctx) { return ctx ? ctx->err.c_str() : g_err.c_str(); }

extern "C" int ddp_create(ddp_ctx **out, int device) {
    if (!out) return fail(nullptr, DDP_EINVAL, "ddp_create: out is NULL");
    *out = nullptr;
    int n = 0;
    hipError_t e = hipGetDeviceCount(&n);
    if (e != hipSuccess) return hip_fail(nullptr, e, "ddp_create: hipGetDeviceCount");
    if (device < 0 || device >= n) return fail(nullptr, DDP_EINVAL, "ddp_create: no such device " + std::to_string(device));
    e = hipSetDevice(device);
    if (e != hipSuccess) return hip_fail(nullptr, e, "ddp_create: hipSetDevice");
    ddp_ctx *c = new (std::nothrow) ddp_ctx();
    if (!c) return fail(nullptr, DDP_ENOMEM, "ddp_create: out of host memory");
    c->device = device;
    // Residency caps are stated in workgroups per CU and turned into an LDS request from what this device reports, so
    // that a part with another LDS size keeps the same residency.
    int lds_cu = 0, lds_wg = 0;
    if (hipDeviceGetAttribute(&lds_cu, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, device) == hipSuccess && lds_cu > 0 &&
        hipDeviceGetAttribute(&lds_wg, hipDeviceAttributeMaxSharedMemoryPerBlock, device) == hipSuccess && lds_wg > 0) {
        c->lds_per_cu = lds_cu;
        c->lds_per_wg_max = lds_wg;
    }
    c->update_lds = residency_pad(c, 2);
    c->mean_lds = residency_pad(c, 2);
    c->copy_lds = residency_pad(c, 6);
    // the device address of the library's fixed scratch array, resolved here once per device (the device is current)
    // (a failure only disables ddp_partial_average_static, which then reports it; everything else works without the array)
    if (static_scratch_for(nullptr, device, &c->static_scratch) != DDP_OK) {
        c->static_scratch = nullptr;
        c->static_scratch_err = g_err;
    }
    *out = c;
    return DDP_OK;
}

extern "C" int ddp_destroy(ddp_ctx *ctx) {
    if (!ctx) return DDP_OK;
    drop_model(ctx);
    delete ctx;
    return DDP_OK;
}

extern "C" int ddp_set_option(ddp_ctx *ctx, const char *name, int64_t value) {
    return guarded(ctx, [&]() -> int {
        if (!ctx || !name) return fail(ctx, DDP_EINVAL, "ddp_set_option: NULL argument");
        std::string k(name);
        auto chunk_ok = [&](int64_t v) { return v >= 1024 && v <= 1048576 && v % 1024 == 0; };
        if (k == "update_chunk" || k == "mean_chunk" || k == "copy_chunk") {
            if (!chunk_ok(value)) return fail(ctx, DDP_EINVAL, "ddp_set_option: chunk must be a multiple of 1024 in [1024, 1048576]");
            if (ctx->registered) return fail(ctx, DDP_ESTATE, "ddp_set_option: chunk sizes must be set before ddp_register_model");
            (k == "update_chunk" ? ctx->update_chunk : k == "mean_chunk" ? ctx->mean_chunk : ctx->copy_chunk) = value;
            return DDP_OK;
        }
        if (k == "dispatch_ways") {
            if (value < 1 || value > 4096) return fail(ctx, DDP_EINVAL, "ddp_set_option: dispatch_ways must be in [1, 4096]");
            if (ctx->registered) return fail(ctx, DDP_ESTATE, "ddp_set_option: dispatch_ways must be set before ddp_register_model");
            ctx->dispatch_ways = (int)value;
            return DDP_OK;
        }
        if (k == "update_wg_per_cu" || k == "mean_wg_per_cu" || k == "copy_wg_per_cu") {
            if (value < 0 || value > 32) return fail(ctx, DDP_EINVAL, "ddp_set_option: workgroups per CU must be in [0, 32] (0 = no cap)");
            (k == "update_wg_per_cu" ? ctx->update_lds : k == "mean_wg_per_cu" ? ctx->mean_lds : ctx->copy_lds) = residency_pad(ctx, (int)value);
            return DDP_OK;
        }
        if (k == "update_lds" || k == "mean_lds" || k == "copy_lds") {
            if (value < 0 || value > 65536) return fail(ctx, DDP_EINVAL, "ddp_set_option: LDS pad must be in [0, 65536] bytes");
            (k == "update_lds" ? ctx->update_lds : k == "mean_lds" ? ctx->mean_lds : ctx->copy_lds) = (int)value;
            return DDP_OK;
        }
        if (k == "dense_path") {
            if (value != 0 && value != 1) return fail(ctx, DDP_EINVAL, "ddp_set_option: dense_path is 0 or 1");
            ctx->dense_path = value != 0;
            return DDP_OK;
        }
        if (k == "nontemporal") {
            if (value != 0 && value != 1) return fail(ctx, DDP_EINVAL, "ddp_set_option: nontemporal is 0 or 1");
            ctx->nontemporal = value != 0;
            return DDP_OK;
        }
        return fail(ctx, DDP_EINVAL, "ddp_set_option: unknown option " + k);
    });
}

extern "C" int ddp_register_model(ddp_ctx *ctx, int L, int T, const int32_t *layer_of, const int64_t *numel, int param_dtype,
                                  int grad_dtype, void *const *sync_ptr, void *const *model_ptr, void *const *grad_ptr,
                                  void *const *state0_ptr, void *const *state1_ptr) {
    try {
        if (!ctx) return fail(nullptr, DDP_EINVAL, "ddp_register_model: ctx is NULL");
        if (L < 1 || T < L) return fail(ctx, DDP_EINVAL, "ddp_register_model: need L >= 1 and T >= L");
        if (!layer_of || !numel || !sync_ptr || !grad_ptr || !state0_ptr) return fail(ctx, DDP_EINVAL, "ddp_register_model: NULL array");
        if (param_dtype != DDP_F32 && param_dtype != DDP_BF16) return fail(ctx, DDP_EINVAL, "ddp_register_model: bad param_dtype");
        if (grad_dtype != DDP_F32 && grad_dtype != DDP_BF16) return fail(ctx, DDP_EINVAL, "ddp_register_model: bad grad_dtype");
        if (param_dtype == DDP_BF16 && !model_ptr) return fail(ctx, DDP_EINVAL, "ddp_register_model: bf16 params need model_ptr");
        int rc = check_device(ctx, "ddp_register_model");
        if (rc != DDP_OK) return rc;

        std::vector<TensorDesc> ts((size_t)T);
        std::vector<int32_t> first((size_t)L + 1, 0);
        const uintptr_t galign = grad_dtype == DDP_F32 ? 4 : 2;
        for (int t = 0; t < T; ++t) {
            const std::string tn = "tensor " + std::to_string(t);
            if (layer_of[t] < 0 || layer_of[t] >= L) return fail(ctx, DDP_EINVAL, "ddp_register_model: " + tn + " has a layer id out of range");
            if (t == 0 ? layer_of[t] != 0 : (layer_of[t] != layer_of[t - 1] && layer_of[t] != layer_of[t - 1] + 1))
                return fail(ctx, DDP_EINVAL, "ddp_register_model: layer_of must be non-decreasing and cover 0..L-1 (" + tn + ")");
            if (numel[t] <= 0) return fail(ctx, DDP_ESHAPE, "ddp_register_model: " + tn + " has numel <= 0");
            if (!sync_ptr[t] || !grad_ptr[t] || !state0_ptr[t]) return fail(ctx, DDP_EINVAL, "ddp_register_model: " + tn + " has a NULL pointer");
            if (param_dtype == DDP_BF16 && !model_ptr[t]) return fail(ctx, DDP_EINVAL, "ddp_register_model: " + tn + " lacks its bf16 model copy");
            if (!aligned(sync_ptr[t], 4) || !aligned(state0_ptr[t], 4) || !aligned(grad_ptr[t], galign) ||
                (state1_ptr && state1_ptr[t] && !aligned(state1_ptr[t], 4)) ||
                (param_dtype == DDP_BF16 && !aligned(model_ptr[t], 2)))
                return fail(ctx, DDP_EALIGN, "ddp_register_model: " + tn + " is not aligned to its element type");
            TensorDesc &d = ts[(size_t)t];
            d.sync = (float *)sync_ptr[t];
            d.model = param_dtype == DDP_BF16 ? (uint16_t *)model_ptr[t] : nullptr;
            d.grad = grad_ptr[t];
            d.state0 = (float *)state0_ptr[t];
            d.state1 = state1_ptr ? (float *)state1_ptr[t] : nullptr;
            d.numel = numel[t];
            first[(size_t)layer_of[t] + 1] = t + 1;
        }
        if (layer_of[T - 1] != L - 1) return fail(ctx, DDP_EINVAL, "ddp_register_model: layer_of does not reach L-1");
        bool has1 = state1_ptr != nullptr;
        if (has1)
            for (int t = 0; t < T; ++t) has1 = has1 && state1_ptr[t] != nullptr;

        drop_model(ctx);
        ctx->L = L;
        ctx->T = T;
        ctx->param_dtype = param_dtype;
        ctx->grad_dtype = grad_dtype;
        ctx->has_state1 = has1;
        ctx->layer_of.assign(layer_of, layer_of + T);
        ctx->numel.assign(numel, numel + T);
        ctx->tensors = ts;
        ctx->layer_first_tensor = first;
        // Dense arenas: every tensor starts where the previous one ends, in every stream, and the streams start on
        // 128-bit (bf16: 64-bit) boundaries.  The update then needs no table.
        ctx->tensor_elem_off.assign((size_t)T + 1, 0);
        for (int t = 0; t < T; ++t) ctx->tensor_elem_off[(size_t)t + 1] = ctx->tensor_elem_off[(size_t)t] + numel[t];
        const uintptr_t gsz = grad_dtype == DDP_F32 ? 4 : 2;
        bool dense = aligned(ts[0].sync, 16) && aligned(ts[0].state0, 16) && aligned(ts[0].grad, 4 * gsz) &&
                     (!has1 || aligned(ts[0].state1, 16)) && (param_dtype != DDP_BF16 || aligned(ts[0].model, 8));
        for (int t = 1; t < T && dense; ++t) {
            const TensorDesc &a = ts[(size_t)t - 1], &b = ts[(size_t)t];
            dense = b.sync == a.sync + a.numel && b.state0 == a.state0 + a.numel && (!has1 || b.state1 == a.state1 + a.numel) &&
                    (const char *)b.grad == (const char *)a.grad + (uintptr_t)a.numel * gsz &&
                    (param_dtype != DDP_BF16 || b.model == a.model + a.numel);
        }
        ctx->dense = dense;

        // update table: every tensor cut into runs of update_chunk elements
        std::vector<UpdateChunk> uc;
        ctx->tensor_chunk_base.assign((size_t)T + 1, 0);
        for (int t = 0; t < T; ++t) {
            ctx->tensor_chunk_base[(size_t)t] = (int32_t)uc.size();
            for (int64_t b = 0; b < numel[t]; b += ctx->update_chunk) {
                int64_t n = std::min<int64_t>(ctx->update_chunk, numel[t] - b);
                uc.push_back({b, t, (int32_t)n});
            }
        }
        if (uc.size() > (size_t)0x7fffffff) {
            drop_model(ctx);
            return fail(ctx, DDP_ESHAPE, "ddp_register_model: more than 2^31-1 update chunks; raise update_chunk");
        }
        ctx->tensor_chunk_base[(size_t)T] = (int32_t)uc.size();
        ctx->n_update = (int64_t)uc.size();
        interleave_segments(uc, ctx->dispatch_ways);
        rc = upload(ctx, ts, &ctx->d_tensors);
        if (rc == DDP_OK) rc = upload(ctx, uc, &ctx->d_update);
        if (rc == DDP_OK) rc = upload(ctx, ctx->tensor_chunk_base, &ctx->d_tensor_chunk_base);
        if (rc != DDP_OK) {
            drop_model(ctx);
            return rc;
        }
        ctx->n_update = (int64_t)uc.size();
        ctx->registered = true;
        return DDP_OK;
    } catch (...) {
        return fail_nothrow(ctx, DDP_ENOMEM, "ddp_register_model: host allocation failed");
    }
}

extern "C" int ddp_set_schedule(ddp_ctx *ctx, int H, const int32_t *set_ptr, const int32_t *set_layers) {
    try {
        if (!ctx) return fail(nullptr, DDP_EINVAL, "ddp_set_schedule: ctx is NULL");
        if (!ctx->registered) return fail(ctx, DDP_ESTATE, "ddp_set_schedule: no model registered");
        if (H < 1 || !set_ptr || !set_layers) return fail(ctx, DDP_EINVAL, "ddp_set_schedule: bad argument");
        if (set_ptr[0] != 0) return fail(ctx, DDP_ESCHED, "ddp_set_schedule: set_ptr[0] must be 0");
        int rc = check_device(ctx, "ddp_set_schedule");
        if (rc != DDP_OK) return rc;
        for (int s = 0; s < H; ++s) {
            if (set_ptr[s + 1] < set_ptr[s]) return fail(ctx, DDP_ESCHED, "ddp_set_schedule: set_ptr is not monotone");
            std::vector<char> seen((size_t)ctx->L, 0);
            for (int j = set_ptr[s]; j < set_ptr[s + 1]; ++j) {
                int l = set_layers[j];
                if (l < 0 || l >= ctx->L) return fail(ctx, DDP_ESCHED, "ddp_set_schedule: layer id out of range in slot " + std::to_string(s));
                if (seen[(size_t)l]) return fail(ctx, DDP_ESCHED, "ddp_set_schedule: layer " + std::to_string(l) + " listed twice in slot " + std::to_string(s));
                seen[(size_t)l] = 1;
            }
        }

        drop_schedule(ctx);
        std::vector<SlotTables> slots((size_t)H);
        // workgroups of the table-free fused kernel, layer by layer in registration order (never more than the update
        // table has chunks, so the reduction scratch sized for the table covers them)
        std::vector<int64_t> dense_wg_base((size_t)ctx->L + 1, 0);
        for (int l = 0; l < ctx->L; ++l) {
            const int64_t n = ctx->tensor_elem_off[(size_t)ctx->layer_first_tensor[(size_t)l + 1]] -
                              ctx->tensor_elem_off[(size_t)ctx->layer_first_tensor[(size_t)l]];
            dense_wg_base[(size_t)l + 1] = dense_wg_base[(size_t)l] + (n + ctx->update_chunk - 1) / ctx->update_chunk;
        }
        int64_t max_mean_chunks = 0;
        for (int s = 0; s < H; ++s) {
            SlotTables &st = slots[(size_t)s];
            st.layer_pos.assign((size_t)ctx->L, -1);
            std::vector<CopyChunk> cc;
            std::vector<MeanChunk> mc;
            std::vector<int32_t> lcp, fused_ranges;
            std::vector<int64_t> tflat((size_t)ctx->T, -1);
            int64_t off = 0;
            for (int j = set_ptr[s]; j < set_ptr[s + 1]; ++j) {
                const int l = set_layers[j];
                st.layers.push_back(l);
                st.layer_begin.push_back(off);
                lcp.push_back((int32_t)mc.size());
                fused_ranges.push_back(ctx->tensor_chunk_base[(size_t)ctx->layer_first_tensor[(size_t)l]]);
                fused_ranges.push_back(ctx->tensor_chunk_base[(size_t)ctx->layer_first_tensor[(size_t)l + 1]]);
                st.layer_pos[(size_t)l] = (int32_t)st.layers.size() - 1;
                st.dense_ranges.push_back((int32_t)dense_wg_base[(size_t)l]);
                st.dense_ranges.push_back((int32_t)dense_wg_base[(size_t)l + 1]);
                const int64_t layer_start = off;
                for (int t = ctx->layer_first_tensor[(size_t)l]; t < ctx->layer_first_tensor[(size_t)l + 1]; ++t) {
                    st.tensors.push_back(t);
                    st.tensor_off.push_back(off);
                    tflat[(size_t)t] = off;
                    for (int64_t b = 0; b < ctx->numel[(size_t)t]; b += ctx->copy_chunk) {
                        int64_t n = std::min<int64_t>(ctx->copy_chunk, ctx->numel[(size_t)t] - b);
                        cc.push_back({b, off + b, t, (int32_t)n});
                    }
                    off += ctx->numel[(size_t)t];
                }
                // mean chunks: cut the layer's flat range at multiples of mean_chunk measured from a 4-element
                // boundary, so that every chunk but the first starts 16-byte aligned
                int64_t b = layer_start;
                while (b < off) {
                    int64_t e = std::min<int64_t>(off, (b / 4) * 4 + ctx->mean_chunk);
                    mc.push_back({b, (int32_t)(e - b), (int32_t)mc.size()});
                    b = e;
                }
            }
            st.layer_begin.push_back(off);
            lcp.push_back((int32_t)mc.size());
            if (mc.size() > (size_t)0x7fffffff || cc.size() > (size_t)0x7fffffff) {
                for (auto &x : slots) free_slot(x);
                return fail(ctx, DDP_ESHAPE, "ddp_set_schedule: more than 2^31-1 chunks in a slot; raise mean_chunk / copy_chunk");
            }
            st.numel = off;
            st.n_copy = (int64_t)cc.size();
            st.n_mean = (int64_t)mc.size();
            max_mean_chunks = std::max(max_mean_chunks, st.n_mean);
            interleave_segments(cc, ctx->dispatch_ways);
            interleave_segments(mc, ctx->dispatch_ways);
            rc = upload(ctx, cc, &st.d_copy);
            if (rc == DDP_OK) rc = upload(ctx, mc, &st.d_mean);
            std::vector<int32_t> mean_ranges;
            for (size_t i = 0; i + 1 < lcp.size(); ++i) {
                mean_ranges.push_back(lcp[i]);
                mean_ranges.push_back(lcp[i + 1]);
                st.max_mean_partials = std::max<int64_t>(st.max_mean_partials, lcp[i + 1] - lcp[i]);
            }
            for (size_t i = 0; i + 1 < fused_ranges.size(); i += 2) {
                st.max_fused_partials = std::max<int64_t>(st.max_fused_partials, fused_ranges[i + 1] - fused_ranges[i]);
                st.max_dense_partials = std::max<int64_t>(st.max_dense_partials, st.dense_ranges[i + 1] - st.dense_ranges[i]);
            }
            if (rc == DDP_OK) rc = upload(ctx, mean_ranges, &st.d_layer_ranges);
            if (rc == DDP_OK) rc = upload(ctx, tflat, &st.d_tensor_flat_off);
            if (rc == DDP_OK) rc = upload(ctx, fused_ranges, &st.d_fused_ranges);
            if (rc == DDP_OK) rc = upload(ctx, st.dense_ranges, &st.d_dense_ranges);
            if (rc != DDP_OK) {
                for (auto &x : slots) free_slot(x);
                return rc;
            }
        }
        max_mean_chunks = std::max(max_mean_chunks, ctx->n_update);  // the fused step keeps one partial per update chunk
        if (max_mean_chunks > 0) {
            hipError_t e = hipMalloc((void **)&ctx->d_partials, ((size_t)max_mean_chunks + (size_t)ctx->L * kStatSlices) * 2 * sizeof(double));
            if (e != hipSuccess) {
                ctx->d_partials = nullptr;
                for (auto &x : slots) free_slot(x);
                return fail(ctx, DDP_ENOMEM, std::string("ddp_set_schedule: hipMalloc of the reduction scratch failed: ") + hipGetErrorString(e));
            }
            ctx->partials_cap = max_mean_chunks;
            ctx->d_slice_sums = ctx->d_partials + 2 * max_mean_chunks;
        }
        ctx->slots = std::move(slots);
        ctx->H = H;
        return DDP_OK;
    } catch (...) {
        return fail_nothrow(ctx, DDP_ENOMEM, "ddp_set_schedule: host allocation failed");
    }
}

static const SlotTables *slot_of(const ddp_ctx *ctx, int slot, const char *who, int *rc) {
    if (!ctx) {
        *rc = fail(nullptr, DDP_EINVAL, std::string(who) + ": ctx is NULL");
        return nullptr;
    }
    if (ctx->H == 0) {
        *rc = fail(ctx, DDP_ESCHED, std::string(who) + ": no schedule installed");
        return nullptr;
    }
    if (slot < 0 || slot >= ctx->H) {
        *rc = fail(ctx, DDP_EINVAL, std::string(who) + ": slot out of range");
        return nullptr;
    }
    *rc = DDP_OK;
    return &ctx->slots[(size_t)slot];
}

extern "C" int64_t ddp_slot_numel(const ddp_ctx *ctx, int slot) {
    int rc;
    const SlotTables *s = slot_of(ctx, slot, "ddp_slot_numel", &rc);
    return s ? s->numel : -(int64_t)rc;
}

extern "C" int ddp_slot_num_layers(const ddp_ctx *ctx, int slot) {
    int rc;
    const SlotTables *s = slot_of(ctx, slot, "ddp_slot_num_layers", &rc);
    return s ? (int)s->layers.size() : -rc;
}

extern "C" int ddp_slot_num_tensors(const ddp_ctx *ctx, int slot) {
    int rc;
    const SlotTables *s = slot_of(ctx, slot, "ddp_slot_num_tensors", &rc);
    return s ? (int)s->tensors.size() : -rc;
}

extern "C" int ddp_slot_layout(const ddp_ctx *ctx, int slot, int32_t *out_tensor_ids, int64_t *out_off, int32_t *out_layer_ids,
                               int64_t *out_layer_begin) {
    int rc;
    const SlotTables *s = slot_of(ctx, slot, "ddp_slot_layout", &rc);
    if (!s) return rc;
    if (out_tensor_ids) std::memcpy(out_tensor_ids, s->tensors.data(), s->tensors.size() * sizeof(int32_t));
    if (out_off) std::memcpy(out_off, s->tensor_off.data(), s->tensor_off.size() * sizeof(int64_t));
    if (out_layer_ids) std::memcpy(out_layer_ids, s->layers.data(), s->layers.size() * sizeof(int32_t));
    if (out_layer_begin) std::memcpy(out_layer_begin, s->layer_begin.data(), s->layer_begin.size() * sizeof(int64_t));
    return DDP_OK;
}

static int check_flat(const ddp_ctx *ctx, const void *p, const char *who, const char *what) {
    if (!p) return fail(ctx, DDP_EINVAL, std::string(who) + ": " + what + " is NULL");
    if (!aligned(p, 16)) return fail(ctx, DDP_EALIGN, std::string(who) + ": " + what + " must be 16-byte aligned");
    return DDP_OK;
}

extern "C" int ddp_pack(ddp_ctx *ctx, int slot, float *flat_local, void *stream) {
    return guarded(ctx, [&]() -> int {
        int rc;
        const SlotTables *s = slot_of(ctx, slot, "ddp_pack", &rc);
        if (!s) return rc;
        if ((rc = check_device(ctx, "ddp_pack")) != DDP_OK) return rc;
        if (s->numel == 0) return DDP_OK;
        if ((rc = check_flat(ctx, flat_local, "ddp_pack", "flat_local")) != DDP_OK) return rc;
        rc = launch_copy(false, ctx->d_tensors, s->d_copy, s->n_copy, flat_local, false, ctx->nontemporal, ctx->copy_lds, stream);
        return after_launch(ctx, "ddp_pack", rc);
    });
}

extern "C" int ddp_unpack(ddp_ctx *ctx, int slot, const float *flat, void *stream) {
    return guarded(ctx, [&]() -> int {
        int rc;
        const SlotTables *s = slot_of(ctx, slot, "ddp_unpack", &rc);
        if (!s) return rc;
        if ((rc = check_device(ctx, "ddp_unpack")) != DDP_OK) return rc;
        if (s->numel == 0) return DDP_OK;
        if ((rc = check_flat(ctx, flat, "ddp_unpack", "flat")) != DDP_OK) return rc;
        rc = launch_copy(true, ctx->d_tensors, s->d_copy, s->n_copy, const_cast<float *>(flat), ctx->param_dtype == DDP_BF16,
                         ctx->nontemporal, ctx->copy_lds, stream);
        return after_launch(ctx, "ddp_unpack", rc);
    });
}

// Shared body of the two averaging entry points; `who` names the caller in messages.  wire16: the replicas are
// bf16 buffers (2 bytes per element) and the output is a separate fp32 buffer.
// scratch: where the per-chunk partial sums and the slice sums of the statistics go (nullptr: the context's own
// reduction scratch), scratch_bytes: its size.
int ddp::partial_average_impl(ddp_ctx *ctx, const char *who, bool wire16, int slot, const void *flat_local, const void *const *peers,
                              int N, int local_rank, float *flat_out, double *layer_stats, void *stream, double *scratch,
                              int64_t scratch_bytes) {
    int rc;
    const SlotTables *s = slot_of(ctx, slot, who, &rc);
    if (!s) return rc;
    double *partials = ctx->d_partials, *slice_sums = ctx->d_slice_sums;
    if (scratch) {
        const int64_t need = (s->n_mean + (int64_t)s->layers.size() * kStatSlices) * 2 * (int64_t)sizeof(double);
        if (layer_stats && need > scratch_bytes)
            return fail(ctx, DDP_ESHAPE, std::string(who) + ": slot " + std::to_string(slot) + " needs " + std::to_string(need) +
                                             " bytes of reduction scratch (" + std::to_string(s->n_mean) + " chunks), the fixed scratch holds " +
                                             std::to_string(scratch_bytes) + "; use ddp_partial_average or a larger mean_chunk");
        partials = scratch;
        slice_sums = scratch + 2 * s->n_mean;
    }
    if ((rc = check_device(ctx, who)) != DDP_OK) return rc;
    if (N < 1 || N > DDP_MAX_REPLICAS) return fail(ctx, DDP_EINVAL, std::string(who) + ": N must be in [1, " + std::to_string((int)DDP_MAX_REPLICAS) + "]");
    if (local_rank < 0 || local_rank >= N) return fail(ctx, DDP_EINVAL, std::string(who) + ": local_rank out of range");
    if (N > 1 && !peers) return fail(ctx, DDP_EINVAL, std::string(who) + ": peers is NULL");
    if (s->numel == 0) return DDP_OK;
    if ((rc = check_flat(ctx, flat_local, who, "flat_local")) != DDP_OK) return rc;
    if ((rc = check_flat(ctx, flat_out, who, "flat_out")) != DDP_OK) return rc;
    if (layer_stats && !aligned(layer_stats, 8)) return fail(ctx, DDP_EALIGN, std::string(who) + ": layer_stats must be 8-byte aligned");
    const uintptr_t out_bytes = (uintptr_t)s->numel * 4, in_bytes = (uintptr_t)s->numel * (wire16 ? 2 : 4);
    auto overlaps_out = [&](const void *in) {
        uintptr_t x = (uintptr_t)in, y = (uintptr_t)flat_out;
        return x < y + out_bytes && y < x + in_bytes;
    };
    // fp32: exactly in place is fine (each element is read before it is written by the same thread)
    if (!(flat_out == flat_local && !wire16) && overlaps_out(flat_local))
        return fail(ctx, DDP_EINVAL, std::string(who) + (wire16 ? ": flat_out overlaps flat_local" : ": flat_out partially overlaps flat_local"));
    MeanLaunch a{};
    int p = 0;
    for (int k = 0; k < N; ++k) {
        if (k == local_rank) {
            a.x[k] = flat_local;
            continue;
        }
        const void *q = peers[p++];
        if ((rc = check_flat(ctx, q, who, "a peer buffer")) != DDP_OK) return rc;
        if (overlaps_out(q)) return fail(ctx, DDP_EINVAL, std::string(who) + ": a peer buffer overlaps flat_out");
        a.x[k] = q;
    }
    a.wire16 = wire16;
    a.n_replicas = N;
    a.inv_n = 1.0f / (float)N;
    a.out = flat_out;
    a.chunks = s->d_mean;
    a.n_chunks = s->n_mean;
    a.partials = layer_stats ? partials : nullptr;
    a.slice_sums = slice_sums;
    a.layer_ranges = s->d_layer_ranges;
    a.n_layers = (int)s->layers.size();
    a.max_partials_per_layer = s->max_mean_partials;
    a.stats = layer_stats;
    a.nontemporal = ctx->nontemporal;
    // bf16 replicas put half the bytes per workgroup in flight: half the pad, twice the workgroups per CU
    a.lds_pad = wire16 ? ctx->mean_lds / 2 : ctx->mean_lds;
    rc = launch_mean(a, stream);
    return after_launch(ctx, who, rc);
}

extern "C" int ddp_partial_average(ddp_ctx *ctx, int slot, const float *flat_local, const float *const *peers, int N,
                                   int local_rank, float *flat_out, double *layer_stats, void *stream) {
    return guarded(ctx, [&]() -> int {
        return partial_average_impl(ctx, "ddp_partial_average", false, slot, flat_local, reinterpret_cast<const void *const *>(peers), N,
                                    local_rank, flat_out, layer_stats, stream, nullptr, 0);
    });
}

extern "C" int ddp_pack_wire16(ddp_ctx *ctx, int slot, uint16_t *flat_local16, void *stream) {
    return guarded(ctx, [&]() -> int {
        int rc;
        const SlotTables *s = slot_of(ctx, slot, "ddp_pack_wire16", &rc);
        if (!s) return rc;
        if ((rc = check_device(ctx, "ddp_pack_wire16")) != DDP_OK) return rc;
        if (s->numel == 0) return DDP_OK;
        if ((rc = check_flat(ctx, flat_local16, "ddp_pack_wire16", "flat_local16")) != DDP_OK) return rc;
        rc = launch_pack16(ctx->d_tensors, s->d_copy, s->n_copy, flat_local16, ctx->nontemporal, ctx->copy_lds, stream);
        return after_launch(ctx, "ddp_pack_wire16", rc);
    });
}

extern "C" int ddp_partial_average_wire16(ddp_ctx *ctx, int slot, const uint16_t *flat_local16, const uint16_t *const *peers16, int N,
                                          int local_rank, float *flat_out, double *layer_stats, void *stream) {
    return guarded(ctx, [&]() -> int {
        return partial_average_impl(ctx, "ddp_partial_average_wire16", true, slot, flat_local16,
                                    reinterpret_cast<const void *const *>(peers16), N, local_rank, flat_out, layer_stats, stream, nullptr, 0);
    });
}

static int make_scalars(ddp_ctx *ctx, const char *who, const ddp_opt *opt, UpdateScalars &s) {
    if (!opt) return fail(ctx, DDP_EINVAL, std::string(who) + ": opt is NULL");
    if (opt->kind == DDP_OPT_SGDM) {
        s.lr = opt->lr;
        s.mu = opt->momentum;
        return DDP_OK;
    }
    if (opt->kind != DDP_OPT_ADAMW) return fail(ctx, DDP_EINVAL, std::string(who) + ": unknown optimizer kind");
    if (!ctx->has_state1) return fail(ctx, DDP_ESTATE, std::string(who) + ": AdamW needs state1_ptr for every tensor");
    if (opt->step < 1) return fail(ctx, DDP_EINVAL, std::string(who) + ": step is 1-based");
    if (!(opt->beta1 >= 0.0f && opt->beta1 < 1.0f && opt->beta2 >= 0.0f && opt->beta2 < 1.0f))
        return fail(ctx, DDP_EINVAL, std::string(who) + ": betas must be in [0, 1)");
    // bias corrections in fp64, handed to the kernel as fp32 factors
    const double bc1 = 1.0 - std::pow((double)opt->beta1, (double)opt->step);
    const double bc2 = 1.0 - std::pow((double)opt->beta2, (double)opt->step);
    const float inv_bc1 = (float)(1.0 / bc1);
    s.beta1 = opt->beta1;
    s.beta2 = opt->beta2;
    s.omb1 = 1.0f - opt->beta1;
    s.omb2 = 1.0f - opt->beta2;
    s.decay = 1.0f - opt->lr * opt->weight_decay;
    s.step_size = opt->lr * inv_bc1;
    s.rsqrt_bc2 = (float)(1.0 / std::sqrt(bc2));
    s.eps = opt->eps;
    return DDP_OK;
}

// Chunk range [c0, c1) of the update table that covers layers [first, first + count); needs the table in
// registration order.
static int layer_chunk_range(ddp_ctx *ctx, const char *who, int first, int count, int64_t *c0, int64_t *c1) {
    if (first < 0 || count < 0 || first > ctx->L || count > ctx->L - first)
        return fail(ctx, DDP_EINVAL, std::string(who) + ": layer range outside [0, " + std::to_string(ctx->L) + ")");
    if (ctx->dispatch_ways != 1 && !(first == 0 && count == ctx->L))
        return fail(ctx, DDP_ESTATE, std::string(who) + ": a layer range needs the update table in registration order (option dispatch_ways = 1)");
    *c0 = ctx->tensor_chunk_base[(size_t)ctx->layer_first_tensor[(size_t)first]];
    *c1 = ctx->tensor_chunk_base[(size_t)ctx->layer_first_tensor[(size_t)(first + count)]];
    return DDP_OK;
}

// The streams of layers [first, first + count) as one dense range, if the model is registered that way, the option
// allows it and the range starts on a vector boundary.
static bool dense_range(const ddp_ctx *ctx, int first, int count, DenseLaunch &d) {
    if (!ctx->dense || !ctx->dense_path) return false;
    const int64_t e0 = ctx->tensor_elem_off[(size_t)ctx->layer_first_tensor[(size_t)first]];
    const int64_t e1 = ctx->tensor_elem_off[(size_t)ctx->layer_first_tensor[(size_t)(first + count)]];
    if (e0 % 4 != 0) return false;
    const TensorDesc &t0 = ctx->tensors[0];
    d.p = t0.sync + e0;
    d.s0 = t0.state0 + e0;
    d.s1 = ctx->has_state1 ? t0.state1 + e0 : nullptr;
    d.g = (const char *)t0.grad + (uintptr_t)e0 * (ctx->grad_dtype == DDP_F32 ? 4 : 2);
    d.mdl = ctx->param_dtype == DDP_BF16 ? t0.model + e0 : nullptr;
    d.n = e1 - e0;
    d.chunk = (int)ctx->update_chunk;
    return true;
}

static int local_update_impl(ddp_ctx *ctx, const char *who, bool whole, int first, int count, const ddp_opt *opt, void *stream) {
    if (!ctx) return fail(nullptr, DDP_EINVAL, std::string(who) + ": ctx is NULL");
    if (!ctx->registered) return fail(ctx, DDP_ESTATE, std::string(who) + ": no model registered");
    UpdateScalars s{};
    int rc = make_scalars(ctx, who, opt, s);
    if (rc != DDP_OK) return rc;
    if ((rc = check_device(ctx, who)) != DDP_OK) return rc;
    int64_t c0 = 0, c1 = ctx->n_update;
    if (!whole && (rc = layer_chunk_range(ctx, who, first, count, &c0, &c1)) != DDP_OK) return rc;
    if (c1 == c0) return DDP_OK;
    DenseLaunch d{};
    if (dense_range(ctx, whole ? 0 : first, whole ? ctx->L : count, d)) {
        rc = launch_update_dense(opt->kind, ctx->grad_dtype, ctx->param_dtype == DDP_BF16, d, s, ctx->nontemporal, ctx->update_lds, stream);
        return after_launch(ctx, who, rc);
    }
    rc = launch_update(opt->kind, ctx->grad_dtype, ctx->param_dtype == DDP_BF16, ctx->d_tensors, ctx->d_update + c0, c1 - c0, s,
                       ctx->nontemporal, ctx->update_lds, stream);
    return after_launch(ctx, who, rc);
}

extern "C" int ddp_local_update(ddp_ctx *ctx, const ddp_opt *opt, void *stream) {
    return guarded(ctx, [&]() -> int {
        return local_update_impl(ctx, "ddp_local_update", true, 0, 0, opt, stream);
    });
}

extern "C" int ddp_local_update_layers(ddp_ctx *ctx, int layer_first, int layer_count, const ddp_opt *opt, void *stream) {
    return guarded(ctx, [&]() -> int {
        return local_update_impl(ctx, "ddp_local_update_layers", false, layer_first, layer_count, opt, stream);
    });
}

// The fused step over layers [first, first + count) of a model registered as dense arenas: one table-free launch per
// scheduled layer and one per run of unscheduled layers.  *done = false (nothing launched) when the model, the
// options, the replica count or an alignment rule the table-free kernels out; the caller then takes the table.
static int fused_dense(ddp_ctx *ctx, const char *who, const SlotTables *st, const void *const *x, bool wire16, bool update_first, int first,
                       int count, int N, int local_rank, double *layer_stats, const ddp_opt *opt, const UpdateScalars &s, void *stream,
                       bool *done) {
    *done = false;
    if (!ctx->dense || !ctx->dense_path || !ctx->nontemporal || !fused_dense_supports(N)) return DDP_OK;
    const std::vector<int32_t> &pos = st->layer_pos;  // layer -> position in the slot, -1 if not scheduled
    auto elem0 = [&](int l) { return ctx->tensor_elem_off[(size_t)ctx->layer_first_tensor[(size_t)l]]; };
    // every launch must start on a vector boundary in the model and, for a scheduled layer, in the flat buffer
    int64_t launches = 0;
    for (int l = first; l < first + count; ++l) {
        const bool sched = pos[(size_t)l] >= 0, run_start = l == first || sched || pos[(size_t)l - 1] >= 0;
        if (run_start && elem0(l) % 4 != 0) return DDP_OK;
        if (sched && ((elem0(l + 1) - elem0(l)) % 4 != 0 || st->layer_begin[(size_t)pos[(size_t)l]] % 4 != 0)) return DDP_OK;
        launches += run_start;
    }
    // one launch per scheduled layer only pays when the launches are long: small layers stay with the single
    // table-driven launch
    if (launches > 1 && (elem0(first + count) - elem0(first)) / launches < (int64_t)1 << 18) return DDP_OK;
    *done = true;
    const bool stats = layer_stats != nullptr;
    int rc = 0;
    for (int l = first; l < first + count && rc == 0;) {
        DenseLaunch d{};
        if (pos[(size_t)l] < 0) {
            int m = l + 1;
            while (m < first + count && pos[(size_t)m] < 0) ++m;
            dense_range(ctx, l, m - l, d);
            rc = launch_update_dense(opt->kind, ctx->grad_dtype, ctx->param_dtype == DDP_BF16, d, s, true, ctx->update_lds, stream);
            l = m;
            continue;
        }
        const int i = pos[(size_t)l];
        FusedDenseLaunch f{};
        dense_range(ctx, l, 1, f.d);
        for (int k = 0; k < N; ++k) f.x[k] = x[k];
        f.wire16 = wire16;
        f.update_first = update_first;
        f.n_replicas = N;
        f.local_rank = local_rank;
        f.inv_n = 1.0f / (float)N;
        f.kind = opt->kind;
        f.grad_dtype = ctx->grad_dtype;
        f.with_model = ctx->param_dtype == DDP_BF16;
        f.fo0 = st->layer_begin[(size_t)i];
        f.s = s;
        f.partials = stats ? ctx->d_partials : nullptr;
        f.pbase = st->dense_ranges[2 * (size_t)i];
        f.lds_pad = ctx->update_lds;
        rc = launch_fused_dense(f, stream);
        ++l;
    }
    // statistics of the slot's layers inside the range: one reduction per run of consecutive slot positions
    const int nl = (int)st->layers.size();
    for (int i = 0; stats && rc == 0 && i < nl;) {
        auto inside = [&](int j) { return st->layers[(size_t)j] >= first && st->layers[(size_t)j] < first + count; };
        if (!inside(i)) {
            ++i;
            continue;
        }
        int j = i + 1;
        while (j < nl && inside(j)) ++j;
        rc = launch_stats(ctx->d_partials, ctx->d_slice_sums + (int64_t)i * 2 * kStatSlices, st->d_dense_ranges + 2 * i, j - i, N,
                          layer_stats + 2 * i, st->max_dense_partials, stream);
        i = j;
    }
    return after_launch(ctx, who, rc);
}

// whole: every layer (any dispatch order).  Otherwise layers [first, first + count) only: their chunks of the update
// table, and the statistics of those of the slot's layers that fall in the range.
static int fused_impl(ddp_ctx *ctx, const char *who, bool wire16, bool update_first, int slot, bool whole, int first, int count,
                      const void *const *peers, int N, int local_rank, double *layer_stats, const ddp_opt *opt, void *stream) {
    int rc;
    const SlotTables *st = slot_of(ctx, slot, who, &rc);
    if (!st) return rc;
    UpdateScalars s{};
    if ((rc = make_scalars(ctx, who, opt, s)) != DDP_OK) return rc;
    if ((rc = check_device(ctx, who)) != DDP_OK) return rc;
    if (N < 1 || N > DDP_MAX_REPLICAS) return fail(ctx, DDP_EINVAL, std::string(who) + ": N must be in [1, " + std::to_string((int)DDP_MAX_REPLICAS) + "]");
    if (local_rank < 0 || local_rank >= N) return fail(ctx, DDP_EINVAL, std::string(who) + ": local_rank out of range");
    if (N > 1 && !peers) return fail(ctx, DDP_EINVAL, std::string(who) + ": peers is NULL");
    if (layer_stats && !aligned(layer_stats, 8)) return fail(ctx, DDP_EALIGN, std::string(who) + ": layer_stats must be 8-byte aligned");
    int64_t c0 = 0, c1 = ctx->n_update;
    if (!whole && (rc = layer_chunk_range(ctx, who, first, count, &c0, &c1)) != DDP_OK) return rc;
    FusedLaunch f{};
    int p = 0;
    for (int k = 0; k < N; ++k) {
        if (k == local_rank) continue;
        const void *q = peers[p++];
        if (st->numel > 0 && (rc = check_flat(ctx, q, who, "a peer buffer")) != DDP_OK) return rc;
        f.x[k] = q;
    }
    if (c1 == c0) return DDP_OK;
    {
        bool done = false;
        rc = fused_dense(ctx, who, st, f.x, wire16, update_first, whole ? 0 : first, whole ? ctx->L : count, N, local_rank, layer_stats,
                         opt, s, stream, &done);
        if (done) return rc;
    }
    f.wire16 = wire16;
    f.update_first = update_first;
    f.n_replicas = N;
    f.local_rank = local_rank;
    f.inv_n = 1.0f / (float)N;
    f.kind = opt->kind;
    f.grad_dtype = ctx->grad_dtype;
    f.with_model = ctx->param_dtype == DDP_BF16;
    f.tensors = ctx->d_tensors;
    f.chunks = ctx->d_update + c0;
    f.n_chunks = c1 - c0;
    f.tensor_flat_off = st->d_tensor_flat_off;
    f.tensor_chunk_base = ctx->d_tensor_chunk_base;
    f.chunk_elems = (int)ctx->update_chunk;
    f.s = s;
    f.lds_pad = ctx->update_lds;
    const int nl = (int)st->layers.size();
    if (!layer_stats || nl == 0) return after_launch(ctx, who, launch_fused(f, stream));
    f.partials = ctx->d_partials;
    f.max_partials_per_layer = st->max_fused_partials;
    if (whole) {
        f.slice_sums = ctx->d_slice_sums;
        f.layer_ranges = st->d_fused_ranges;
        f.n_layers = nl;
        f.stats = layer_stats;
        return after_launch(ctx, who, launch_fused(f, stream));
    }
    // Statistics of the slot's layers inside the range: one reduction per run of consecutive slot positions (a
    // schedule in backward order gives a single run).  The first launch also carries the kernel itself.
    bool launched = false;
    for (int i = 0; i < nl;) {
        if (st->layers[(size_t)i] < first || st->layers[(size_t)i] >= first + count) {
            ++i;
            continue;
        }
        int j = i + 1;
        while (j < nl && st->layers[(size_t)j] >= first && st->layers[(size_t)j] < first + count) ++j;
        f.slice_sums = ctx->d_slice_sums + (int64_t)i * 2 * kStatSlices;
        f.layer_ranges = st->d_fused_ranges + 2 * i;
        f.n_layers = j - i;
        f.stats = layer_stats + 2 * i;
        if (!launched) {
            rc = launch_fused(f, stream);
            launched = true;
        } else {
            rc = launch_stats(f.partials, f.slice_sums, f.layer_ranges, f.n_layers, N, f.stats, f.max_partials_per_layer, stream);
        }
        if (rc != 0) return after_launch(ctx, who, rc);
        i = j;
    }
    if (!launched) {  // no scheduled layer in the range: plain update of these layers, no partials written
        f.partials = nullptr;
        rc = launch_fused(f, stream);
    }
    return after_launch(ctx, who, rc);
}

extern "C" int ddp_fused_sync_update(ddp_ctx *ctx, int slot, const float *const *peers, int N, int local_rank, double *layer_stats,
                                     const ddp_opt *opt, void *stream) {
    return guarded(ctx, [&]() -> int {
        return fused_impl(ctx, "ddp_fused_sync_update", false, false, slot, true, 0, 0, reinterpret_cast<const void *const *>(peers), N, local_rank,
                          layer_stats, opt, stream);
    });
}

extern "C" int ddp_fused_sync_update_wire16(ddp_ctx *ctx, int slot, const uint16_t *const *peers16, int N, int local_rank,
                                            double *layer_stats, const ddp_opt *opt, void *stream) {
    return guarded(ctx, [&]() -> int {
        return fused_impl(ctx, "ddp_fused_sync_update_wire16", true, false, slot, true, 0, 0, reinterpret_cast<const void *const *>(peers16), N,
                          local_rank, layer_stats, opt, stream);
    });
}

extern "C" int ddp_fused_sync_update_layers(ddp_ctx *ctx, int slot, int layer_first, int layer_count, const void *const *peers,
                                            int wire_dtype, int order, int N, int local_rank, double *layer_stats, const ddp_opt *opt,
                                            void *stream) {
    return guarded(ctx, [&]() -> int {
        if (wire_dtype != DDP_F32 && wire_dtype != DDP_BF16) return fail(ctx, DDP_EINVAL, "ddp_fused_sync_update_layers: bad wire_dtype");
        if (order != DDP_SYNC_THEN_UPDATE && order != DDP_UPDATE_THEN_SYNC) return fail(ctx, DDP_EINVAL, "ddp_fused_sync_update_layers: bad order");
        return fused_impl(ctx, "ddp_fused_sync_update_layers", wire_dtype == DDP_BF16, order == DDP_UPDATE_THEN_SYNC, slot, false, layer_first,
                          layer_count, peers, N, local_rank, layer_stats, opt, stream);
    });
}
