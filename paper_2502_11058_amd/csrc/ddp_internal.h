// Internal declarations shared by the host side of the library (context, tables) and its kernels.
#ifndef DDP_INTERNAL_H
#define DDP_INTERNAL_H

#include <cstdint>
#include <string>
#include <vector>

#include "dreamddp.h"

namespace ddp {

// Record a failure message (on the context, or thread-local when ctx is NULL) and return the code.
int fail(const ddp_ctx *ctx, int code, const std::string &msg);

// The same from a catch block: if recording the message throws as well, the code alone is returned.
inline int fail_nothrow(const ddp_ctx *ctx, int code, const char *msg) noexcept {
    try {
        return fail(ctx, code, msg);
    } catch (...) {
        return code;
    }
}

// No C++ exception crosses the C boundary: the entry points build messages and small host vectors, so a failed host
// allocation (or anything else thrown) is turned into DDP_ENOMEM here.
template <class F>
int guarded(const ddp_ctx *ctx, F &&body) noexcept {
    try {
        return body();
    } catch (...) {
        return fail_nothrow(ctx, DDP_ENOMEM, "host allocation failed");
    }
}

// ---- device tables -------------------------------------------------------------------------------------------
// Everything a kernel needs to find its work is in small read-only tables in HBM, built once when the model
// is registered or the schedule installed.  One workgroup handles one "chunk": a run of elements that lies
// inside one tensor (copy, update) or one layer (mean), so ragged tensor and layer boundaries never fall
// inside a workgroup's vector loop, and per-layer reductions never mix layers.

struct TensorDesc {   // one registered tensor
    float *sync;      // fp32 params or master weights
    uint16_t *model;  // bf16 model copy or nullptr
    void *grad;       // fp32 or bf16
    float *state0;    // momentum / first moment
    float *state1;    // second moment or nullptr
    int64_t numel;
};

struct UpdateChunk {  // local_update: elements [begin, begin+count) of tensor `tensor`
    int64_t begin;
    int32_t tensor;
    int32_t count;
};

struct CopyChunk {  // pack / unpack: tensor elements [t_begin, +count) <-> flat elements [flat_begin, +count)
    int64_t t_begin;
    int64_t flat_begin;
    int32_t tensor;
    int32_t count;
};

struct MeanChunk {  // partial_average: flat elements [begin, +count), all inside one layer of the slot
    int64_t begin;
    int32_t count;
    int32_t partial;  // where this chunk's partial sums go: its index in flat order, whatever the dispatch order
};

struct SlotTables {
    // host copies (introspection, validation)
    std::vector<int32_t> layers;       // layer ids in flat order
    std::vector<int64_t> layer_begin;  // n_layers + 1 flat offsets
    std::vector<int32_t> tensors;      // tensor ids in flat order
    std::vector<int64_t> tensor_off;
    int64_t numel = 0;
    // device tables
    CopyChunk *d_copy = nullptr;
    int64_t n_copy = 0;
    MeanChunk *d_mean = nullptr;
    int64_t n_mean = 0;
    int32_t *d_layer_ranges = nullptr;     // per layer of the slot: [first, last) mean chunk
    int64_t *d_tensor_flat_off = nullptr;  // per registered tensor: first flat index in this slot, -1 if unscheduled
    int32_t *d_fused_ranges = nullptr;     // per layer of the slot: [first, last) update chunk (registration order)
    // dense arenas: per layer of the slot [first, last) index of its workgroups' partials (layers numbered in
    // registration order, ceil(layer elements / update_chunk) workgroups each)
    std::vector<int32_t> dense_ranges;
    int64_t max_mean_partials = 0, max_fused_partials = 0, max_dense_partials = 0;  // largest per-layer count of each range table
    std::vector<int32_t> layer_pos;  // [L] layer -> position in this slot, -1 if not scheduled
    int32_t *d_dense_ranges = nullptr;
};

// ---- launchers (ddp_kernels.hip) -------------------------------------------------------------------------------
struct MeanLaunch {
    const void *x[DDP_MAX_REPLICAS];  // replicas in rank order (fp32, or bf16 when wire16)
    bool wire16;
    int n_replicas;
    float inv_n;
    float *out;
    const MeanChunk *chunks;
    int64_t n_chunks;
    double *partials;  // [n_chunks][2] or nullptr when no statistics are wanted
    double *slice_sums;  // [n_layers][64][2] scratch of the two-stage reduction
    const int32_t *layer_ranges;  // per layer [first, last) partial index
    int n_layers;
    int64_t max_partials_per_layer;
    double *stats;  // [n_layers][2]
    bool nontemporal;
    int lds_pad;
};

struct UpdateScalars {
    float lr, mu;                                                // SGD-m
    float beta1, beta2, omb1, omb2, decay, step_size, rsqrt_bc2, eps;  // AdamW
};

int launch_copy(bool unpack, const TensorDesc *tensors, const CopyChunk *chunks, int64_t n_chunks, float *flat,
                bool with_model, bool nontemporal, int lds_pad, void *stream);
int launch_mean(const MeanLaunch &a, void *stream);
// Per-layer statistics from per-chunk partials: layer l of n_layers adds partials [ranges[2l], ranges[2l+1]) in a fixed
// order through kStatSlices slice sums (slice_sums: [n_layers][kStatSlices][2]) into stats[2l], stats[2l+1].
// With at most kStatSingleMax partials in any of the layers (max_partials_per_layer, an upper bound is enough) one launch
// does it all; beyond that the two stages.
constexpr int kStatSlices = 64;
constexpr int64_t kStatSingleMax = 4096;
int launch_stats(const double *partials, double *slice_sums, const int32_t *ranges, int n_layers, int n_replicas, double *stats,
                 int64_t max_partials_per_layer, void *stream);
int launch_pack16(const TensorDesc *tensors, const CopyChunk *chunks, int64_t n_chunks, uint16_t *flat16, bool nontemporal, int lds_pad,
                  void *stream);
struct FusedLaunch {
    const void *x[DDP_MAX_REPLICAS];  // peers in rank order (entry local_rank unused); fp32, or bf16 when wire16
    bool wire16;
    bool update_first;  // Eq. (5) as printed: the local value takes the optimizer step before it is averaged
    int n_replicas, local_rank;
    float inv_n;
    int kind, grad_dtype;
    bool with_model;
    const TensorDesc *tensors;
    const UpdateChunk *chunks;
    int64_t n_chunks;
    const int64_t *tensor_flat_off;
    const int32_t *tensor_chunk_base;
    int chunk_elems;
    UpdateScalars s;
    double *partials;  // nullptr: no statistics
    double *slice_sums;
    const int32_t *layer_ranges;
    int n_layers;
    int64_t max_partials_per_layer;
    double *stats;
    int lds_pad;
};
int launch_fused(const FusedLaunch &f, void *stream);
// The update over tensors that lie back to back in every stream: the range's first element in each stream (aligned
// for 128-bit access, bf16 streams for 64-bit), its length and the elements per workgroup.
struct DenseLaunch {
    const void *g;
    float *p, *s0, *s1;
    uint16_t *mdl;
    int64_t n;
    int chunk;
};
int launch_update_dense(int kind, int grad_dtype, bool with_model, const DenseLaunch &d, const UpdateScalars &s, bool nontemporal,
                        int lds_pad, void *stream);
// One scheduled layer of a dense model through the fused kernel: local streams d (d.n a multiple of 4), peers' flat
// buffers x, the layer's first flat index fo0 (a multiple of 4); workgroup b's partial pair goes to partials[2 * (pbase + b)]
// (nullptr: no statistics).  Replica counts fused_dense_supports() accepts only.
struct FusedDenseLaunch {
    DenseLaunch d;
    const void *x[DDP_MAX_REPLICAS];
    bool wire16, update_first;
    int n_replicas, local_rank;
    float inv_n;
    int kind, grad_dtype;
    bool with_model;
    int64_t fo0;
    UpdateScalars s;
    double *partials;
    int64_t pbase;
    int lds_pad;
};
bool fused_dense_supports(int n_replicas);
int launch_fused_dense(const FusedDenseLaunch &f, void *stream);
int launch_update(int kind, int grad_dtype, bool with_model, const TensorDesc *tensors, const UpdateChunk *chunks,
                  int64_t n_chunks, const UpdateScalars &s, bool nontemporal, int lds_pad, void *stream);

// Shared body of the averaging entry points (ddp_context.hip).  scratch == nullptr: the context's reduction scratch.
int partial_average_impl(ddp_ctx *ctx, const char *who, bool wire16, int slot, const void *flat_local, const void *const *peers, int N,
                         int local_rank, float *flat_out, double *layer_stats, void *stream, double *scratch, int64_t scratch_bytes);

// The fixed reduction scratch of ddp_partial_average_static on the current device (ddp_noalloc.hip): resolves the
// device address of the library's static array once per device.  Call with `device` current.
int static_scratch_for(const ddp_ctx *ctx, int device, double **ptr);

}  // namespace ddp

struct ddp_ctx {
    int device = 0;
    mutable std::string err;
    // options
    int64_t update_chunk = 2048, mean_chunk = 2048, copy_chunk = 2048;
    bool nontemporal = true;
    int dispatch_ways = 1;
    int lds_per_cu = 163840, lds_per_wg_max = 65536;  // what the device reports (ddp_create); gfx950 values until then
    int update_lds = 64512, mean_lds = 64512, copy_lds = 26112;  // dynamic-LDS pad per workgroup: caps residency per CU (2 / 2 / 6)
    // model
    bool registered = false;
    int L = 0, T = 0;
    int param_dtype = DDP_F32, grad_dtype = DDP_F32;
    bool has_state1 = false;
    std::vector<int32_t> layer_of;
    std::vector<int64_t> numel;
    std::vector<ddp::TensorDesc> tensors;
    std::vector<int32_t> layer_first_tensor;  // L + 1
    std::vector<int64_t> tensor_elem_off;     // T + 1: elements before each tensor, registration order
    bool dense = false;      // tensors lie back to back in every stream and the streams' starts are vector-aligned
    bool dense_path = true;  // option: use the table-free kernels where `dense` allows it
    ddp::TensorDesc *d_tensors = nullptr;
    ddp::UpdateChunk *d_update = nullptr;
    int64_t n_update = 0;
    std::vector<int32_t> tensor_chunk_base;  // T + 1: first update chunk of each tensor, registration order
    int32_t *d_tensor_chunk_base = nullptr;
    // schedule
    int H = 0;
    std::vector<ddp::SlotTables> slots;
    double *d_partials = nullptr;  // reduction scratch for per-layer statistics: one partial pair per chunk ...
    double *d_slice_sums = nullptr;  // ... followed by 64 slice sums per layer (same allocation)
    int64_t partials_cap = 0;
    double *static_scratch = nullptr;  // this device's copy of the library's fixed scratch array (ddp_partial_average_static)
    std::string static_scratch_err;    // why it could not be resolved, if it could not
};

#endif
