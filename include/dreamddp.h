/*
 * dreamddp.h - C ABI of the MI355X (gfx950) library for one worker's per-iteration step of local SGD with
 * partial synchronisation (PLSGD, Algorithm 1 and Definition 1 / Eq. (5) of the DreamDDP paper) and for the
 * layer-to-iteration scheduling problem of its Sec. 3.3 (Eq. (8), Algorithm 2).
 *
 * One iteration r (0-based) of one worker, with slot = r mod H:
 *
 *     ddp_pack(slot)             gather the slot's layers (the fp32 copy that is synchronised) into a flat buffer
 *     [network: the N-1 peers' flat buffers of the same layers arrive; here they are staged device buffers]
 *     ddp_partial_average(slot)  mean over the N replicas in rank order; per-layer divergence and norm
 *     ddp_unpack(slot)           scatter the mean back into the model (and refresh the bf16 model copy)
 *     ddp_local_update()         fused SGD-momentum or AdamW step on every layer
 *
 * Conventions
 *   - Every function returns a ddp_status (0 = success).  Nothing throws, aborts or prints.  After a failure
 *     ddp_last_error() gives a message.  Arguments are validated on the host before any kernel is launched.
 *   - "device pointer" = address in the HBM of the context's GPU; "host pointer" = ordinary memory.
 *     All device memory passed in is owned by the caller and must stay valid while the context uses it.
 *   - The four per-iteration calls only enqueue kernels on the caller's stream (a hipStream_t passed as
 *     void*, NULL = the default stream).  They never allocate, free, copy to the host or synchronise.
 *   - A context holds nothing of the training state: only tables derived from the registration and the schedule, and a
 *     reduction scratch that every call writes before it reads.  Parameters, optimizer state, model copy and the step
 *     counter (ddp_opt.step) are the caller's: a checkpoint is those tensors plus the iteration number, and a new
 *     context registered over the restored tensors continues with the bits of the uninterrupted run.
 *   - A context is not thread-safe; calls that share a context or device buffers must be ordered by the caller
 *     (stream order is enough): the statistics go through one reduction scratch per context.  The only calls that
 *     may be in flight together on one context are the layer-range calls, for disjoint ranges.
 *   - ddp_fused_sync_update does average, unpack and update of the list above in one pass over the model (no local
 *     flat buffer);
 *     the *_wire16 entry points exchange bf16 instead of fp32; the *_layers entry points act on a range of layers.
 *   - Layers are numbered 0..L-1 from the input side (the paper's layer 1) to the output side (layer L);
 *     the backward pass visits L-1, L-2, ..., 0.  Times are integer nanoseconds.
 */
#ifndef DREAMDDP_H
#define DREAMDDP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ddp_ctx ddp_ctx; /* opaque: owns only derived device tables and a small reduction scratch */

typedef enum {
    DDP_OK = 0,
    DDP_EINVAL = 1, /* bad argument value (NULL, out of range, duplicate layer, ...) */
    DDP_ESHAPE = 2, /* sizes do not match what was registered */
    DDP_EALIGN = 3, /* pointer alignment requirement violated */
    DDP_ENOMEM = 4, /* allocation of the context's tables failed */
    DDP_EHIP = 5,   /* a HIP runtime call failed (message holds hipGetErrorString) */
    DDP_ESCHED = 6, /* schedule missing or inconsistent with the registered model */
    DDP_ESTATE = 7  /* call made in the wrong order (e.g. pack before register) */
} ddp_status;

enum { DDP_F32 = 0, DDP_BF16 = 1 };
enum { DDP_OPT_SGDM = 0, DDP_OPT_ADAMW = 1 };
enum { DDP_MAX_REPLICAS = 64 };

/* Schedule policies.
 *   ENP          Example 1 (equal-number partition): consecutive groups of floor/ceil(L/H) layers in BP order,
 *                the remainder going to the earliest sets.
 *   ROUND_ROBIN  slot = layer mod H (non-contiguous sets; Definition 1 only needs disjoint subsets).
 *   FULL         every layer in the last slot: local SGD with full synchronisation, Eq. (2).
 *   EVERY        every layer in every slot: per-iteration model averaging.
 *   OPT          exact minimiser of Eq. (8) over all cuts of the BP-ordered layer sequence into H consecutive,
 *                possibly empty sets; ties -> lexicographically largest (|L_1|, |L_2|, ...).
 *   ALG2         Algorithm 2: depth-first search pruned by Properties 1-3, argmin over its solution set
 *                (first minimum in visiting order, assign-branch visited first).  The solution set can grow
 *                exponentially with min(L, H) (Sec. 3.3): the search gives up after 5e7 placement steps (well under
 *                a second) with DDP_ESCHED; OPT solves the same objective exactly in O(L^2 H). */
enum {
    DDP_SCHED_ENP = 0,
    DDP_SCHED_ROUND_ROBIN = 1,
    DDP_SCHED_FULL = 2,
    DDP_SCHED_EVERY = 3,
    DDP_SCHED_OPT = 4,
    DDP_SCHED_ALG2 = 5
};

/* Sec. 3.3, Eq. (8)-(11), Algorithm 2.  CPU only: needs no context and no GPU.
 *   t_fp_ns, t_bp_ns, t_comm_ns  host, [L], per-layer forward / backward / communication time, >= 0.
 *                                t_fp_ns may be NULL (it is a constant of the objective); t_bp_ns and t_comm_ns
 *                                may be NULL for ENP, ROUND_ROBIN, FULL, EVERY.
 *   out_slot        host, [L]: slot of each layer (EVERY: all zero, meaningless).
 *   out_set_ptr     host, [H+1], out_set_layers host, [L] ([L*H] for EVERY): CSR; the layers of slot s are
 *                   out_set_layers[out_set_ptr[s] .. out_set_ptr[s+1]) in BP order (descending layer id).
 *   out_cost_ns     host, nullable: Eq. (8) of the result (only for contiguous policies ENP, FULL, OPT, ALG2;
 *                   -1 otherwise).
 * Errors: DDP_EINVAL for L < 1, H < 1, unknown policy, NULL outputs, negative times, or time sums that
 * would overflow int64; DDP_ESCHED when ALG2's search exceeds its step budget. */
int ddp_schedule(int policy, int L, int H, const int64_t *t_fp_ns, const int64_t *t_bp_ns, const int64_t *t_comm_ns,
                 int32_t *out_slot, int32_t *out_set_ptr, int32_t *out_set_layers, int64_t *out_cost_ns);

/* Eq. (8) of a given schedule (CSR as above).  Every set must be a run of consecutive layers in BP order and
 * the sets must follow each other in BP order (a cut of L-1..0), else DDP_ESCHED.  Host pointers. */
int ddp_schedule_cost(int L, int H, const int64_t *t_bp_ns, const int64_t *t_comm_ns, const int32_t *set_ptr,
                      const int32_t *set_layers, int64_t *out_cost_ns);

/* Size of Algorithm 2's solution set Omega for the instance (Sec. 3.3, complexity analysis).  Host pointers.
 * DDP_ESCHED if the search exceeds its step budget (see DDP_SCHED_ALG2). */
int ddp_schedule_alg2_solutions(int L, int H, const int64_t *t_bp_ns, const int64_t *t_comm_ns, int64_t *out_count);

/* Sec. 3.4 "filling the bubble time", Eq. (12), Algorithm 2 lines 3-6.  Input: a schedule that is a cut of the
 * BP-ordered layers (as ddp_schedule writes for ENP, FULL, OPT, ALG2).  Every set additionally takes the longest
 * prefix L-1, L-2, ..., l of the BP order that is disjoint from it and keeps
 *     max(rem(h0), t_COMM(set) + t_COMM(prefix)) <= max(rem(h0), t_COMM(set)),
 * rem(h0) = backward time left after the set's first layer (for an empty set: after the top layer), t_COMM = plain
 * sums.  Layers of the prefix are then synchronised more than once per period.
 *   out_set_ptr [H+1], out_set_layers [capacity L*H]: CSR of the filled schedule, each set in BP order (the
 *   prefix first); out_extra [H], nullable: number of layers added per set.  Host pointers.
 * Errors: DDP_EINVAL (arguments, negative times), DDP_ESCHED (input is not a cut). */
int ddp_schedule_fill_bubbles(int L, int H, const int64_t *t_bp_ns, const int64_t *t_comm_ns, const int32_t *set_ptr,
                              const int32_t *set_layers, int32_t *out_set_ptr, int32_t *out_set_layers, int32_t *out_extra);

/* Eq. (7): wall-clock model of one synchronisation period with communication timestamps.  Within an iteration
 * the communication of a scheduled layer starts when that layer's backward is done and the previous
 * communication has ended (tau recursion); the iteration lasts forward + max(end of backward, end of the last
 * communication).  Sets may be any distinct layers listed in BP order (descending id), e.g. a filled schedule.
 *   t_fp_ns nullable (then 0).  out_iter_ns [H]: time of each iteration; out_exposed_ns [H], nullable:
 *   communication time not hidden by the backward pass; out_period_ns, nullable: sum over the H iterations
 *   (T_P-LSGD of Eq. (7) for R = H).  Host pointers.
 * Errors: DDP_EINVAL, DDP_ESCHED (set not in BP order, layer out of range). */
int ddp_schedule_time_model(int L, int H, const int64_t *t_fp_ns, const int64_t *t_bp_ns, const int64_t *t_comm_ns,
                            const int32_t *set_ptr, const int32_t *set_layers, int64_t *out_iter_ns, int64_t *out_exposed_ns,
                            int64_t *out_period_ns);

/* Context on GPU `device` (HIP ordinal).  The device must be the caller's current device in later calls. */
int ddp_create(ddp_ctx **out, int device);
int ddp_destroy(ddp_ctx *ctx);

/* Tuning knobs.  The first two groups shape the tables built by ddp_register_model / ddp_set_schedule and must be
 * set before them (DDP_ESTATE otherwise); the others take effect at the next launch.
 *   "update_chunk", "mean_chunk", "copy_chunk"  elements per workgroup (multiple of 1024, 1024..1048576;
 *                                               defaults 2048 / 2048 / 2048)
 *   "dispatch_ways"                             1..4096 (default 1): launch order of the workgroups; w > 1 cuts every
 *                                               chunk table into w contiguous segments and visits them round-robin
 *   "update_wg_per_cu", "mean_wg_per_cu",       0..32 (defaults 2 / 2 / 6; 0 = no cap): most workgroups of that kernel family resident per
 *   "copy_wg_per_cu"                            CU.  Few resident workgroups keep the window of DRAM rows in flight narrow, which
 *                                               measures faster than full occupancy for these streaming kernels.  Enforced by
 *                                               requesting (not using) dynamic LDS: LDS-per-CU / k bytes per workgroup, from the
 *                                               sizes the device reports, so the cap holds on parts with another LDS size; a
 *                                               kernel that needs LDS of its own gets the larger of the two.  The bf16-wire
 *                                               average runs at twice mean_wg_per_cu (half the bytes per workgroup in flight)
 *   "update_lds", "mean_lds", "copy_lds"        0..65536: the same cap given directly as bytes of LDS per workgroup (for sweeps)
 *   "nontemporal"                               0/1 (default 1): streaming cache hints on loads and stores
 *   "dense_path"                                0/1 (default 1): when the registered tensors lie back to back in every
 *                                               stream (one arena per stream, starts 16-byte aligned, bf16 streams
 *                                               8-byte), the update addresses its data from the block index alone
 *                                               instead of through the chunk table; 0 forces the table
 * Unknown names or bad values: DDP_EINVAL. */
int ddp_set_option(ddp_ctx *ctx, const char *name, int64_t value);

/* Describe the local replica (Algorithm 1 input w_0 and its optimizer state): T tensors, tensor t belongs
 * to layer layer_of[t] (host, [T], non-decreasing, covering 0..L-1) and has numel[t] > 0 elements (host, [T]).
 *   sync_ptr[t]    device fp32 [numel]: the copy that is averaged and updated (the parameters themselves, or
 *                  the fp32 master weights when param_dtype is DDP_BF16)
 *   model_ptr[t]   device bf16 [numel]: the model copy, rewritten by round-to-nearest-even whenever sync_ptr
 *                  changes; required iff param_dtype == DDP_BF16 (model_ptr itself may be NULL for DDP_F32)
 *   grad_ptr[t]    device [numel] of grad_dtype (DDP_F32 or DDP_BF16)
 *   state0_ptr[t]  device fp32 [numel]: momentum buffer (SGD-m) or first moment (AdamW)
 *   state1_ptr[t]  device fp32 [numel]: second moment; the array may be NULL if AdamW is never used
 * The pointer arrays are host arrays of device pointers.  Tensors need only the alignment of their element
 * type; tensors whose pointers are 16-byte aligned (8 for bf16) take the 128-bit path throughout.
 * Re-registering replaces the previous model and drops the schedule. */
int ddp_register_model(ddp_ctx *ctx, int L, int T, const int32_t *layer_of, const int64_t *numel, int param_dtype,
                       int grad_dtype, void *const *sync_ptr, void *const *model_ptr, void *const *grad_ptr,
                       void *const *state0_ptr, void *const *state1_ptr);

/* Install the iteration -> layer-set mapping (Definition 1; output Psi* of Algorithm 2) as CSR host arrays in
 * the layout ddp_schedule writes.  Builds the per-slot device offset tables: the flat buffer of a slot is the
 * dense concatenation of its layers in the order listed, each layer's tensors in registration order.
 * A layer may appear in several slots but only once per slot. */
int ddp_set_schedule(ddp_ctx *ctx, int H, const int32_t *set_ptr, const int32_t *set_layers);

/* Introspection for callers and parity checks (host outputs). */
int64_t ddp_slot_numel(const ddp_ctx *ctx, int slot);   /* elements in the slot's flat buffer; < 0 on error */
int ddp_slot_num_layers(const ddp_ctx *ctx, int slot);  /* < 0 on error */
int ddp_slot_num_tensors(const ddp_ctx *ctx, int slot); /* < 0 on error */
/* out_tensor_ids[j], out_off[j]: j-th tensor in flat order and its first element's flat index;
 * out_layer_ids[i], out_layer_begin[i] (+ out_layer_begin[n_layers] = total): layers in flat order.
 * Any output may be NULL. */
int ddp_slot_layout(const ddp_ctx *ctx, int slot, int32_t *out_tensor_ids, int64_t *out_off, int32_t *out_layer_ids,
                    int64_t *out_layer_begin);

/* Algorithm 1, the operand of the averaging: flat_local[off_t + i] = sync_t[i] for the slot's tensors.
 *   flat_local  device fp32, >= ddp_slot_numel(slot) elements, 16-byte aligned. */
int ddp_pack(ddp_ctx *ctx, int slot, float *flat_local, void *stream);

/* Eq. (5), second case: flat_out[i] = (x_0[i] + x_1[i] + ... + x_{N-1}[i]) * (1.0f / N), added left to right in
 * fp32 in global rank order, where x_{local_rank} = flat_local and the other x_k are peers[0..N-2] in rank
 * order.  Bit-reproducible: the same inputs give the same bits on every worker.
 *   peers        host array of N-1 device pointers (fp32, >= slot numel, 16-byte aligned); may be NULL if N == 1
 *   flat_out     device fp32, may be the same buffer as flat_local (no other overlap allowed)
 *   layer_stats  device double [2 * ddp_slot_num_layers(slot)], nullable.  For the i-th layer of the slot:
 *                [2i]   Gamma^l = (1/N) sum_k sum_j (flat_out[j] - x_k[j])^2   (model divergence, Sec. 3.4),
 *                [2i+1] sum_j flat_out[j]^2; differences in fp32, squares and sums in fp64, fixed order. */
int ddp_partial_average(ddp_ctx *ctx, int slot, const float *flat_local, const float *const *peers, int N,
                        int local_rank, float *flat_out, double *layer_stats, void *stream);

/* Algorithm 1, w_{r+1}^{k,l} = average: sync_t[i] = flat[off_t + i]; with a bf16 model copy also
 * model_t[i] = bf16_rne(flat[off_t + i]).  flat: device fp32, 16-byte aligned. */
int ddp_unpack(ddp_ctx *ctx, int slot, const float *flat, void *stream);

/* Eq. (5), first case (Algorithm 1 "update model") with the optimizers of the paper's experiments.
 * kind DDP_OPT_SGDM:  buf = momentum*buf + g;  p = p - lr*buf
 * kind DDP_OPT_ADAMW (decoupled weight decay, bias-corrected moments), exactly this sequence of fp32 operations:
 *     per call, on the host:  bc1 = 1 - beta1^step and bc2 = 1 - beta2^step in fp64;
 *                             step_size = lr * fp32(1/bc1)   (the reciprocal rounded to fp32, then one fp32 product)
 *                             rs2       = fp32(1/sqrt(bc2))  (computed in fp64, rounded to fp32 once)
 *                             decay     = 1 - lr*weight_decay,  omb1 = 1 - beta1,  omb2 = 1 - beta2   (fp32)
 *     per element:            m = beta1*m + omb1*g;   v = beta2*v + (omb2*g)*g;   p = p*decay;
 *                             p = p - step_size * ( m / (sqrt(v)*rs2 + eps) )
 *   i.e. the bias corrections enter as multiplications by rounded reciprocals, not as the divisions
 *   m/bc1 and sqrt(v)/sqrt(bc2) of the textbook form; the two forms agree to a few fp32 ulps per step, not bit for bit.
 *   sqrt and the division are the correctly rounded IEEE operations.
 * step is 1-based.  Every product and sum is a separate fp32 operation (no fused multiply-add); bf16 gradients are
 * widened exactly; the bf16 model copy, if registered, is rewritten from the new p by round-to-nearest-even.
 * Applies to every registered tensor. */
typedef struct {
    int32_t kind;
    float lr, momentum, beta1, beta2, eps, weight_decay;
    int64_t step;
} ddp_opt;
int ddp_local_update(ddp_ctx *ctx, const ddp_opt *opt, void *stream);

/* Both cases of Eq. (5) in one pass over the model (the "sync into update" fusion): for the tensors of the slot's
 * layers the average over the N replicas is formed from the local tensor and the peers' flat buffers (read at the
 * tensor's flat offset of this slot) and the optimizer step is applied to it; all other tensors get the optimizer
 * step only.  Parameters, optimizer state and model copy are bit-identical to ddp_pack -> ddp_partial_average ->
 * ddp_unpack -> ddp_local_update with the same arguments (the statistics agree to fp64 rounding: their partial sums are
 * grouped differently), but the local flat buffer is never written or read: HBM traffic is 4(N-1) bytes per scheduled element
 * plus the update's bytes per parameter.  peers, N, local_rank, layer_stats as in ddp_partial_average; opt as in
 * ddp_local_update.  No flat_local / flat_out: the result lives in the model tensors only. */
int ddp_fused_sync_update(ddp_ctx *ctx, int slot, const float *const *peers, int N, int local_rank, double *layer_stats,
                          const ddp_opt *opt, void *stream);

/* bf16 on the wire (an option of this library, not a step of the paper: the paper leaves the precision of the
 * exchanged parameters open, and its cost model, Sec. 3.1 / Eq. (7), charges communication per byte, so halving
 * the bytes of a layer halves its t_comm).  Reading taken here: every replica, the local one included, contributes
 * bf16_rne of its fp32 value, so that all workers average the same N buffers and stay bit-identical after a
 * synchronisation (Algorithm 1's invariant); the sum is still fp32 in rank order, times fp32(1/N), and the result is
 * an fp32 buffer.  Buffers named *16 hold bf16 bit patterns (2 bytes per element), device memory, 16-byte aligned,
 * ddp_slot_numel(slot) elements, same flat layout as ddp_pack.
 *
 * ddp_pack_wire16:            flat_local16[off_t + i] = bf16_rne(sync_t[i])
 * ddp_partial_average_wire16: flat_out[j] = ( sum_{k in rank order} widen(x16_k[j]) ) * fp32(1/N); statistics as in
 *                             ddp_partial_average with x_k = widen(x16_k).  flat_out (fp32) must not overlap any input.
 * ddp_fused_sync_update_wire16: as ddp_fused_sync_update with bf16 peer buffers; bit-identical to
 *                             ddp_pack_wire16 -> ddp_partial_average_wire16 -> ddp_unpack -> ddp_local_update. */
int ddp_pack_wire16(ddp_ctx *ctx, int slot, uint16_t *flat_local16, void *stream);
int ddp_partial_average_wire16(ddp_ctx *ctx, int slot, const uint16_t *flat_local16, const uint16_t *const *peers16, int N,
                               int local_rank, float *flat_out, double *layer_stats, void *stream);
int ddp_fused_sync_update_wire16(ddp_ctx *ctx, int slot, const uint16_t *const *peers16, int N, int local_rank,
                                 double *layer_stats, const ddp_opt *opt, void *stream);

/* Layer-wise launches for overlap with back-propagation (Sec. 3.2: the synchronisation of a layer starts as soon as
 * its backward pass has produced its gradient, while the layers below are still in BP; Algorithm 1 per layer).
 * Both calls restrict their whole-model counterpart to the registered layers [layer_first, layer_first + layer_count):
 *
 * ddp_local_update_layers:      ddp_local_update on the tensors of those layers only.
 * ddp_fused_sync_update_layers: ddp_fused_sync_update (wire_dtype DDP_F32: peers are fp32 buffers) or
 *                               ddp_fused_sync_update_wire16 (DDP_BF16: bf16 buffers) on those layers only: the ones the
 *                               slot schedules are averaged and updated, the others updated.  layer_stats has the layout of
 *                               the whole-slot call (two doubles per layer of the slot, flat order); only the entries of
 *                               scheduled layers inside the range are written.
 *                               order DDP_SYNC_THEN_UPDATE: average, then the optimizer step on the average (what the
 *                               whole-model fused calls do).  order DDP_UPDATE_THEN_SYNC: Eq. (5) / Algorithm 1 as printed:
 *                               the local value takes the optimizer step first and the result is averaged with the
 *                               peers' buffers (which then hold the peers' values after their step); bit-identical to
 *                               ddp_local_update -> ddp_pack[_wire16] -> ddp_partial_average[_wire16] -> ddp_unpack, and
 *                               the statistics are those of that average.
 *
 * Calling either for a partition of [0, L) into ranges, once each, in any order, gives bit for bit the result of the
 * whole-model call.  Calls for disjoint ranges may be in flight at the same time on different streams of the device
 * (their reduction scratch is disjoint); calls whose ranges overlap must be ordered by the caller, as must the producer
 * of the range's gradients and this call (stream order or an event).  Needs option dispatch_ways = 1 (the default),
 * else DDP_ESTATE.  A range with layer_count == 0 is a no-op. */
int ddp_local_update_layers(ddp_ctx *ctx, int layer_first, int layer_count, const ddp_opt *opt, void *stream);
enum { DDP_SYNC_THEN_UPDATE = 0, DDP_UPDATE_THEN_SYNC = 1 };
int ddp_fused_sync_update_layers(ddp_ctx *ctx, int slot, int layer_first, int layer_count, const void *const *peers,
                                 int wire_dtype, int order, int N, int local_rank, double *layer_stats, const ddp_opt *opt,
                                 void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): ddp_partial_average with its reduction scratch (one pair of fp64 partial sums per chunk of
 * mean_chunk elements, then 64 slice sums per layer of the slot) in a fixed array of DDP_STATIC_SCRATCH_BYTES inside the
 * library's device image, one copy per GPU, instead of memory owned by the context.  Same arguments, same kernels and
 * bit for bit the same flat_out and layer_stats as ddp_partial_average.  Neither this call nor anything it calls
 * allocates or frees device or pinned memory; the device address of the array is resolved once per device in ddp_create
 * (if that fails, the context still works and this call alone returns DDP_ESTATE with the reason).
 *   - A slot whose statistics need more than the fixed array (more than about 2^20 chunks: 2.1 G elements at the default
 *     mean_chunk) is rejected with DDP_ESHAPE before anything is launched; with layer_stats == NULL any size passes,
 *     since the scratch is then not used.
 *   - Every call on a GPU, from any context or thread, shares that GPU's array: calls that may overlap in time on one GPU
 *     (different streams, different contexts) race on it and must be ordered by the caller.  The array keeps the last
 *     call's contents; nothing in it has to start at zero, because every partial a call reads it has written before. */
enum { DDP_STATIC_SCRATCH_BYTES = 16 << 20 };
int ddp_partial_average_static(ddp_ctx *ctx, int slot, const float *flat_local, const float *const *peers, int N,
                               int local_rank, float *flat_out, double *layer_stats, void *stream);

/* Streams for the overlap of Sec. 3.2 on one GPU.  The paper hides a layer's synchronisation under the backward pass of
 * the layers below it; on a single GPU the synchronisation + update kernels and the backward kernels would compete for
 * the same compute units (a matrix product that fills every CU leaves no slot for a second stream).  A stream made here
 * runs its kernels only on compute units [cu_first, cu_first + cu_count) of the device's enumeration (the order of the
 * bits of hipExtStreamCreateWithCUMask, which the driver spreads evenly over the chip's XCDs), at the default priority.
 * The caller gives the backward pass a stream over one range and the layer-wise calls (ddp_fused_sync_update_layers, ...)
 * a stream over the rest, and orders the two with events as with any two streams.  The handle is a hipStream_t; it is
 * owned by the caller and released with ddp_stream_destroy once its work is complete.  `device` must be the current
 * device.  Errors: DDP_EINVAL (range), DDP_ESTATE (device not current), DDP_EHIP. */
int ddp_device_cu_count(int device, int *out_cus);
int ddp_stream_create_cu_range(int device, int cu_first, int cu_count, void **out_stream);
int ddp_stream_destroy(void *stream);

/* Measurement aid, not a step of the method: one kernel in the launch shape of the library's streaming kernels (256-thread
 * workgroups, chunk_bytes of every stream per workgroup, 128-bit buffer accesses with the streaming hint, two vectors per
 * thread and stream in flight, lds_pad bytes of unused dynamic LDS per workgroup to cap residency) that only reads n_read
 * streams and writes n_write streams of `bytes` bytes each (every written vector is 1 + the sum of the vectors read).
 * Timed by the caller with events on `stream`, it shows what the memory system gives a kernel with that mix of
 * streams: the practical ceiling beside the 8 TB/s peak that the roofline fractions are quoted against.
 *   read_ptrs / write_ptrs  host arrays of n_read / n_write device pointers, 16-byte aligned, each >= bytes long, no overlap
 *   n_read in {0, 1, 2, 3, 4, 8, 16}, n_write in [0, 4], not both 0; bytes a multiple of 16; chunk_bytes a multiple of 4096
 *   in [4096, 4 MiB]; lds_pad in [0, 65536].  Uses the current device; needs no context.  Errors: DDP_EINVAL, DDP_EALIGN,
 *   DDP_EHIP; message via ddp_last_error(NULL). */
int ddp_stream_probe(int n_read, int n_write, int64_t bytes, const void *const *read_ptrs, void *const *write_ptrs,
                     int chunk_bytes, int lds_pad, void *stream);

/* Message of the last failure on this context (ctx == NULL: last failure of ddp_create / ddp_schedule* in
 * this thread).  Never NULL; valid until the next call on the same context / thread. */
const char *ddp_last_error(const ddp_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* DREAMDDP_H */
