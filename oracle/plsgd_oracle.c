/*
 * CPU oracle for one worker's partial-synchronisation + local-update step of local SGD with partial
 * synchronisation (PLSGD), and for the layer-to-iteration scheduling problem.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, by-the-definition implementation used only to
 * check the GPU library and to be timed beside it as a CPU baseline.  It shares no code with the GPU path,
 * includes none of its headers, and nothing in the product may call it.
 *
 * What is followed:
 *   - Algorithm 1 and Definition 1 / Eq. (5): every iteration each worker updates all layers locally; the
 *     layers whose subset index matches the iteration's phase are replaced by the average over the workers.
 *   - Sec. 3.4 (divergence): Gamma = 1/K sum_k ||wbar - w^k||^2, taken per layer.
 *   - Sec. 3.3, Eq. (8): the scheduling objective P_H^L over partitions of the layer sequence L..1 into H
 *     consecutive sets; Definitions 2-3, Properties 1-3 and Algorithm 2: the pruned depth-first search.
 *
 * Readings where the paper is silent (each also listed in the design notes):
 *   - reduction: fp32, one add at a time, replicas in global rank order, then one multiply by 1.0f/N;
 *   - mixed precision: the fp32 master copy is what is averaged; the bf16 model copy is re-derived from it
 *     by round-to-nearest-even;
 *   - optimizers: SGD with momentum (buf = mu*buf + g; p = p - lr*buf) and AdamW with decoupled decay and
 *     bias correction; every product and sum is its own fp32 operation (build with -ffp-contract=off);
 *   - scheduling: integer nanoseconds; "brute force" means all ways to cut the BP-ordered layer sequence
 *     into H consecutive, possibly empty, sets.
 *
 * Parity pins live in tests/test_oracle_*.py (closed forms, invariants, library witnesses, hand-worked
 * schedules).  No function here is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------------------------------------ */
/* bf16 <-> fp32                                                                                           */
/* ------------------------------------------------------------------------------------------------------ */

/* Round an fp32 value to bfloat16 (upper 16 bits of the fp32 pattern), ties to even; NaN stays a quiet NaN. */
static uint16_t bf16_rne_one(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lower = u & 0xffffu;
    uint32_t upper = u >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) upper += 1u; /* carries into exponent correctly */
    return (uint16_t)upper;
}

static float bf16_widen_one(uint16_t h) {
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

void orc_bf16_rne(const float *x, uint16_t *out, int64_t n) {
    for (int64_t i = 0; i < n; ++i) out[i] = bf16_rne_one(x[i]);
}

void orc_bf16_widen(const uint16_t *x, float *out, int64_t n) {
    for (int64_t i = 0; i < n; ++i) out[i] = bf16_widen_one(x[i]);
}

/* ------------------------------------------------------------------------------------------------------ */
/* flat layout of one iteration's scheduled layers                                                         */
/* ------------------------------------------------------------------------------------------------------ */

/* Dense concatenation order: the set's layers in the order given (BP order), each layer's tensors in
 * registration order.  dst_off[t] = -1 for tensors that are not scheduled.  Returns the total element count. */
int64_t orc_slot_offsets(int T, const int32_t *layer_of, const int64_t *numel, int n_set, const int32_t *set_layers,
                         int64_t *dst_off, int32_t *order, int32_t *n_order) {
    for (int t = 0; t < T; ++t) dst_off[t] = -1;
    int64_t off = 0;
    int cnt = 0;
    for (int j = 0; j < n_set; ++j) {
        for (int t = 0; t < T; ++t) {
            if (layer_of[t] != set_layers[j]) continue;
            dst_off[t] = off;
            off += numel[t];
            order[cnt++] = t;
        }
    }
    *n_order = cnt;
    return off;
}

/* gather: flat[off_t + i] = tensor_t[i] */
void orc_pack(int n, const float *const *src, const int64_t *numel, const int64_t *off, float *flat) {
    for (int t = 0; t < n; ++t)
        for (int64_t i = 0; i < numel[t]; ++i) flat[off[t] + i] = src[t][i];
}

/* scatter: tensor_t[i] = flat[off_t + i]; model copy (may be NULL per tensor) = bf16 RNE of the same value */
void orc_unpack(int n, float *const *dst, uint16_t *const *model, const int64_t *numel, const int64_t *off,
                const float *flat) {
    for (int t = 0; t < n; ++t) {
        for (int64_t i = 0; i < numel[t]; ++i) {
            float v = flat[off[t] + i];
            dst[t][i] = v;
            if (model && model[t]) model[t][i] = bf16_rne_one(v);
        }
    }
}

/* ------------------------------------------------------------------------------------------------------ */
/* Eq. (5), second case: the average over the N replicas                                                   */
/* ------------------------------------------------------------------------------------------------------ */

/* x[k] is replica k's flat buffer, k in global rank order.  out may alias any x[k]. */
void orc_mean(int N, const float *const *x, int64_t n, float *out) {
    const float inv_n = 1.0f / (float)N;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        float acc = x[0][i];
        for (int k = 1; k < N; ++k) acc = acc + x[k][i];
        out[i] = acc * inv_n;
    }
}

/* Per-layer divergence and squared norm over flat range [begin, end):
 *   gamma = (1/N) sum_k sum_i (mean[i] - x_k[i])^2,  msq = sum_i mean[i]^2.
 * Each difference is formed in fp32 (the precision the replicas are held in); its square is exact in fp64.
 * The running sums are kept in extended precision (x87 long double, 64-bit mantissa): a plain fp64 running sum
 * over the 5e8 terms of a 65 M-element layer drifts by 5e-10 relative, which would make the oracle the less
 * accurate side of the comparison.  The result is rounded to fp64 once at the end. */
void orc_layer_stats(int N, const float *const *x, const float *mean, int64_t begin, int64_t end, double *gamma,
                     double *msq) {
    long double g = 0.0L, m = 0.0L;
    for (int64_t i = begin; i < end; ++i) {
        for (int k = 0; k < N; ++k) {
            float d = mean[i] - x[k][i];
            g += (long double)((double)d * (double)d);
        }
        m += (long double)((double)mean[i] * (double)mean[i]);
    }
    *gamma = (double)(g / (long double)N);
    *msq = (double)m;
}

/* ------------------------------------------------------------------------------------------------------ */
/* bf16 on the wire (an option of this build, not of the paper, which does not discuss precision)           */
/* ------------------------------------------------------------------------------------------------------ */

/* Reading: what travels is bf16_rne of each replica's fp32 value, the local replica's included, so that every
 * worker averages the same N numbers and all replicas still agree bit for bit after a synchronisation.  The sum
 * runs over the widened values in fp32, rank order, then one multiply by 1.0f/N; the result is kept in fp32. */
void orc_pack_wire16(int n, const float *const *src, const int64_t *numel, const int64_t *off, uint16_t *flat) {
    for (int t = 0; t < n; ++t)
        for (int64_t i = 0; i < numel[t]; ++i) flat[off[t] + i] = bf16_rne_one(src[t][i]);
}

void orc_mean_wire16(int N, const uint16_t *const *x, int64_t n, float *out) {
    const float inv_n = 1.0f / (float)N;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        float acc = bf16_widen_one(x[0][i]);
        for (int k = 1; k < N; ++k) acc = acc + bf16_widen_one(x[k][i]);
        out[i] = acc * inv_n;
    }
}

/* Divergence and norm as in orc_layer_stats, measured against the values that were actually averaged. */
void orc_layer_stats_wire16(int N, const uint16_t *const *x, const float *mean, int64_t begin, int64_t end, double *gamma,
                            double *msq) {
    long double g = 0.0L, m = 0.0L;
    for (int64_t i = begin; i < end; ++i) {
        for (int k = 0; k < N; ++k) {
            float d = mean[i] - bf16_widen_one(x[k][i]);
            g += (long double)((double)d * (double)d);
        }
        m += (long double)((double)mean[i] * (double)mean[i]);
    }
    *gamma = (double)(g / (long double)N);
    *msq = (double)m;
}

/* ------------------------------------------------------------------------------------------------------ */
/* Eq. (5), first case: the local update (Algorithm 1, "update model"), with the optimizers of Sec. 5.1     */
/* ------------------------------------------------------------------------------------------------------ */

/* SGD with momentum, no dampening, no Nesterov, no weight decay.  mu = 0 is the plain step of Sec. 2.1. */
void orc_sgdm(float *p, const float *g, float *buf, int64_t n, float lr, float mu) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        float b = mu * buf[i];
        b = b + g[i];
        buf[i] = b;
        float s = lr * b;
        p[i] = p[i] - s;
    }
}

/* Host-side scalars of one AdamW step (1-based step t).  Bias corrections are formed in fp64 and handed to
 * the elementwise loop as fp32 factors. */
void orc_adamw_scalars(float lr, float beta1, float beta2, float wd, int64_t step, float *out5) {
    double bc1 = 1.0 - pow((double)beta1, (double)step);
    double bc2 = 1.0 - pow((double)beta2, (double)step);
    float inv_bc1 = (float)(1.0 / bc1);
    float rsqrt_bc2 = (float)(1.0 / sqrt(bc2));
    out5[0] = 1.0f - beta1;
    out5[1] = 1.0f - beta2;
    out5[2] = 1.0f - lr * wd;   /* decoupled decay factor */
    out5[3] = lr * inv_bc1;     /* step size */
    out5[4] = rsqrt_bc2;
}

/* AdamW on fp32 master p with fp32 moments m, v.  The gradient comes as fp32 (g32) or as bf16 (g16, widened
 * exactly); exactly one of the two is non-NULL.  model (nullable) receives bf16 RNE of the new p. */
void orc_adamw(float *p, const float *g32, const uint16_t *g16, float *m, float *v, uint16_t *model, int64_t n,
               float lr, float beta1, float beta2, float eps, float wd, int64_t step) {
    float s[5];
    orc_adamw_scalars(lr, beta1, beta2, wd, step, s);
    const float omb1 = s[0], omb2 = s[1], decay = s[2], step_size = s[3], rsqrt_bc2 = s[4];
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        float g = g32 ? g32[i] : bf16_widen_one(g16[i]);
        float a = beta1 * m[i];
        float b = omb1 * g;
        float mi = a + b;
        float c = beta2 * v[i];
        float d = omb2 * g;
        float e = d * g;
        float vi = c + e;
        float pi = p[i] * decay;
        float r = sqrtf(vi);
        float den = r * rsqrt_bc2;
        den = den + eps;
        float q = mi / den;
        float u = step_size * q;
        pi = pi - u;
        m[i] = mi;
        v[i] = vi;
        p[i] = pi;
        if (model) model[i] = bf16_rne_one(pi);
    }
}

/* ------------------------------------------------------------------------------------------------------ */
/* Scheduling: Eq. (8) and Algorithm 2                                                                     */
/* ------------------------------------------------------------------------------------------------------ */

/* Layers are 0-based, 0 = input side; BP visits L-1, L-2, ..., 0.  A schedule is a cut of that sequence into
 * H consecutive sets: sizes[h] layers go to set h (h = 0..H-1), sum sizes = L. */

/* Eq. (8), written term by term as printed:
 *   sum_h [ t_BP(L_1..L_{h-1}) + t_BP(h0) + max( t_BP(L_h..L_H) - t_BP(h0), t_COMM(L_h) ) ]
 * h0 = first layer of set h in BP order; t_COMM(L_h) = plain sum over the set (Eq. (10) footnote text).
 * For an empty set there is no h0: the iteration costs the whole backward pass and hides nothing. */
int64_t orc_sched_cost(int L, int H, const int64_t *bp, const int64_t *comm, const int32_t *sizes) {
    int64_t total = 0;
    int pos = 0; /* number of layers (in BP order) already placed in earlier sets */
    for (int h = 0; h < H; ++h) {
        int64_t bp_before = 0; /* t_BP of sets 1..h-1 */
        for (int j = 0; j < pos; ++j) bp_before += bp[L - 1 - j];
        int64_t bp_from = 0;   /* t_BP of sets h..H */
        for (int j = pos; j < L; ++j) bp_from += bp[L - 1 - j];
        if (sizes[h] == 0) {
            total += bp_before + bp_from;
            continue;
        }
        int h0 = L - 1 - pos;
        int64_t c = 0;
        for (int j = pos; j < pos + sizes[h]; ++j) c += comm[L - 1 - j];
        int64_t rem = bp_from - bp[h0];
        total += bp_before + bp[h0] + (rem > c ? rem : c);
        pos += sizes[h];
    }
    return total;
}

static int sizes_lex_greater(int H, const int32_t *a, const int32_t *b) {
    for (int h = 0; h < H; ++h) {
        if (a[h] != b[h]) return a[h] > b[h];
    }
    return 0;
}

static void brute_rec(int L, int H, const int64_t *bp, const int64_t *comm, int h, int left, int32_t *cur,
                      int32_t *best, int64_t *best_cost, int64_t *count) {
    if (h == H - 1) {
        cur[h] = left;
        int64_t c = orc_sched_cost(L, H, bp, comm, cur);
        ++*count;
        if (*best_cost < 0 || c < *best_cost || (c == *best_cost && sizes_lex_greater(H, cur, best))) {
            *best_cost = c;
            memcpy(best, cur, sizeof(int32_t) * (size_t)H);
        }
        return;
    }
    for (int s = 0; s <= left; ++s) {
        cur[h] = s;
        brute_rec(L, H, bp, comm, h + 1, left - s, cur, best, best_cost, count);
    }
}

/* Exhaustive search over every cut (C(L+H-1, H-1) of them).  Among equal costs the lexicographically largest
 * size vector wins (synchronise as early as possible).  Returns the optimum; n_enumerated is for tests. */
int64_t orc_sched_brute(int L, int H, const int64_t *bp, const int64_t *comm, int32_t *best_sizes,
                        int64_t *n_enumerated) {
    int32_t *cur = (int32_t *)calloc((size_t)H, sizeof(int32_t));
    int64_t best = -1, count = 0;
    brute_rec(L, H, bp, comm, 0, L, cur, best_sizes, &best, &count);
    free(cur);
    if (n_enumerated) *n_enumerated = count;
    return best;
}

/* Algorithm 2, procedure SolveSubProblem.  State: sizes[] of sets 0..h, next layer index in BP order `pos`
 * (layer id L-1-pos), current set h.  The printed listing recurses with an undefined copy and with h-1 in its
 * search branch; following Eq. (10) the two branches are "assign l to set h, go on with l-1 in set h" and
 * "leave set h, try l in set h+1".  Solutions are collected in visiting order, assign-branch first. */
typedef struct {
    int L, H;
    const int64_t *bp, *comm;
    int32_t *omega; /* n_solutions x H */
    int64_t cap, n;
} alg2_t;

static void alg2_record(alg2_t *a, const int32_t *sizes) {
    if (a->n < a->cap) memcpy(a->omega + a->n * a->H, sizes, sizeof(int32_t) * (size_t)a->H);
    a->n++;
}

static void alg2_rec(alg2_t *a, int32_t *sizes, int pos, int h) {
    const int L = a->L, H = a->H;
    if (pos == L) { /* l == 0: every layer placed; later sets stay empty */
        alg2_record(a, sizes);
        return;
    }
    if (h == H - 1) { /* last set takes all remaining layers */
        int32_t keep = sizes[h];
        sizes[h] += L - pos;
        alg2_record(a, sizes);
        sizes[h] = keep;
        return;
    }
    int l = L - 1 - pos;
    if (sizes[h] == 0) { /* Property 3, at-least-one */
        sizes[h] = 1;
        alg2_rec(a, sizes, pos + 1, h);
        sizes[h] = 0;
        return;
    }
    int h0 = l + sizes[h]; /* first layer of set h */
    int64_t rem = 0;       /* t_BP(L_h..L_H) - t_BP(h0): backward work left after h0's own backward */
    for (int j = 0; j < h0; ++j) rem += a->bp[j];
    int64_t c_set = 0;
    for (int j = l + 1; j <= h0; ++j) c_set += a->comm[j];
    int64_t c_with = c_set + a->comm[l];
    if (rem >= c_with) { /* Definition 3 / Property 1: communication-hide assignment */
        sizes[h] += 1;
        alg2_rec(a, sizes, pos + 1, h);
        sizes[h] -= 1;
    } else if (rem < c_set) { /* Property 2: the set already overflows, delay l */
        alg2_rec(a, sizes, pos, h + 1);
    } else { /* search both */
        sizes[h] += 1;
        alg2_rec(a, sizes, pos + 1, h);
        sizes[h] -= 1;
        alg2_rec(a, sizes, pos, h + 1);
    }
}

/* Runs the DFS, stores up to omega_cap solutions (each H sizes) in omega, returns |Omega|.
 * best_sizes = first solution of minimal Eq. (8) cost (strict <), best_cost its cost. */
int64_t orc_sched_alg2(int L, int H, const int64_t *bp, const int64_t *comm, int32_t *best_sizes, int64_t *best_cost,
                       int32_t *omega, int64_t omega_cap) {
    alg2_t a = {L, H, bp, comm, omega, omega_cap, 0};
    int32_t *sizes = (int32_t *)calloc((size_t)H, sizeof(int32_t));
    alg2_rec(&a, sizes, 0, 0);
    free(sizes);
    int64_t nb = a.n < a.cap ? a.n : a.cap;
    int64_t bc = -1;
    for (int64_t s = 0; s < nb; ++s) {
        int64_t c = orc_sched_cost(L, H, bp, comm, omega + s * H);
        if (bc < 0 || c < bc) {
            bc = c;
            memcpy(best_sizes, omega + s * H, sizeof(int32_t) * (size_t)H);
        }
    }
    *best_cost = bc;
    return a.n;
}

/* Example 1 (equal-number partition): consecutive groups of floor/ceil(L/H) layers in BP order, the
 * remainder going to the earliest sets. */
void orc_sched_enp(int L, int H, int32_t *sizes) {
    for (int h = 0; h < H; ++h) sizes[h] = L / H + (h < L % H ? 1 : 0);
}

/* ------------------------------------------------------------------------------------------------------ */
/* Eq. (7): wall-clock model with communication timestamps; Sec. 3.4 / Eq. (12): filling the bubbles       */
/* ------------------------------------------------------------------------------------------------------ */

/* One summand of Eq. (7) as printed, for the set that covers BP positions [pos, pos+size) (position j is layer
 * L-1-j): t_BP(sets before) + t_BP(h0) + max( t_BP(sets h..H) - t_BP(h0), t_COMM(L_h) ), where
 *   tau(h_0) = t_BP(h_0),  tau(h_j) = max( t_BP(h_0..h_j), tau(h_{j-1}) + t_COMM(h_{j-1}) ),
 *   t_COMM(L_h) = tau(h_last) + t_COMM(h_last) - tau(h_0).
 * An empty set costs one whole backward pass. */
int64_t orc_eq7_summand(int L, const int64_t *bp, const int64_t *comm, int pos, int size) {
    int64_t before = 0, from = 0;
    for (int j = 0; j < pos; ++j) before += bp[L - 1 - j];
    for (int j = pos; j < L; ++j) from += bp[L - 1 - j];
    if (size == 0) return before + from;
    int h0 = L - 1 - pos;
    int64_t bp_run = bp[h0]; /* t_BP(h_0..h_j), running */
    int64_t tau0 = bp_run, tau = tau0;
    for (int j = 1; j < size; ++j) {
        int prev = L - 1 - (pos + j - 1), cur = L - 1 - (pos + j);
        bp_run += bp[cur];
        int64_t after_prev = tau + comm[prev];
        tau = bp_run > after_prev ? bp_run : after_prev;
    }
    int last = L - 1 - (pos + size - 1);
    int64_t span = tau + comm[last] - tau0;
    int64_t rem = from - bp[h0];
    return before + bp[h0] + (rem > span ? rem : span);
}

/* The same model for an arbitrary set given as layer ids in BP order (descending), on the time line of one
 * iteration's backward pass: layer l finishes its backward at done(l) = sum of bp over layers >= l; a layer's
 * communication starts when its backward is done and the previous communication has ended.  Returns the end of
 * backward-plus-communication; *exposed = how far the communication runs past the end of the backward pass. */
int64_t orc_iteration_timeline(int L, const int64_t *bp, const int64_t *comm, int n, const int32_t *layers, int64_t *exposed) {
    int64_t total = 0;
    for (int l = 0; l < L; ++l) total += bp[l];
    int64_t comm_end = 0;
    for (int j = 0; j < n; ++j) {
        int l = layers[j];
        int64_t done = 0;
        for (int k = l; k < L; ++k) done += bp[k];
        int64_t start = done > comm_end ? done : comm_end;
        comm_end = start + comm[l];
    }
    if (exposed) *exposed = comm_end > total ? comm_end - total : 0;
    return comm_end > total ? comm_end : total;
}

/* Sec. 3.4, Eq. (12), Algorithm 2 lines 3-6: after scheduling, set h additionally synchronises the top layers
 * L-1, L-2, ..., l (a prefix of the BP order, disjoint from the set) as long as
 *   max( rem(h0), t_COMM(L_h) + t_COMM(extra) ) <= max( rem(h0), t_COMM(L_h) ),
 * with plain sums for t_COMM and h0 the set's own first layer.  The largest such prefix is taken.  An empty set
 * has no h0 of its own: its first layer would be the top layer, so rem is taken after the top layer's backward.
 * sizes[] describes the cut; extra[h] receives the number of top layers added to set h. */
void orc_fill_bubbles(int L, int H, const int64_t *bp, const int64_t *comm, const int32_t *sizes, int32_t *extra) {
    int pos = 0;
    for (int h = 0; h < H; ++h) {
        int limit = sizes[h] ? pos : L;          /* the prefix must stay disjoint from the set */
        int h0 = sizes[h] ? L - 1 - pos : L - 1;
        int64_t rem = 0;
        for (int l = 0; l < h0; ++l) rem += bp[l];
        int64_t c_set = 0;
        for (int j = pos; j < pos + sizes[h]; ++j) c_set += comm[L - 1 - j];
        int64_t budget = rem > c_set ? rem : c_set;  /* right-hand side of Eq. (12) */
        int e = 0;
        int64_t c_extra = 0;
        while (e < limit) {
            int64_t with = c_set + c_extra + comm[L - 1 - e];
            int64_t lhs = rem > with ? rem : with;
            if (lhs > budget) break;
            c_extra += comm[L - 1 - e];
            ++e;
        }
        extra[h] = e;
        pos += sizes[h];
    }
}
