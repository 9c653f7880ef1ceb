// Layer-to-iteration scheduler (CPU).  Sec. 3.3 of the paper: objective P_H^L of Eq. (8), the exact optimum over
// cuts of the BP-ordered layer sequence, and Algorithm 2 (depth-first search pruned by Properties 1-3).
//
// Internal view: position j = 0..L-1 walks the layers in BP order (position j is layer L-1-j).  With prefix
// sums PB / PC of backward and communication times over positions, a non-empty set that covers positions
// [a, b) starts its communication after the backward of position a, so the backward work that can still hide
// it is rem(a) = PB[L] - PB[a+1], and its cost beyond the H plain backward passes is
//     excess(a, b) = max(0, (PC[b] - PC[a]) - rem(a)).
// Eq. (8) is then H * PB[L] + sum of excess over the non-empty sets: the first two terms of each summand of
// Eq. (8) plus the `rem` inside its max always add up to one whole backward pass.
#include <algorithm>
#include <cstdint>
#include <exception>
#include <limits>
#include <string>
#include <vector>

#include "ddp_internal.h"

namespace {

struct Instance {
    int L = 0, H = 0;
    std::vector<int64_t> PB, PC;  // prefix sums over BP-order positions, size L+1
    int64_t rem(int a) const { return PB[L] - PB[a + 1]; }
    int64_t excess(int a, int b) const {
        if (a == b) return 0;
        int64_t c = PC[b] - PC[a];
        int64_t r = rem(a);
        return c > r ? c - r : 0;
    }
    int64_t base() const { return (int64_t)H * PB[L]; }
};

int make_instance(int L, int H, const int64_t *bp, const int64_t *comm, Instance &in) {
    in.L = L;
    in.H = H;
    in.PB.assign(L + 1, 0);
    in.PC.assign(L + 1, 0);
    __int128 sb = 0, sc = 0;
    for (int j = 0; j < L; ++j) {
        int l = L - 1 - j;
        if (bp[l] < 0 || comm[l] < 0) return ddp::fail(nullptr, DDP_EINVAL, "negative time for layer " + std::to_string(l));
        sb += bp[l];
        sc += comm[l];
        in.PB[j + 1] = (int64_t)sb;
        in.PC[j + 1] = (int64_t)sc;
        if (sb * H + sc > (__int128)std::numeric_limits<int64_t>::max())
            return ddp::fail(nullptr, DDP_EINVAL, "time sums overflow int64 nanoseconds");
    }
    return DDP_OK;
}

int64_t cost_of_cuts(const Instance &in, const std::vector<int> &cut) {  // cut[h]..cut[h+1] = positions of set h
    int64_t c = in.base();
    for (int h = 0; h < in.H; ++h) c += in.excess(cut[h], cut[h + 1]);
    return c;
}

// Exact optimum by dynamic programming over (set index, first unplaced position): O(L^2 H).
// f[h][a] = least excess when positions a..L-1 are split over sets h..H-1.
std::vector<int> solve_opt(const Instance &in) {
    const int L = in.L, H = in.H;
    const int64_t INF = std::numeric_limits<int64_t>::max();
    std::vector<std::vector<int64_t>> f(H, std::vector<int64_t>(L + 1, INF));
    for (int a = 0; a <= L; ++a) f[H - 1][a] = in.excess(a, L);
    for (int h = H - 2; h >= 0; --h)
        for (int a = 0; a <= L; ++a) {
            int64_t best = INF;
            for (int b = a; b <= L; ++b) best = std::min(best, in.excess(a, b) + f[h + 1][b]);
            f[h][a] = best;
        }
    // walk forward taking, at each set, the longest run that still reaches the optimum
    std::vector<int> cut(H + 1, 0);
    int a = 0;
    for (int h = 0; h < H - 1; ++h) {
        int pick = a;
        for (int b = L; b >= a; --b)
            if (in.excess(a, b) + f[h + 1][b] == f[h][a]) {
                pick = b;
                break;
            }
        cut[h + 1] = pick;
        a = pick;
    }
    cut[H] = L;
    return cut;
}

// Algorithm 2 without recursion.  The search walks one partial solution at a time: cut[0..h] fixed, set h open and
// starting at cut[h], `pos` the next position to place.  Where neither property decides, the "delay" continuation
// (pos, h + 1) goes on a stack and the walk goes on with "assign"; a continuation taken from the stack re-opens set
// h + 1 at pos.  Everything below index h + 1 of `cut` is still what it was when the continuation was pushed, because
// the walk in between only ever wrote entries above h.  Solutions are therefore visited in the order of the recursive
// formulation with the assign-branch first, and "first minimum found" picks the same solution.
//
// The solution set can grow exponentially with min(L, H) (Sec. 3.3 bounds it by a power of two): the walk stops after
// kAlg2StepBudget placement steps and reports that, so that no instance can hold the caller for long.
constexpr int64_t kAlg2StepBudget = 50'000'000;

struct Alg2Result {
    std::vector<int> best;
    int64_t best_cost = -1;
    int64_t n_solutions = 0;
    bool exhausted = false;  // the step budget ran out before the search was complete
};

Alg2Result solve_alg2(const Instance &in, int64_t step_budget = kAlg2StepBudget) {
    const int L = in.L, H = in.H;
    struct Delayed {
        int pos, h;  // set h opens at position pos
    };
    Alg2Result res;
    std::vector<int> cut(H + 1, 0);
    std::vector<Delayed> stack;
    stack.push_back({0, 0});
    int64_t steps = 0;
    while (!stack.empty()) {
        const Delayed fr = stack.back();
        stack.pop_back();
        int pos = fr.pos, h = fr.h;
        cut[h] = pos;
        for (;;) {
            if (++steps > step_budget) {
                res.exhausted = true;
                return res;
            }
            if (pos == L || h == H - 1) {
                // every layer placed (later sets stay empty), or the last set takes all that is left
                for (int k = h + 1; k <= H; ++k) cut[k] = L;
                int64_t c = cost_of_cuts(in, cut);
                if (res.best_cost < 0 || c < res.best_cost) {
                    res.best_cost = c;
                    res.best = cut;
                }
                ++res.n_solutions;
                break;
            }
            const int start = cut[h];
            if (pos == start) {  // Property 3: an empty set takes the layer
                ++pos;
                continue;
            }
            const int64_t r = in.rem(start);
            const int64_t c_set = in.PC[pos] - in.PC[start];
            const int64_t c_with = in.PC[pos + 1] - in.PC[start];
            if (r >= c_with) {  // Definition 3 / Property 1: the assignment is hidden, take it
                ++pos;
            } else if (r < c_set) {  // Property 2: the set overflows already, the layer waits for the next set
                cut[h + 1] = pos;
                ++h;
            } else {  // neither property decides: keep "delay" for later, go on with "assign"
                stack.push_back({pos, h + 1});
                ++pos;
            }
        }
    }
    return res;
}

int alg2_exhausted(const char *who) {
    return ddp::fail(nullptr, DDP_ESCHED, std::string(who) + ": Algorithm 2's search exceeded " + std::to_string(kAlg2StepBudget) +
                                              " steps on this instance (its solution set grows exponentially); use DDP_SCHED_OPT, the exact "
                                              "O(L^2 H) optimum of the same objective");
}

void emit_cut(int L, int H, const std::vector<int> &cut, int32_t *out_slot, int32_t *out_set_ptr, int32_t *out_set_layers) {
    for (int h = 0; h <= H; ++h) out_set_ptr[h] = cut[h];
    for (int h = 0; h < H; ++h)
        for (int j = cut[h]; j < cut[h + 1]; ++j) {
            out_set_layers[j] = L - 1 - j;
            out_slot[L - 1 - j] = h;
        }
}

}  // namespace

extern "C" int ddp_schedule(int policy, int L, int H, const int64_t *t_fp_ns, const int64_t *t_bp_ns,
                            const int64_t *t_comm_ns, int32_t *out_slot, int32_t *out_set_ptr, int32_t *out_set_layers,
                            int64_t *out_cost_ns) {
    try {
        (void)t_fp_ns;  // R * t_FP is a constant of Eq. (7); it does not influence the partition
        if (L < 1 || H < 1) return ddp::fail(nullptr, DDP_EINVAL, "ddp_schedule: L and H must be >= 1");
        if (!out_slot || !out_set_ptr || !out_set_layers) return ddp::fail(nullptr, DDP_EINVAL, "ddp_schedule: NULL output");
        if (policy < DDP_SCHED_ENP || policy > DDP_SCHED_ALG2) return ddp::fail(nullptr, DDP_EINVAL, "ddp_schedule: unknown policy");
        const bool needs_times = policy == DDP_SCHED_OPT || policy == DDP_SCHED_ALG2;
        if (needs_times && (!t_bp_ns || !t_comm_ns)) return ddp::fail(nullptr, DDP_EINVAL, "ddp_schedule: policy needs t_bp_ns and t_comm_ns");
        Instance in;
        const bool have_times = t_bp_ns && t_comm_ns;
        if (have_times) {
            int rc = make_instance(L, H, t_bp_ns, t_comm_ns, in);
            if (rc != DDP_OK) return rc;
        }
        if (out_cost_ns) *out_cost_ns = -1;

        if (policy == DDP_SCHED_ROUND_ROBIN) {
            int n = 0;
            for (int s = 0; s < H; ++s) {
                out_set_ptr[s] = n;
                for (int l = L - 1; l >= 0; --l)
                    if (l % H == s) {
                        out_set_layers[n++] = l;
                        out_slot[l] = s;
                    }
            }
            out_set_ptr[H] = n;
            return DDP_OK;
        }
        if (policy == DDP_SCHED_EVERY) {
            int n = 0;
            for (int s = 0; s < H; ++s) {
                out_set_ptr[s] = n;
                for (int l = L - 1; l >= 0; --l) out_set_layers[n++] = l;
            }
            out_set_ptr[H] = n;
            for (int l = 0; l < L; ++l) out_slot[l] = 0;
            return DDP_OK;
        }

        std::vector<int> cut(H + 1, 0);
        if (policy == DDP_SCHED_ENP) {
            for (int h = 0; h < H; ++h) cut[h + 1] = cut[h] + L / H + (h < L % H ? 1 : 0);
        } else if (policy == DDP_SCHED_FULL) {
            cut[H] = L;  // sets 0..H-2 empty, the last one holds everything: synchronise when (r+1) % H == 0
        } else if (policy == DDP_SCHED_OPT) {
            cut = solve_opt(in);
        } else {
            Alg2Result r = solve_alg2(in);
            if (r.exhausted) return alg2_exhausted("ddp_schedule");
            cut = std::move(r.best);
        }
        emit_cut(L, H, cut, out_slot, out_set_ptr, out_set_layers);
        if (out_cost_ns && have_times) *out_cost_ns = cost_of_cuts(in, cut);
        return DDP_OK;
    } catch (...) {
        return ddp::fail_nothrow(nullptr, DDP_ENOMEM, "ddp_schedule: host allocation failed");
    }
}

extern "C" int ddp_schedule_cost(int L, int H, const int64_t *t_bp_ns, const int64_t *t_comm_ns, const int32_t *set_ptr,
                                 const int32_t *set_layers, int64_t *out_cost_ns) {
    try {
        if (L < 1 || H < 1 || !t_bp_ns || !t_comm_ns || !set_ptr || !set_layers || !out_cost_ns)
            return ddp::fail(nullptr, DDP_EINVAL, "ddp_schedule_cost: bad argument");
        Instance in;
        int rc = make_instance(L, H, t_bp_ns, t_comm_ns, in);
        if (rc != DDP_OK) return rc;
        if (set_ptr[0] != 0 || set_ptr[H] != L) return ddp::fail(nullptr, DDP_ESCHED, "ddp_schedule_cost: sets must cover every layer once");
        std::vector<int> cut(H + 1, 0);
        for (int h = 0; h < H; ++h) {
            if (set_ptr[h + 1] < set_ptr[h]) return ddp::fail(nullptr, DDP_ESCHED, "ddp_schedule_cost: set_ptr not monotone");
            cut[h + 1] = set_ptr[h + 1];
        }
        for (int j = 0; j < L; ++j)
            if (set_layers[j] != L - 1 - j)
                return ddp::fail(nullptr, DDP_ESCHED, "ddp_schedule_cost: sets are not a cut of the BP-ordered layer sequence");
        *out_cost_ns = cost_of_cuts(in, cut);
        return DDP_OK;
    } catch (...) {
        return ddp::fail_nothrow(nullptr, DDP_ENOMEM, "ddp_schedule_cost: host allocation failed");
    }
}

extern "C" int ddp_schedule_alg2_solutions(int L, int H, const int64_t *t_bp_ns, const int64_t *t_comm_ns, int64_t *out_count) {
    try {
        if (L < 1 || H < 1 || !t_bp_ns || !t_comm_ns || !out_count)
            return ddp::fail(nullptr, DDP_EINVAL, "ddp_schedule_alg2_solutions: bad argument");
        Instance in;
        int rc = make_instance(L, H, t_bp_ns, t_comm_ns, in);
        if (rc != DDP_OK) return rc;
        const Alg2Result r = solve_alg2(in);
        if (r.exhausted) return alg2_exhausted("ddp_schedule_alg2_solutions");
        *out_count = r.n_solutions;
        return DDP_OK;
    } catch (...) {
        return ddp::fail_nothrow(nullptr, DDP_ENOMEM, "ddp_schedule_alg2_solutions: host allocation failed");
    }
}

// Reads a CSR schedule that must be a cut of the BP-ordered layer sequence; fills cut[0..H].
static int read_cut(const char *who, int L, int H, const int32_t *set_ptr, const int32_t *set_layers, std::vector<int> &cut) {
    if (set_ptr[0] != 0 || set_ptr[H] != L) return ddp::fail(nullptr, DDP_ESCHED, std::string(who) + ": sets must cover every layer once");
    cut.assign(H + 1, 0);
    for (int h = 0; h < H; ++h) {
        if (set_ptr[h + 1] < set_ptr[h]) return ddp::fail(nullptr, DDP_ESCHED, std::string(who) + ": set_ptr not monotone");
        cut[h + 1] = set_ptr[h + 1];
    }
    for (int j = 0; j < L; ++j)
        if (set_layers[j] != L - 1 - j)
            return ddp::fail(nullptr, DDP_ESCHED, std::string(who) + ": sets are not a cut of the BP-ordered layer sequence");
    return DDP_OK;
}

// Sec. 3.4, Eq. (12).  The extra layers of a set are always a prefix of the BP order, so the work per set is one
// walk over a prefix sum: the set may take top layers while its total communication stays within
// max(rem, own communication), i.e. within the backward work that hides it (or not at all if it already overflows).
extern "C" int ddp_schedule_fill_bubbles(int L, int H, const int64_t *t_bp_ns, const int64_t *t_comm_ns, const int32_t *set_ptr,
                                         const int32_t *set_layers, int32_t *out_set_ptr, int32_t *out_set_layers, int32_t *out_extra) {
    try {
        if (L < 1 || H < 1 || !t_bp_ns || !t_comm_ns || !set_ptr || !set_layers || !out_set_ptr || !out_set_layers)
            return ddp::fail(nullptr, DDP_EINVAL, "ddp_schedule_fill_bubbles: bad argument");
        Instance in;
        int rc = make_instance(L, H, t_bp_ns, t_comm_ns, in);
        if (rc != DDP_OK) return rc;
        std::vector<int> cut;
        rc = read_cut("ddp_schedule_fill_bubbles", L, H, set_ptr, set_layers, cut);
        if (rc != DDP_OK) return rc;
        int n = 0;
        for (int h = 0; h < H; ++h) {
            const int a = cut[h], b = cut[h + 1];
            const bool empty = a == b;
            const int64_t rem = in.rem(empty ? 0 : a);  // an empty set would start with the top layer
            const int64_t own = in.PC[b] - in.PC[a];
            const int64_t budget = std::max(rem, own);
            const int limit = empty ? L : a;  // stay disjoint from the set itself
            int e = 0;
            while (e < limit && own + in.PC[e + 1] <= budget) ++e;  // PC[e+1] = communication of the top e+1 layers
            out_set_ptr[h] = n;
            for (int j = 0; j < e; ++j) out_set_layers[n++] = L - 1 - j;
            for (int j = a; j < b; ++j) out_set_layers[n++] = L - 1 - j;
            if (out_extra) out_extra[h] = e;
        }
        out_set_ptr[H] = n;
        return DDP_OK;
    } catch (...) {
        return ddp::fail_nothrow(nullptr, DDP_ENOMEM, "ddp_schedule_fill_bubbles: host allocation failed");
    }
}

// Eq. (7) on the time line of one iteration: layer l's backward is done at D(l) = sum of t_bp over layers >= l
// (= PB[L-l] in BP positions); communications of the iteration's set run one after the other, each starting
// once its layer's backward is done.  The iteration ends when both the backward pass and the last communication
// have ended.  Works for any set listed in BP order, contiguous or not.
extern "C" int ddp_schedule_time_model(int L, int H, const int64_t *t_fp_ns, const int64_t *t_bp_ns, const int64_t *t_comm_ns,
                                       const int32_t *set_ptr, const int32_t *set_layers, int64_t *out_iter_ns,
                                       int64_t *out_exposed_ns, int64_t *out_period_ns) {
    try {
        if (L < 1 || H < 1 || !t_bp_ns || !t_comm_ns || !set_ptr || !set_layers || !out_iter_ns)
            return ddp::fail(nullptr, DDP_EINVAL, "ddp_schedule_time_model: bad argument");
        Instance in;
        int rc = make_instance(L, H, t_bp_ns, t_comm_ns, in);
        if (rc != DDP_OK) return rc;
        __int128 fp_total = 0;
        if (t_fp_ns)
            for (int l = 0; l < L; ++l) {
                if (t_fp_ns[l] < 0) return ddp::fail(nullptr, DDP_EINVAL, "ddp_schedule_time_model: negative forward time");
                fp_total += t_fp_ns[l];
            }
        if (set_ptr[0] != 0) return ddp::fail(nullptr, DDP_ESCHED, "ddp_schedule_time_model: set_ptr[0] must be 0");
        __int128 period = 0;
        for (int h = 0; h < H; ++h) {
            if (set_ptr[h + 1] < set_ptr[h]) return ddp::fail(nullptr, DDP_ESCHED, "ddp_schedule_time_model: set_ptr not monotone");
            __int128 comm_end = 0;
            int prev = L;
            for (int j = set_ptr[h]; j < set_ptr[h + 1]; ++j) {
                const int l = set_layers[j];
                if (l < 0 || l >= L || l >= prev)
                    return ddp::fail(nullptr, DDP_ESCHED, "ddp_schedule_time_model: a set must list distinct layers in BP order (descending)");
                prev = l;
                const __int128 done = in.PB[L - l];
                comm_end = std::max(done, comm_end) + t_comm_ns[l];
            }
            const __int128 bp_end = in.PB[L];
            const __int128 end = std::max(bp_end, comm_end) + fp_total;
            if (end > (__int128)std::numeric_limits<int64_t>::max() || period + end > (__int128)std::numeric_limits<int64_t>::max())
                return ddp::fail(nullptr, DDP_EINVAL, "ddp_schedule_time_model: times overflow int64 nanoseconds");
            out_iter_ns[h] = (int64_t)end;
            if (out_exposed_ns) out_exposed_ns[h] = (int64_t)(comm_end > bp_end ? comm_end - bp_end : 0);
            period += end;
        }
        if (out_period_ns) *out_period_ns = (int64_t)period;
        return DDP_OK;
    } catch (...) {
        return ddp::fail_nothrow(nullptr, DDP_ENOMEM, "ddp_schedule_time_model: host allocation failed");
    }
}
