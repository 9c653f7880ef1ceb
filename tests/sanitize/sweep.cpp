// Host-sanitizer sweep: the library's scheduler (ddp_schedule.cpp, built for the host with a stub for the error
// recorder) and the CPU oracle (plsgd_oracle.c) run random instances side by side under AddressSanitizer and
// UndefinedBehaviorSanitizer.  Any out-of-bounds access, overflow or disagreement ends the program with a non-zero status.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <string>
#include <vector>

#include "dreamddp.h"

struct ddp_ctx;
namespace ddp {
static std::string g_last;
int fail(const ddp_ctx *, int code, const std::string &msg) {
    g_last = msg;
    return code;
}
}  // namespace ddp

extern "C" {
int64_t orc_sched_cost(int L, int H, const int64_t *bp, const int64_t *comm, const int32_t *sizes);
int64_t orc_sched_brute(int L, int H, const int64_t *bp, const int64_t *comm, int32_t *best_sizes, int64_t *n_enumerated);
int64_t orc_sched_alg2(int L, int H, const int64_t *bp, const int64_t *comm, int32_t *best_sizes, int64_t *best_cost, int32_t *omega,
                       int64_t omega_cap);
void orc_sched_enp(int L, int H, int32_t *sizes);
int64_t orc_iteration_timeline(int L, const int64_t *bp, const int64_t *comm, int n, const int32_t *layers, int64_t *exposed);
void orc_fill_bubbles(int L, int H, const int64_t *bp, const int64_t *comm, const int32_t *sizes, int32_t *extra);
int64_t orc_slot_offsets(int T, const int32_t *layer_of, const int64_t *numel, int n_set, const int32_t *set_layers, int64_t *dst_off,
                         int32_t *order, int32_t *n_order);
void orc_pack(int n, const float *const *src, const int64_t *numel, const int64_t *off, float *flat);
void orc_unpack(int n, float *const *dst, uint16_t *const *model, const int64_t *numel, const int64_t *off, const float *flat);
void orc_mean(int N, const float *const *x, int64_t n, float *out);
void orc_layer_stats(int N, const float *const *x, const float *mean, int64_t begin, int64_t end, double *gamma, double *msq);
void orc_sgdm(float *p, const float *g, float *buf, int64_t n, float lr, float mu);
void orc_adamw(float *p, const float *g32, const uint16_t *g16, float *m, float *v, uint16_t *model, int64_t n, float lr, float beta1,
               float beta2, float eps, float wd, int64_t step);
void orc_bf16_rne(const float *x, uint16_t *out, int64_t n);
void orc_bf16_widen(const uint16_t *x, float *out, int64_t n);
}

#define CHECK(cond)                                                                  \
    do {                                                                             \
        if (!(cond)) {                                                               \
            std::fprintf(stderr, "%s:%d: check failed: %s (last error: %s)\n", __FILE__, __LINE__, #cond, ddp::g_last.c_str()); \
            std::exit(1);                                                            \
        }                                                                            \
    } while (0)

static std::vector<int32_t> sizes_of(int H, const std::vector<int32_t> &sp) {
    std::vector<int32_t> s(H);
    for (int h = 0; h < H; ++h) s[h] = sp[h + 1] - sp[h];
    return s;
}

int main(int argc, char **argv) {
    const int rounds = argc > 1 ? std::atoi(argv[1]) : 400;
    std::mt19937_64 rng(2024);
    auto uni = [&](int64_t lo, int64_t hi) { return (int64_t)(lo + rng() % (uint64_t)(hi - lo + 1)); };
    int64_t n_sched = 0, n_elem = 0;

    for (int it = 0; it < rounds; ++it) {
        // ---- scheduler: OPT vs exhaustive search, ALG2 vs its recursive statement, bubbles, time model -------------
        const int L = (int)uni(1, it % 4 == 0 ? 11 : 6), H = (int)uni(1, it % 4 == 0 ? 5 : 3);
        std::vector<int64_t> bp(L), comm(L), fp(L);
        const int64_t scale = it % 7 == 0 ? (int64_t)1 << 40 : 30;  // large values exercise the overflow guards' neighbourhood
        for (int l = 0; l < L; ++l) {
            bp[l] = uni(0, scale);
            comm[l] = uni(0, 2 * scale);
            fp[l] = uni(0, scale);
        }
        std::vector<int32_t> slot(L), sp(H + 1), sl(L * H + 1), best(H), omega(4096 * H);
        int64_t cost = -1, n_enum = 0, best_cost = -1;
        for (int policy = DDP_SCHED_ENP; policy <= DDP_SCHED_ALG2; ++policy) {
            CHECK(ddp_schedule(policy, L, H, fp.data(), bp.data(), comm.data(), slot.data(), sp.data(), sl.data(), &cost) == DDP_OK);
            CHECK(sp[0] == 0 && sp[H] == (policy == DDP_SCHED_EVERY ? L * H : L));
            if (policy == DDP_SCHED_OPT) {
                const int64_t ref = orc_sched_brute(L, H, bp.data(), comm.data(), best.data(), &n_enum);
                CHECK(ref == cost && sizes_of(H, sp) == best);
            }
            if (policy == DDP_SCHED_ALG2) {
                const int64_t n = orc_sched_alg2(L, H, bp.data(), comm.data(), best.data(), &best_cost, omega.data(), 4096);
                int64_t n_lib = -1;
                CHECK(n <= 4096 && best_cost == cost && sizes_of(H, sp) == best);
                CHECK(ddp_schedule_alg2_solutions(L, H, bp.data(), comm.data(), &n_lib) == DDP_OK && n_lib == n);
            }
            if (policy == DDP_SCHED_ENP || policy == DDP_SCHED_FULL || policy == DDP_SCHED_OPT || policy == DDP_SCHED_ALG2) {
                const std::vector<int32_t> sz = sizes_of(H, sp);
                int64_t c2 = -1;
                CHECK(orc_sched_cost(L, H, bp.data(), comm.data(), sz.data()) == cost);
                CHECK(ddp_schedule_cost(L, H, bp.data(), comm.data(), sp.data(), sl.data(), &c2) == DDP_OK && c2 == cost);
                // Eq. (12): bubble filling, then Eq. (7) on the filled schedule
                std::vector<int32_t> fsp(H + 1), fsl(L * H + 1), extra(H), oextra(H);
                CHECK(ddp_schedule_fill_bubbles(L, H, bp.data(), comm.data(), sp.data(), sl.data(), fsp.data(), fsl.data(), extra.data()) == DDP_OK);
                orc_fill_bubbles(L, H, bp.data(), comm.data(), sz.data(), oextra.data());
                CHECK(extra == oextra);
                std::vector<int64_t> iter(H), exposed(H);
                int64_t period = 0, fp_sum = 0, sum = 0;
                for (int l = 0; l < L; ++l) fp_sum += fp[l];
                CHECK(ddp_schedule_time_model(L, H, fp.data(), bp.data(), comm.data(), fsp.data(), fsl.data(), iter.data(), exposed.data(), &period) == DDP_OK);
                for (int h = 0; h < H; ++h) {
                    int64_t ex = -1;
                    const int64_t t = orc_iteration_timeline(L, bp.data(), comm.data(), fsp[h + 1] - fsp[h], fsl.data() + fsp[h], &ex);
                    CHECK(iter[h] == t + fp_sum && exposed[h] == ex);
                    sum += iter[h];
                }
                CHECK(sum == period);
            }
            ++n_sched;
        }
        // argument errors must come back as codes
        CHECK(ddp_schedule(DDP_SCHED_OPT, 0, H, nullptr, bp.data(), comm.data(), slot.data(), sp.data(), sl.data(), nullptr) == DDP_EINVAL);
        CHECK(ddp_schedule(DDP_SCHED_OPT, L, H, nullptr, nullptr, comm.data(), slot.data(), sp.data(), sl.data(), nullptr) == DDP_EINVAL);
        CHECK(ddp_schedule(99, L, H, nullptr, bp.data(), comm.data(), slot.data(), sp.data(), sl.data(), nullptr) == DDP_EINVAL);
        std::vector<int64_t> neg = bp;
        neg[0] = -1;
        CHECK(ddp_schedule(DDP_SCHED_OPT, L, H, nullptr, neg.data(), comm.data(), slot.data(), sp.data(), sl.data(), nullptr) == DDP_EINVAL);
        std::vector<int64_t> huge(L, INT64_MAX / 2 + 1);  // backward + communication of one layer already pass int64
        CHECK(ddp_schedule(DDP_SCHED_OPT, L, H, nullptr, huge.data(), huge.data(), slot.data(), sp.data(), sl.data(), nullptr) == DDP_EINVAL);

        // ---- oracle, elementwise: ragged sizes, every buffer exactly as long as stated (ASan guards the ends) -----
        const int T = (int)uni(1, 6), Lw = (int)uni(1, T), N = (int)uni(1, 9);
        std::vector<int32_t> layer_of(T), set_layers;
        std::vector<int64_t> numel(T), off(T);
        for (int t = 0; t < T; ++t) {
            layer_of[t] = (int32_t)((int64_t)t * Lw / T);
            numel[t] = uni(1, 300);
        }
        for (int l = Lw - 1; l >= 0; --l)
            if (uni(0, 1)) set_layers.push_back(l);
        std::vector<int32_t> order(T);
        int32_t n_order = 0;
        const int64_t total = orc_slot_offsets(T, layer_of.data(), numel.data(), (int)set_layers.size(), set_layers.data(), off.data(), order.data(), &n_order);
        std::vector<std::vector<float>> tens(T);
        std::vector<std::vector<uint16_t>> model(T);
        for (int t = 0; t < T; ++t) {
            tens[t].resize(numel[t]);
            model[t].resize(numel[t]);
            for (auto &v : tens[t]) v = (float)uni(-1000, 1000) / 512.0f;
        }
        std::vector<const float *> src;
        std::vector<float *> dst;
        std::vector<uint16_t *> mdl;
        std::vector<int64_t> ne, of;
        for (int j = 0; j < n_order; ++j) {
            const int t = order[j];
            src.push_back(tens[t].data());
            dst.push_back(tens[t].data());
            mdl.push_back(model[t].data());
            ne.push_back(numel[t]);
            of.push_back(off[t]);
        }
        std::vector<float> flat(total), out(total);
        orc_pack(n_order, src.data(), ne.data(), of.data(), flat.data());
        std::vector<std::vector<float>> reps(N, std::vector<float>(total));
        std::vector<const float *> xs(N);
        for (int k = 0; k < N; ++k) {
            for (int64_t i = 0; i < total; ++i) reps[k][i] = flat[i] + (float)uni(-8, 8) / 1024.0f;
            xs[k] = reps[k].data();
        }
        orc_mean(N, xs.data(), total, out.data());
        double g = -1, m = -1;
        orc_layer_stats(N, xs.data(), out.data(), 0, total, &g, &m);
        CHECK(g >= 0 && m >= 0);
        orc_unpack(n_order, dst.data(), mdl.data(), ne.data(), of.data(), out.data());
        for (int t = 0; t < T; ++t) {
            const int64_t n = numel[t];
            std::vector<float> gr(n), s0(n, 0.0f), s1(n, 0.0f), wide(n);
            std::vector<uint16_t> g16(n);
            for (auto &v : gr) v = (float)uni(-100, 100) / 4096.0f;
            orc_bf16_rne(gr.data(), g16.data(), n);
            orc_bf16_widen(g16.data(), wide.data(), n);
            orc_sgdm(tens[t].data(), gr.data(), s0.data(), n, 0.01f, 0.9f);
            orc_adamw(tens[t].data(), nullptr, g16.data(), s0.data(), s1.data(), model[t].data(), n, 3e-4f, 0.9f, 0.95f, 1e-8f, 0.1f, 1 + it % 5);
            orc_adamw(tens[t].data(), wide.data(), nullptr, s0.data(), s1.data(), nullptr, n, 3e-4f, 0.9f, 0.95f, 1e-8f, 0.1f, 2 + it % 5);
            n_elem += 3 * n;
        }
    }
    // the bounded search of Algorithm 2 on an instance whose solution set explodes
    {
        const int L = 128, H = 64;
        std::vector<int64_t> bp(L, 1), comm(L);
        for (int l = 0; l < L; ++l) comm[l] = l % 2 ? 1000000 : 0;
        std::vector<int32_t> slot(L), sp(H + 1), sl(L);
        CHECK(ddp_schedule(DDP_SCHED_ALG2, L, H, nullptr, bp.data(), comm.data(), slot.data(), sp.data(), sl.data(), nullptr) == DDP_ESCHED);
        CHECK(ddp_schedule(DDP_SCHED_OPT, L, H, nullptr, bp.data(), comm.data(), slot.data(), sp.data(), sl.data(), nullptr) == DDP_OK);
    }
    std::printf("sanitizer sweep ok: %lld schedules, %lld optimizer elements\n", (long long)n_sched, (long long)n_elem);
    return 0;
}
