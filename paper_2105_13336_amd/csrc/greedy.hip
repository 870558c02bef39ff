// Greedy plan generation (swap phase of the paper's Alg. 3 with the placement of
// Alg. 2): a host loop around the evaluation and scoring kernels.  Per
// iteration the device analyses the current plan (B = 1) and scores every
// tensor; the host orders the candidates, places the two transfers of each on
// the exclusive host link, and appends the first one that still covers the peak.
#include "common.h"

#include <algorithm>

namespace tensile {
namespace {

// Link timeline at step resolution: busy[t] != 0 when a transfer occupies step t.
struct Link {
    const std::vector<int64_t> &C;
    std::vector<uint8_t> busy;
    explicit Link(const std::vector<int64_t> &c, int32_t T) : C(c), busy(static_cast<size_t>(T), 0) {}

    // first step e >= u with C[e+1] - C[u] >= x (C non-decreasing); may be past the end
    int32_t end_of_transfer_from(int32_t u, int64_t x) const {
        const int64_t target = C[u] + x;
        return static_cast<int32_t>(std::lower_bound(C.begin() + u + 1, C.end(), target) - C.begin()) - 1;
    }
    // last step c <= v with C[v+1] - C[c] >= x; may be negative
    int32_t start_of_transfer_to(int32_t v, int64_t x) const {
        const int64_t target = C[v + 1] - x;
        return static_cast<int32_t>(std::upper_bound(C.begin(), C.begin() + v + 1, target) - C.begin()) - 1;
    }

    // Earliest run of free steps [a..e] inside [lo, hi] whose duration covers x.
    bool place_earliest(int32_t lo, int32_t hi, int64_t x, int32_t *a, int32_t *e) const {
        int32_t u = lo;
        while (u <= hi) {
            while (u <= hi && busy[u]) ++u;
            if (u > hi) break;
            int32_t v = u;                       // maximal free run [u..v]
            while (v + 1 <= hi && !busy[v + 1]) ++v;
            const int32_t end = end_of_transfer_from(u, x);
            if (end <= v) {
                *a = u;
                *e = end;
                return true;
            }
            u = v + 2;                           // v+1 is busy (or past hi)
        }
        return false;
    }
    // Latest run of free steps [c..d] inside [lo, hi] whose duration covers x.
    bool place_latest(int32_t lo, int32_t hi, int64_t x, int32_t *c, int32_t *d) const {
        int32_t v = hi;
        while (v >= lo) {
            while (v >= lo && busy[v]) --v;
            if (v < lo) break;
            int32_t u = v;                       // maximal free run [u..v]
            while (u - 1 >= lo && !busy[u - 1]) --u;
            const int32_t start = start_of_transfer_to(v, x);
            if (start >= u) {
                *c = start;
                *d = v;
                return true;
            }
            v = u - 2;
        }
        return false;
    }
    void occupy(int32_t from, int32_t to) { std::fill(busy.begin() + from, busy.begin() + to + 1, 1); }
};

struct Cand {
    int32_t tensor;
    int64_t score, size;
};

}  // namespace
}  // namespace tensile

using namespace tensile;

extern "C" int tensile_greedy_plan(const tensile_tas *tas, int64_t budget_bytes, const tensile_greedy_opts *opts,
                                   int32_t capacity, int32_t n_initial, int32_t *iv_tensor, int32_t *iv_out,
                                   int32_t *iv_in, uint8_t *iv_kind, int32_t *n_intervals, int64_t *peak_trace,
                                   int64_t *final_peak) {
    if (!tas || !n_intervals || !final_peak) { set_error("greedy_plan: NULL argument"); return TENSILE_E_INVAL; }
    if (capacity < 0 || n_initial < 0 || n_initial > capacity) {
        set_error("greedy_plan: need 0 <= n_initial <= capacity");
        return TENSILE_E_INVAL;
    }
    if (capacity > 0 && (!iv_tensor || !iv_out || !iv_in || !iv_kind)) {
        set_error("greedy_plan: interval arrays are NULL");
        return TENSILE_E_INVAL;
    }
    const tensile_greedy_opts defaults{0, 100, 0, nullptr, 1};
    const tensile_greedy_opts &opt = opts ? *opts : defaults;
    const int32_t T = tas->T, N = tas->N;
    const int32_t max_new = opt.max_iters > 0 ? opt.max_iters : INT32_MAX;

    try {
        // device state: the growing plan (B = 1) and one row of every output
        DevBuf<int64_t> d_offs, d_res, d_peak, d_min, d_score;
        DevBuf<int32_t> d_t, d_o, d_r, d_arg, d_wo, d_wi;
        TS_HIP(d_offs.reserve(2));
        TS_HIP(d_t.reserve(capacity)); TS_HIP(d_o.reserve(capacity)); TS_HIP(d_r.reserve(capacity));
        TS_HIP(d_res.reserve(T)); TS_HIP(d_peak.reserve(1)); TS_HIP(d_min.reserve(1)); TS_HIP(d_arg.reserve(1));
        TS_HIP(d_score.reserve(N)); TS_HIP(d_wo.reserve(N)); TS_HIP(d_wi.reserve(N));
        if (n_initial > 0) {
            TS_HIP(hipMemcpy(d_t.p, iv_tensor, n_initial * 4, hipMemcpyHostToDevice));
            TS_HIP(hipMemcpy(d_o.p, iv_out, n_initial * 4, hipMemcpyHostToDevice));
            TS_HIP(hipMemcpy(d_r.p, iv_in, n_initial * 4, hipMemcpyHostToDevice));
        }
        std::vector<int64_t> score(N);
        std::vector<int32_t> wo(N), wi(N);
        std::vector<Cand> cand;
        cand.reserve(N);
        std::vector<int64_t> hist;
        std::vector<int64_t> swapped(static_cast<size_t>(tas->J), 0);
        int64_t swapped_total = 0;
        Link link(tas->h_C, T);

        int32_t n = n_initial;
        int64_t P = 0;
        for (;;) {
            const int32_t it = n - n_initial;
            const int64_t h_offs[2] = {0, n};
            TS_HIP(hipMemcpy(d_offs.p, h_offs, sizeof h_offs, hipMemcpyHostToDevice));
            tensile_plans pl{1, n, d_offs.p, d_t.p, d_o.p, d_r.p, nullptr};
            int rc = tensile_eval_plans(tas, &pl, d_res.p, d_peak.p, d_arg.p, d_min.p, nullptr);
            if (rc != TENSILE_OK) return rc;
            int32_t tstar = 0;
            TS_HIP(hipMemcpy(&P, d_peak.p, 8, hipMemcpyDeviceToHost));
            TS_HIP(hipMemcpy(&tstar, d_arg.p, 4, hipMemcpyDeviceToHost));
            hist.push_back(P);
            if (peak_trace) peak_trace[it] = P;
            if (it >= max_new || n >= capacity) break;
            if (opt.stop_at_budget && P <= budget_bytes) break;
            if (it > opt.min_iters && it >= 3 && (hist[it - 3] - P) * 10000 < 5 * hist[it - 3]) break;
            if (N == 0) break;

            rc = tensile_score_candidates(tas, &pl, d_res.p, d_peak.p, d_arg.p, d_score.p, d_wo.p, d_wi.p, nullptr);
            if (rc != TENSILE_OK) return rc;
            TS_HIP(hipMemcpy(score.data(), d_score.p, static_cast<size_t>(N) * 8, hipMemcpyDeviceToHost));
            TS_HIP(hipMemcpy(wo.data(), d_wo.p, static_cast<size_t>(N) * 4, hipMemcpyDeviceToHost));
            TS_HIP(hipMemcpy(wi.data(), d_wi.p, static_cast<size_t>(N) * 4, hipMemcpyDeviceToHost));

            cand.clear();
            const int64_t tot = std::max<int64_t>(1, swapped_total);
            for (int32_t i = 0; i < N; ++i) {
                if (wo[i] < 0) continue;
                if (opt.msr_num) {
                    const int32_t j = tas->h_job[i];
                    if (!(swapped[j] * opt.msr_den <= opt.msr_num[j] * tot)) continue;
                }
                cand.push_back(Cand{i, score[i], tas->h_size[i]});
            }
            std::sort(cand.begin(), cand.end(), [](const Cand &a, const Cand &b) {
                if (a.score != b.score) return a.score > b.score;
                if (a.size != b.size) return a.size > b.size;
                return a.tensor < b.tensor;
            });

            bool accepted = false;
            for (const Cand &c : cand) {
                const int32_t i = c.tensor;
                const int32_t q = wi[i];                         // p_{g+1}
                // p_g: the touch point just before q in the tensor's list
                const int32_t *tb = tas->h_touch.data() + tas->h_touch_off[i];
                const int32_t *te = tas->h_touch.data() + tas->h_touch_off[i + 1];
                const int32_t p = *(std::lower_bound(tb, te, q) - 1);
                const int64_t x = tas->h_x[i];
                int32_t o_placed = p, r_placed = q, a = -1, e = -1, cs = -1, d = -1;
                if (x != 0) {
                    if (!link.place_earliest(p + 1, q - 1, x, &a, &e)) continue;
                    if (!link.place_latest(e + 1, q - 1, x, &cs, &d)) continue;
                    o_placed = e;
                    r_placed = d + 1;
                }
                if (!(o_placed < tstar && tstar < r_placed)) continue;
                if (x != 0) {
                    link.occupy(a, e);
                    link.occupy(cs, d);
                }
                iv_tensor[n] = i;
                iv_out[n] = o_placed;
                iv_in[n] = r_placed;
                iv_kind[n] = 0;
                const int32_t triple[3] = {i, o_placed, r_placed};
                TS_HIP(hipMemcpy(d_t.p + n, &triple[0], 4, hipMemcpyHostToDevice));
                TS_HIP(hipMemcpy(d_o.p + n, &triple[1], 4, hipMemcpyHostToDevice));
                TS_HIP(hipMemcpy(d_r.p + n, &triple[2], 4, hipMemcpyHostToDevice));
                ++swapped[tas->h_job[i]];
                ++swapped_total;
                ++n;
                accepted = true;
                break;
            }
            if (!accepted) break;
        }
        *n_intervals = n;
        *final_peak = P;
    } catch (const std::bad_alloc &) {
        set_error("greedy_plan: out of host memory");
        return TENSILE_E_NOMEM;
    }
    return TENSILE_OK;
}
