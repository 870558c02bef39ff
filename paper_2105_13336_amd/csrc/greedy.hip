// Greedy plan generation (swap phase of the paper's Alg. 3 with the placement of
// Alg. 2): a host loop around the evaluation and scoring kernels.  Per
// iteration the device analyses the current plan (B = 1) and scores every
// tensor; the host orders the candidates, places the two transfers of each on
// the exclusive host link, and appends the first one that still covers the peak.
#include "common.h"

#include <algorithm>
#include <chrono>

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
    int32_t wo, wi;
};

typedef ScoreHeader Header;
typedef ScoreCand CandOut;

__global__ void peak_only_kernel(const int64_t *peak, const int32_t *arg, Header *hdr) { *hdr = Header{*peak, *arg, 0}; }

// Pinned host memory that frees itself (after everything the device still does with it).
struct PinnedBuf {
    void *p = nullptr;
    ~PinnedBuf() {
        if (!p) return;
        (void)hipDeviceSynchronize();
        (void)hipHostFree(p);
    }
    hipError_t reserve(size_t bytes) { return hipHostMalloc(&p, bytes, hipHostMallocDefault); }
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
    if (opt.msr_num && opt.msr_den <= 0) {
        set_error("greedy_plan: msr_den must be positive when msr_num is given");
        return TENSILE_E_INVAL;
    }
    if (opt.msr_num) {
        for (int32_t j = 0; j < tas->J; ++j)
            if (opt.msr_num[j] < 0) { set_error("greedy_plan: msr_num[%d] is negative", j); return TENSILE_E_INVAL; }
    }
    const int32_t T = tas->T, N = tas->N;
    const int32_t max_new = opt.max_iters > 0 ? opt.max_iters : INT32_MAX;

    try {
        // device state: the growing plan (B = 1), one row of every output, the compacted candidates
        DevBuf<int64_t> d_offs, d_res, d_peak, d_min;
        DevBuf<int32_t> d_t, d_o, d_r, d_arg;
        DevBuf<Header> d_hdr;           // the header of the last analysis, which scores nothing
        TS_HIP(d_offs.reserve(2));
        TS_HIP(d_t.reserve(capacity)); TS_HIP(d_o.reserve(capacity)); TS_HIP(d_r.reserve(capacity));
        TS_HIP(d_res.reserve(T)); TS_HIP(d_peak.reserve(1)); TS_HIP(d_min.reserve(1)); TS_HIP(d_arg.reserve(1));
        static_assert(sizeof(Header) == 16 && sizeof(CandOut) == 24, "layout of the iteration record");
        const size_t rec_bytes = sizeof(Header) + static_cast<size_t>(N) * sizeof(CandOut);
        TS_HIP(d_hdr.reserve(1));
        // The iteration's record lives in pinned host memory and the scoring kernel writes it there itself,
        // then stores the iteration's number to a word next to it: the host waits for that word instead of
        // the stream (no copy to enqueue, no wake-up through the driver).
        PinnedBuf h_rec, h_ready;
        TS_HIP(h_rec.reserve(rec_bytes));
        TS_HIP(h_ready.reserve(64));
        const Header *hdr = static_cast<const Header *>(h_rec.p);
        const CandOut *h_cands = reinterpret_cast<const CandOut *>(hdr + 1);
        volatile unsigned long long *ready = static_cast<volatile unsigned long long *>(h_ready.p);
        *ready = 0;
        void *rec_dev = nullptr, *ready_dev = nullptr;   // the same memory as the kernels address it
        TS_HIP(hipHostGetDevicePointer(&rec_dev, h_rec.p, 0));
        TS_HIP(hipHostGetDevicePointer(&ready_dev, h_ready.p, 0));
        unsigned long long ready_seq = 0;
        if (n_initial > 0) {
            TS_HIP(hipMemcpy(d_t.p, iv_tensor, n_initial * 4, hipMemcpyHostToDevice));
            TS_HIP(hipMemcpy(d_o.p, iv_out, n_initial * 4, hipMemcpyHostToDevice));
            TS_HIP(hipMemcpy(d_r.p, iv_in, n_initial * 4, hipMemcpyHostToDevice));
        }
        {
            const int64_t h_offs[2] = {0, n_initial};
            TS_HIP(hipMemcpy(d_offs.p, h_offs, sizeof h_offs, hipMemcpyHostToDevice));
        }
        std::vector<Cand> cand;
        cand.reserve(N);
        std::vector<int64_t> hist;
        std::vector<int64_t> swapped(static_cast<size_t>(tas->J), 0);
        int64_t swapped_total = 0;
        Link link(tas->h_C, T);

        int32_t n = n_initial;
        int64_t P = 0;
        // Scores of the current plan (swap or recomputation candidates), compacted and fetched:
        // header plus the first candidates in one copy, the rest only when there are more.
        tensile_plans pl{1, 0, d_offs.p, d_t.p, d_o.p, d_r.p, nullptr};
        auto score_and_fetch = [&](bool recompute_scores) -> int {
            // the scoring kernel writes the record itself: {peak, peak step, count}, then one entry per tensor with a window
            int rc = recompute_scores ? ensure_recompute_index(tas) : TENSILE_OK;
            if (rc != TENSILE_OK) return rc;
            const unsigned long long want = ++ready_seq;
            {
                WorkspaceLock ws = acquire_workspace(tas, nullptr);
                rc = launch_score(tas, *ws, recompute_scores ? tas->recompute_index : tas->index, recompute_scores, &pl, d_res.p,
                                  d_peak.p, d_arg.p, nullptr, nullptr, nullptr, static_cast<Header *>(rec_dev),
                                  reinterpret_cast<CandOut *>(static_cast<Header *>(rec_dev) + 1),
                                  static_cast<unsigned long long *>(ready_dev), want);
            }
            if (rc != TENSILE_OK) return rc;
            // wait for the word; should it not arrive (a failed launch shows up in the stream), ask the stream
            const auto t_start = std::chrono::steady_clock::now();
            for (unsigned spins = 0; __atomic_load_n(const_cast<unsigned long long *>(ready), __ATOMIC_ACQUIRE) != want; ++spins) {
                if ((spins & 0xfff) == 0xfff && std::chrono::steady_clock::now() - t_start > std::chrono::seconds(2)) {
                    TS_HIP(hipStreamSynchronize(nullptr));
                    if (__atomic_load_n(const_cast<unsigned long long *>(ready), __ATOMIC_ACQUIRE) != want) {
                        set_error("greedy_plan: the scoring kernel finished without its record");
                        return TENSILE_E_HIP;
                    }
                    break;
                }
            }
            return TENSILE_OK;
        };
        // (the device copy of the plan receives the interval from the next iteration's update kernel)
        auto append = [&](int32_t i, int32_t o, int32_t r, uint8_t kind) -> int {
            iv_tensor[n] = i;
            iv_out[n] = o;
            iv_in[n] = r;
            iv_kind[n] = kind;
            ++n;
            return TENSILE_OK;
        };

        // One swap iteration on the candidates just fetched (Alg. 2's placement); false when none is accepted.
        int swap_error = TENSILE_OK;
        int32_t tstar_now = 0;
        auto try_swap = [&]() -> bool {
            const int32_t tstar = tstar_now;
            const int64_t tot = std::max<int64_t>(1, swapped_total);
            auto allowed = [&](const CandOut &c) {      // the job's swapping rate limit (section IV-C)
                if (!opt.msr_num) return true;
                const int32_t j = tas->h_job[c.tensor];
                return swapped[j] * opt.msr_den <= opt.msr_num[j] * tot;
            };
            // candidates are tried in the order (score desc, size desc, tensor asc)
            auto later = [](const Cand &a, const Cand &b) {      // a comes after b
                if (a.score != b.score) return a.score < b.score;
                if (a.size != b.size) return a.size < b.size;
                return a.tensor > b.tensor;
            };
            // 1 accepted, 0 cannot be placed around the peak, -1 error
            auto place = [&](const Cand &c) -> int {
                const int32_t i = c.tensor;
                const int32_t q = c.wi;                          // p_{g+1}
                // p_g: the touch point just before q in the tensor's list
                const int32_t *tb = tas->h_touch.data() + tas->h_touch_off[i];
                const int32_t *te = tas->h_touch.data() + tas->h_touch_off[i + 1];
                const int32_t p = *(std::lower_bound(tb, te, q) - 1);
                const int64_t x = tas->h_x[i];
                int32_t o_placed = p, r_placed = q, a = -1, e = -1, cs = -1, d = -1;
                if (x != 0) {
                    if (!link.place_earliest(p + 1, q - 1, x, &a, &e)) return 0;
                    if (!link.place_latest(e + 1, q - 1, x, &cs, &d)) return 0;
                    o_placed = e;
                    r_placed = d + 1;
                }
                if (!(o_placed < tstar && tstar < r_placed)) return 0;
                if (x != 0) {
                    link.occupy(a, e);
                    link.occupy(cs, d);
                }
                const int rc_append = append(i, o_placed, r_placed, 0);
                if (rc_append != TENSILE_OK) { swap_error = rc_append; return -1; }
                ++swapped[tas->h_job[i]];
                ++swapped_total;
                return 1;
            };
            // usually the very first candidate is accepted: find it by one pass over the record ...
            bool have = false;
            Cand first{};
            for (int32_t k = 0; k < hdr->count; ++k) {
                const CandOut &c = h_cands[k];
                if (!allowed(c)) continue;
                const Cand cur{c.tensor, c.score, tas->h_size[c.tensor], c.wo, c.wi};
                if (!have || later(first, cur)) {
                    first = cur;
                    have = true;
                }
            }
            if (!have) return false;
            int got = place(first);
            if (got != 0) return got > 0;
            // ... and only when it cannot be placed order the rest (a heap is popped instead of sorting them all)
            cand.clear();
            for (int32_t k = 0; k < hdr->count; ++k) {
                const CandOut &c = h_cands[k];
                if (allowed(c) && c.tensor != first.tensor) cand.push_back(Cand{c.tensor, c.score, tas->h_size[c.tensor], c.wo, c.wi});
            }
            std::make_heap(cand.begin(), cand.end(), later);
            for (auto end = cand.end(); end != cand.begin(); --end) {
                std::pop_heap(cand.begin(), end, later);
                got = place(*(end - 1));
                if (got != 0) return got > 0;
            }
            return false;
        };

        bool swap_phase = true;
        for (;;) {
            // One round trip per iteration: evaluate, score and compact on the device (the scores
            // of the last iteration are computed in vain), then fetch.
            const int32_t it = n - n_initial;
            const bool last = it >= max_new || n >= capacity || N == 0;
            pl.n_intervals = n;
            // the first footprint comes from the whole plan; afterwards exactly one interval has joined
            // since the last analysis and only its window of the row is brought up to date
            int rc;
            if (it == 0) {
                rc = tensile_eval_plans(tas, &pl, d_res.p, d_peak.p, d_arg.p, d_min.p, nullptr);
            } else {
                const ApplyAppend last_one{iv_tensor[n - 1], iv_out[n - 1], iv_in[n - 1], n - 1, d_t.p, d_o.p, d_r.p, d_offs.p};
                WorkspaceLock ws = acquire_workspace(tas, nullptr);
                rc = launch_apply(tas, *ws, 1, nullptr, nullptr, nullptr, d_res.p, d_peak.p, d_arg.p, d_min.p, &last_one);
            }
            if (rc != TENSILE_OK) return rc;
            if (last) {
                hipLaunchKernelGGL(peak_only_kernel, dim3(1), dim3(1), 0, nullptr, d_peak.p, d_arg.p, d_hdr.p);
                TS_HIP(hipGetLastError());
                TS_HIP(hipMemcpyAsync(h_rec.p, d_hdr.p, sizeof(Header), hipMemcpyDeviceToHost, nullptr));
                TS_HIP(hipStreamSynchronize(nullptr));
            } else {
                rc = score_and_fetch(!swap_phase);
                if (rc != TENSILE_OK) return rc;
            }
            P = hdr->P;
            tstar_now = hdr->tstar;
            hist.push_back(P);
            if (peak_trace) peak_trace[it] = P;
            if (last) break;
            if (opt.stop_at_budget && P <= budget_bytes) break;
            if (it > opt.min_iters && it >= 3 && (hist[it - 3] - P) * 10000 < 5 * hist[it - 3]) break;

            const bool swapped_one = swap_phase && try_swap();
            if (swap_error != TENSILE_OK) return swap_error;
            if (!swapped_one) {
                // Recomputation branch of Alg. 3: swapping is over for good; while the peak does not fit,
                // release the never-released tensor with the largest MSPS over its whole gap.
                if (swap_phase) {
                    swap_phase = false;
                    if (!(opt.recompute && P > budget_bytes)) break;
                    rc = score_and_fetch(true);        // same plan, same footprint: only the scores differ
                    if (rc != TENSILE_OK) return rc;
                } else if (!(P > budget_bytes)) {
                    break;
                }
                const CandOut *best = nullptr;
                int64_t best_time = 1;
                for (int32_t k = 0; k < hdr->count; ++k) {
                    const CandOut &c = h_cands[k];
                    if (c.score <= 0) continue;
                    const int32_t born = tas->h_touch[tas->h_touch_off[c.tensor]];
                    const int64_t time = tas->timed ? tas->h_C[born + 1] - tas->h_C[born] : 1;
                    bool better = best == nullptr;
                    if (!better) {
                        const __int128 l = static_cast<__int128>(c.score) * best_time, r = static_cast<__int128>(best->score) * time;
                        if (l != r) better = l > r;
                        else if (c.score != best->score) better = c.score > best->score;
                        else if (tas->h_size[c.tensor] != tas->h_size[best->tensor]) better = tas->h_size[c.tensor] > tas->h_size[best->tensor];
                        else better = c.tensor < best->tensor;
                    }
                    if (better) {
                        best = &c;
                        best_time = time;
                    }
                }
                if (!best) break;
                rc = append(best->tensor, best->wo, best->wi, 1);
                if (rc != TENSILE_OK) return rc;
            }
        }
        TS_HIP(hipDeviceSynchronize());
        *n_intervals = n;
        *final_peak = P;
    } catch (const std::bad_alloc &) {
        set_error("greedy_plan: out of host memory");
        return TENSILE_E_NOMEM;
    }
    return TENSILE_OK;
}
