// Greedy plan generation (swap phase of the paper's Alg. 3 with the placement of
// Alg. 2, then its recomputation branch): a host loop with ONE kernel launch per
// iteration.  The device keeps the plan's footprint row and the maxima of its
// 256-step blocks from iteration to iteration; an iteration takes the interval
// the host has just chosen out of the row (only its window is written), patches
// the block maxima the window touches, finds the peak and its earliest step from
// them, and scores every tensor (score.hip: greedy_step_kernel).  The host
// orders the candidates, places the two transfers of each on the exclusive host
// link, and appends the first one that still covers the peak.
#include "common.h"

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <memory>

namespace tensile {
namespace {

// The host link's timeline: the transfers placed so far as disjoint runs of steps [from, to], sorted.  (The
// placement rules speak of maximal runs of FREE steps; walking the busy runs between them costs a step per
// transfer in the way instead of a step per step of the gap, which matters once the link is crowded and most
// candidates no longer fit.)
struct Link {
    const std::vector<int64_t> &C;
    struct Run { int32_t from, to; };
    std::vector<Run> busy;
    explicit Link(const std::vector<int64_t> &c, int32_t) : C(c) {}

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
    // the first busy run that ends at or after step u
    std::vector<Run>::const_iterator first_ending_from(int32_t u) const {
        return std::lower_bound(busy.begin(), busy.end(), u, [](const Run &r, int32_t step) { return r.to < step; });
    }

    // Earliest run of free steps [a..e] inside [lo, hi] whose duration covers x: the maximal free runs are tried
    // from the left, each from its first step.
    bool place_earliest(int32_t lo, int32_t hi, int64_t x, int32_t *a, int32_t *e) const {
        int32_t u = lo;
        auto it = first_ending_from(u);
        while (u <= hi) {
            if (it != busy.end() && it->from <= u) {      // u is busy: on to the step after this run
                u = it->to + 1;
                ++it;
                continue;
            }
            const int32_t v = (it != busy.end() && it->from - 1 < hi) ? it->from - 1 : hi;   // maximal free run [u..v]
            const int32_t end = end_of_transfer_from(u, x);
            if (end <= v) {
                *a = u;
                *e = end;
                return true;
            }
            u = v + 1;                                    // busy, or past hi
        }
        return false;
    }
    // Latest run of free steps [c..d] inside [lo, hi] whose duration covers x: the maximal free runs are tried
    // from the right, each up to its last step.
    bool place_latest(int32_t lo, int32_t hi, int64_t x, int32_t *c, int32_t *d) const {
        int32_t v = hi;
        auto it = first_ending_from(v);                   // kept as: the first run that ends at or after v
        while (v >= lo) {
            if (it != busy.end() && it->from <= v) {      // v is busy: on to the step before this run
                v = it->from - 1;
                if (it != busy.begin() && (it - 1)->to >= v) --it;   // (a run that ends right there)
                continue;
            }
            const bool any_before = it != busy.begin();
            const int32_t u = (any_before && (it - 1)->to + 1 > lo) ? (it - 1)->to + 1 : lo;   // maximal free run [u..v]
            const int32_t start = start_of_transfer_to(v, x);
            if (start >= u) {
                *c = start;
                *d = v;
                return true;
            }
            if (!any_before) break;
            --it;                                         // the run that ends at u - 1 (or before lo: the loop ends)
            v = u - 1;
        }
        return false;
    }
    void occupy(int32_t from, int32_t to) {
        auto at = std::lower_bound(busy.begin(), busy.end(), from, [](const Run &r, int32_t step) { return r.from < step; });
        busy.insert(at, Run{from, to});
    }
};

struct Cand {
    int32_t tensor;
    int64_t score, size;
    int32_t wo, wi, gap;
};

typedef ScoreHeader Header;
typedef ScoreCand CandOut;

#ifdef TENSILE_GREEDY_PROF
double g_prof_launch = 0, g_prof_wait = 0;
#endif

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

// Everything a run of the planner allocates: the growing plan (B = 1), its row and the tables the iterations
// keep up to date, the record the device writes for the host.  Allocating it (pinned host memory above all)
// costs more than a dozen iterations, so a finished run leaves it with the handle and the next run takes it.
struct GreedyBuffers {
    int32_t capacity = -1;          // intervals the plan arrays hold
    DevBuf<int64_t> d_offs, d_res, d_peak, d_min, d_blk;
    DevBuf<int32_t> d_t, d_o, d_r, d_arg, d_blk_arg;
    DevBuf<uint8_t> d_gap_taken, d_tensor_taken;
    PinnedBuf h_rec, h_ready;
    void *rec_dev = nullptr, *ready_dev = nullptr;   // the pinned memory as the kernels address it
    int allocate(const tensile_tas *tas, int32_t cap) {
        const size_t T = static_cast<size_t>(tas->T), N = static_cast<size_t>(tas->N), n_blk = (T + kScoreMini - 1) / kScoreMini;
        TS_HIP(d_offs.reserve(2));
        TS_HIP(d_t.reserve(cap)); TS_HIP(d_o.reserve(cap)); TS_HIP(d_r.reserve(cap));
        TS_HIP(d_res.reserve(T)); TS_HIP(d_peak.reserve(1)); TS_HIP(d_min.reserve(1)); TS_HIP(d_arg.reserve(1));
        TS_HIP(d_blk.reserve(n_blk)); TS_HIP(d_blk_arg.reserve(n_blk));
        TS_HIP(d_gap_taken.reserve(static_cast<size_t>(tas->G))); TS_HIP(d_tensor_taken.reserve(N));
        static_assert(sizeof(ScoreHeader) == 16 && sizeof(ScoreCand) == 24, "layout of the iteration record");
        TS_HIP(h_rec.reserve(sizeof(ScoreHeader) + N * sizeof(ScoreCand)));
        TS_HIP(h_ready.reserve(64));
        TS_HIP(hipHostGetDevicePointer(&rec_dev, h_rec.p, 0));
        TS_HIP(hipHostGetDevicePointer(&ready_dev, h_ready.p, 0));
        capacity = cap;
        return TENSILE_OK;
    }
};

void drop_greedy_cache(const tensile_tas *tas) {
    std::lock_guard<std::mutex> g(tas->greedy_mu);
    delete tas->greedy_cache;
    tas->greedy_cache = nullptr;
}

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
        // the buffers: the last run's, if this handle has them and they are large enough, else new ones
        std::unique_ptr<GreedyBuffers> bufs;
        {
            std::lock_guard<std::mutex> g(tas->greedy_mu);
            if (tas->greedy_cache && tas->greedy_cache->capacity >= capacity) {
                bufs.reset(tas->greedy_cache);
                tas->greedy_cache = nullptr;
            }
        }
        if (!bufs) {
            bufs.reset(new GreedyBuffers());
            const int rc_alloc = bufs->allocate(tas, capacity);
            if (rc_alloc != TENSILE_OK) return rc_alloc;
        }
        struct Return {     // (on every way out: the run has synchronised or failed; a failed run's buffers are dropped)
            const tensile_tas *tas;
            std::unique_ptr<GreedyBuffers> &bufs;
            bool ok = false;
            ~Return() {
                if (!ok || !bufs) return;
                std::lock_guard<std::mutex> g(tas->greedy_mu);
                if (!tas->greedy_cache || tas->greedy_cache->capacity < bufs->capacity) {
                    delete tas->greedy_cache;
                    tas->greedy_cache = bufs.release();
                }
            }
        } give_back{tas, bufs};
        DevBuf<int64_t> &d_offs = bufs->d_offs, &d_res = bufs->d_res, &d_peak = bufs->d_peak, &d_min = bufs->d_min;
        DevBuf<int32_t> &d_t = bufs->d_t, &d_o = bufs->d_o, &d_r = bufs->d_r, &d_arg = bufs->d_arg;
        const GreedyTables tables{bufs->d_blk.p, bufs->d_blk_arg.p, bufs->d_gap_taken.p, bufs->d_tensor_taken.p};
        // The iteration's record lives in pinned host memory and the kernel writes it there itself, then stores
        // the iteration's number to a word next to it: the host waits for that word instead of the stream (no copy
        // to enqueue, no wake-up through the driver).
        const Header *hdr = static_cast<const Header *>(bufs->h_rec.p);
        const CandOut *h_cands = reinterpret_cast<const CandOut *>(hdr + 1);
        volatile unsigned long long *ready = static_cast<volatile unsigned long long *>(bufs->h_ready.p);
        *ready = 0;
        void *rec_dev = bufs->rec_dev, *ready_dev = bufs->ready_dev;
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
        {   // which gaps and tensors the plan to extend has dealt with already (the kernel adds the new intervals' flags)
            std::vector<uint8_t> gap_taken(static_cast<size_t>(tas->G) + 1, 0), tensor_taken(static_cast<size_t>(N) + 1, 0);
            for (int32_t k = 0; k < n_initial; ++k) {
                const int32_t i = iv_tensor[k], o = iv_out[k], r = iv_in[k];
                if (i < 0 || i >= N || o < 0 || r > T || r <= o) continue;      // cannot be applied: counts for nothing
                tensor_taken[i] = 1;
                // the gap (p, q) of the tensor with p <= o and r <= q, if it is one of those of length >= 2
                const int32_t *tb = tas->h_touch.data() + tas->h_touch_off[i], *te = tas->h_touch.data() + tas->h_touch_off[i + 1];
                const int32_t *after = std::upper_bound(tb, te, o);              // first touch point > o
                if (after == tb || after == te || r > *after) continue;
                const int32_t p = *(after - 1);
                const int32_t *g0 = tas->h_gp.data() + tas->h_gap_first[i], *g1 = tas->h_gp.data() + tas->h_gap_first[i + 1];
                const int32_t *g = std::lower_bound(g0, g1, p);
                if (g != g1 && *g == p) gap_taken[g - tas->h_gp.data()] = 1;
            }
            if (tas->G > 0) TS_HIP(hipMemcpy(tables.gap_taken, gap_taken.data(), static_cast<size_t>(tas->G), hipMemcpyHostToDevice));
            if (N > 0) TS_HIP(hipMemcpy(tables.tensor_taken, tensor_taken.data(), static_cast<size_t>(N), hipMemcpyHostToDevice));
        }
        std::vector<Cand> cand;
        cand.reserve(N);
        std::vector<int64_t> hist;
        std::vector<int64_t> swapped(static_cast<size_t>(tas->J), 0);
        int64_t swapped_total = 0;
        Link link(tas->h_C, T);
        // per gap, the window its swap got at the last attempt to place it: last resident step and step the bytes
        // are back (see try_swap); the true ones can only have moved towards each other since
        std::vector<int32_t> out_from(static_cast<size_t>(tas->G) + 1, -1), in_until(static_cast<size_t>(tas->G) + 1, INT32_MAX);

        int32_t n = n_initial;
        int64_t P = 0;
        // Scores of the current plan (swap or recomputation candidates), compacted and fetched:
        // header plus the first candidates in one copy, the rest only when there are more.
        tensile_plans pl{1, 0, d_offs.p, d_t.p, d_o.p, d_r.p, nullptr};
#ifdef TENSILE_GREEDY_PROF      // where the host's time goes, for tuning: printed when the run ends
        double prof_launch = 0, prof_wait = 0, prof_first = 0, prof_rest = 0, prof_recompute = 0;
        long prof_fallbacks = 0, prof_tried = 0;
        auto prof_now = [] { return std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now().time_since_epoch()).count(); };
#endif
        // One launch: `fresh` (or nothing) joins the plan on the device, peak and peak step are found, and - unless
        // this is the last analysis - the swap or recomputation candidates are scored.  The kernel writes the record
        // {peak, peak step, count}, then one entry per tensor with a window, and last the word the host waits for.
        auto analyse = [&](bool recompute_scores, const GreedyNew *fresh, bool rebuild, bool do_score) -> int {
            int rc = (recompute_scores && do_score) ? ensure_recompute_index(tas) : TENSILE_OK;
            if (rc != TENSILE_OK) return rc;
            const unsigned long long want = ++ready_seq;
#ifdef TENSILE_GREEDY_PROF
            const double prof_t0 = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now().time_since_epoch()).count();
#endif
            {
                WorkspaceLock ws = acquire_workspace(tas, nullptr);
                rc = launch_greedy_step(tas, *ws, recompute_scores ? tas->recompute_index : tas->index, recompute_scores, &pl, d_res.p,
                                        tables, rebuild, fresh, do_score, static_cast<Header *>(rec_dev),
                                        reinterpret_cast<CandOut *>(static_cast<Header *>(rec_dev) + 1),
                                        static_cast<unsigned long long *>(ready_dev), want);
            }
            if (rc != TENSILE_OK) return rc;
#ifdef TENSILE_GREEDY_PROF
            const double prof_t1 = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now().time_since_epoch()).count();
            g_prof_launch += prof_t1 - prof_t0;
            struct Waited { double t1; ~Waited() { g_prof_wait += std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now().time_since_epoch()).count() - t1; } } waited{prof_t1};
#endif
            // wait for the word; should it not arrive (a failed launch shows up in the stream), ask the stream
            const auto t_start = std::chrono::steady_clock::now();
            for (unsigned spins = 0; __atomic_load_n(const_cast<unsigned long long *>(ready), __ATOMIC_ACQUIRE) != want; ++spins) {
                if ((spins & 0xfff) == 0xfff && std::chrono::steady_clock::now() - t_start > std::chrono::seconds(2)) {
                    TS_HIP(hipStreamSynchronize(nullptr));
                    if (__atomic_load_n(const_cast<unsigned long long *>(ready), __ATOMIC_ACQUIRE) != want) {
                        set_error("greedy_plan: the analysis kernel finished without its record");
                        return TENSILE_E_HIP;
                    }
                    break;
                }
            }
            return TENSILE_OK;
        };
        // (the device copy of the plan receives the interval from the next iteration's kernel)
        int32_t last_gap = -1;      // the gap of the interval appended last (handed to the next iteration's kernel)
        auto append = [&](int32_t i, int32_t o, int32_t r, uint8_t kind, int32_t gap) -> int {
            last_gap = gap;
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
            // 1 accepted, 0 cannot be placed around the peak, -1 error.  The link only fills up and a gap does not
            // move, so from one attempt to the next a gap's swap-out can only end later and its swap-in only start
            // earlier (or stop fitting at all).  The window of the last attempt is remembered per gap: a candidate
            // whose remembered window already misses the peak step is passed over without placing it again, which is
            // what trying it again would come to.
            auto hopeless = [&](int32_t gap) { return gap >= 0 && (out_from[gap] >= tstar || in_until[gap] <= tstar); };
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
                    if (!link.place_earliest(p + 1, q - 1, x, &a, &e) || !link.place_latest(e + 1, q - 1, x, &cs, &d)) {
                        if (c.gap >= 0) out_from[c.gap] = INT32_MAX;      // no room any more, and never again
                        return 0;
                    }
                    o_placed = e;
                    r_placed = d + 1;
                    if (c.gap >= 0) {
                        out_from[c.gap] = o_placed;
                        in_until[c.gap] = r_placed;
                    }
                }
                if (!(o_placed < tstar && tstar < r_placed)) return 0;
                if (x != 0) {
                    link.occupy(a, e);
                    link.occupy(cs, d);
                }
                const int rc_append = append(i, o_placed, r_placed, 0, c.gap);
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
                if (!allowed(c) || hopeless(c.gap)) continue;
                const Cand cur{c.tensor, c.score, tas->h_size[c.tensor], c.wo, c.wi, c.gap};
                if (!have || later(first, cur)) {
                    first = cur;
                    have = true;
                }
            }
            if (!have) return false;
            int got = place(first);
#ifdef TENSILE_GREEDY_PROF
            ++prof_tried;
#endif
            if (got != 0) return got > 0;
#ifdef TENSILE_GREEDY_PROF
            ++prof_fallbacks;
            const double prof_f0 = prof_now();
            struct Rest { double t0; double &acc; decltype(prof_now) &now; ~Rest() { acc += now() - t0; } } rest{prof_f0, prof_rest, prof_now};
#endif
            // ... and only when it cannot be placed order the rest (a heap is popped instead of sorting them all)
            cand.clear();
            for (int32_t k = 0; k < hdr->count; ++k) {
                const CandOut &c = h_cands[k];
                if (allowed(c) && c.tensor != first.tensor && !hopeless(c.gap)) cand.push_back(Cand{c.tensor, c.score, tas->h_size[c.tensor], c.wo, c.wi, c.gap});
            }
            std::make_heap(cand.begin(), cand.end(), later);
            for (auto end = cand.end(); end != cand.begin(); --end) {
                std::pop_heap(cand.begin(), end, later);
                got = place(*(end - 1));
#ifdef TENSILE_GREEDY_PROF
                ++prof_tried;
#endif
                if (got != 0) return got > 0;
            }
            return false;
        };

        bool swap_phase = true;
        for (;;) {
            // One round trip per iteration (the scores of the last iteration's plan are not needed).
            const int32_t it = n - n_initial;
            const bool last = it >= max_new || n >= capacity || N == 0;
            pl.n_intervals = n;
            // the first footprint comes from the whole plan; afterwards exactly one interval has joined since
            // the last analysis and only its window of the row and the block maxima it touches are brought up to date
            int rc;
            if (it == 0) {
                rc = tensile_eval_plans(tas, &pl, d_res.p, d_peak.p, d_arg.p, d_min.p, nullptr);
                if (rc != TENSILE_OK) return rc;
                rc = analyse(!swap_phase, nullptr, true, !last);
            } else {
                const GreedyNew last_one{iv_tensor[n - 1], iv_out[n - 1], iv_in[n - 1], n - 1, last_gap, d_t.p, d_o.p, d_r.p};
                rc = analyse(!swap_phase, &last_one, false, !last);
            }
            if (rc != TENSILE_OK) return rc;
            P = hdr->P;
            tstar_now = hdr->tstar;
            hist.push_back(P);
            if (peak_trace) peak_trace[it] = P;
            if (last) break;
            if (opt.stop_at_budget && P <= budget_bytes) break;
            if (it > opt.min_iters && it >= 3 && (hist[it - 3] - P) * 10000 < 5 * hist[it - 3]) break;

#ifdef TENSILE_GREEDY_PROF
            const double prof_s0 = prof_now();
#endif
            const bool swapped_one = swap_phase && try_swap();
#ifdef TENSILE_GREEDY_PROF
            prof_first += prof_now() - prof_s0;
#endif
            if (swap_error != TENSILE_OK) return swap_error;
            if (!swapped_one) {
                // Recomputation branch of Alg. 3: swapping is over for good; while the peak does not fit,
                // release the never-released tensor with the largest MSPS over its whole gap.
                if (swap_phase) {
                    swap_phase = false;
                    if (!(opt.recompute && P > budget_bytes)) break;
                    rc = analyse(true, nullptr, false, true);        // same plan, same footprint: only the scores differ
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
                rc = append(best->tensor, best->wo, best->wi, 1, best->gap);
                if (rc != TENSILE_OK) return rc;
            }
        }
        TS_HIP(hipStreamSynchronize(nullptr));
#ifdef TENSILE_GREEDY_PROF
        fprintf(stderr, "[greedy prof] %d iterations: enqueue %.1f us, wait %.1f us, swap choice %.1f us (of which after the first candidate failed %.1f us, %ld times; %ld placements tried) per iteration\n",
                n - n_initial, g_prof_launch / (n - n_initial + 1), g_prof_wait / (n - n_initial + 1), prof_first / (n - n_initial + 1),
                prof_rest / (n - n_initial + 1), prof_fallbacks, prof_tried);
        g_prof_launch = g_prof_wait = 0;
        (void)prof_launch; (void)prof_wait; (void)prof_recompute;
#endif
        give_back.ok = true;
        *n_intervals = n;
        *final_peak = P;
    } catch (const std::bad_alloc &) {
        set_error("greedy_plan: out of host memory");
        return TENSILE_E_NOMEM;
    }
    return TENSILE_OK;
}
