// Candidate scoring (section IV-C of the paper): for every plan, how much would
// evicting each tensor that is resident and idle at the peak lower the peak,
// given the earliest swap-out / latest swap-in the host link's speed allows:
//   score = P - max( max MF[0..o], max MF[q..T), P - size ).
//
// Which tensors can be candidates at a peak step t* does not depend on the plan:
// they are the gaps (p, q) of the TAS with a feasible earliest swap-out step o
// (a property of the gap alone: it follows from p, q, the transfer time and the
// cumulative latency) and o < t* < q.  tensile_tas_load files every such gap
// under each bucket of 2^shift steps that (o, q) overlaps, so a plan looks at the
// one bucket of its t* (see CandIndex in common.h).  Everything a plan needs
// beyond its own footprint row and interval list is static, shared by all plans
// with the same bucket, and read in order; the row is read exactly once, in
// order, and nothing per plan is kept in global memory (except, for rows longer
// than 131,072 steps, one word per 256 steps).  The recomputation savings
// (section IV-D) use the same kernel on a second index in which every gap is
// filed with o = p, and any interval of a tensor cancels its entries.
//
// One workgroup walks a plan at a time (persistent workgroups, plans dealt
// round-robin).  Per plan, with acc[] one word per bucket entry in LDS:
//   1. the plan's output rows are cleared (score 0, windows -1); acc = -inf;
//   2. the plan's own intervals cancel candidates: an interval inside the gap of
//      an entry of its tensor sets acc = +inf (Alg. 2 of the paper only takes tensors
//      that are not swapped out yet).  A per-bucket bit filter over tensors, kept in LDS,
//      turns most intervals away; the others probe the bucket's hash table;
//   3. every wavefront streams its own contiguous span of the row, 256 steps at a
//      time, four consecutive steps per lane.  With two wave-level scans it forms,
//      per lane, the running maximum from the span's start up to the lane's steps
//      and the maximum from after them to the end of the 256, and puts both, with
//      the values themselves, in a small LDS buffer of its own; the entries whose
//      o (resp. q) falls inside these 256 steps complete their value from the
//      buffer and fold it into acc (atomic max).  Entries are met in order because
//      the bucket is sorted by o, and a second list is sorted by q; both lists sit
//      in LDS (reloaded only when the bucket changes) and the wavefront takes them
//      up 64 at a time.  The maxima of the 256-step pieces go to a table
//      (LDS), suffix-scanned within the span at the end.  The waves of a workgroup
//      meet at one barrier after this step; nothing inside it needs one;
//   4. an entry with o < t* < q and acc != +inf scores
//      P - max( acc, pieces after q's in its span, spans before o's, spans after q's, P - size ).
// Buckets with more entries than acc holds are processed in slices of kMaxLocal
// entries, one full pass per slice; the index keeps the q order and the
// wavefronts' start positions per slice.
#include <atomic>

#include "score_body.h"

namespace tensile {

namespace {

}  // namespace

int launch_score(const tensile_tas *tas, Workspace &ws, const CandIndex &ix, bool any_interval, const tensile_plans *plans,
                 const int64_t *resident, const int64_t *peak, const int32_t *argmax, int64_t *score, int32_t *win_out,
                 int32_t *win_in, ScoreHeader *hdr, ScoreCand *compact, unsigned long long *ready,
                 unsigned long long ready_value) {
    if (plans->B == 0 || tas->N == 0) return TENSILE_OK;
    const hipStream_t stream = ws.stream;
    if (compact && (plans->B != 1 || !hdr)) { set_error("score: the compact form takes one plan"); return TENSILE_E_INVAL; }
    // as many workgroups as the device keeps resident, the plans dealt evenly among them
    const bool big_t = (tas->T + kMini - 1) / kMini > kTabLds;
    static std::atomic<int> per_cu_of[2];   // (0 = not asked yet; every thread that asks stores the same answer)
    int per_cu = per_cu_of[big_t ? 1 : 0].load(std::memory_order_relaxed);
    if (per_cu == 0) {
        int n = 0;
        if (big_t) TS_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, score_kernel<true, true, false>, kThreads, 0));
        else TS_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, score_kernel<false, true, false>, kThreads, 0));
        per_cu = n > 0 ? n : 1;
        per_cu_of[big_t ? 1 : 0].store(per_cu, std::memory_order_relaxed);
    }
    const int64_t resident_blocks = static_cast<int64_t>(tas->num_cus) * per_cu;
    const int64_t rounds = (plans->B + resident_blocks - 1) / resident_blocks;
    int32_t blocks = static_cast<int32_t>((plans->B + rounds - 1) / rounds);
    if (const int v = g_tuning.score_blocks; v > 0)   // tuning knob: size of the grid (plans are dealt round-robin)
        blocks = v < plans->B ? v : plans->B;
    ScoreArgs a = make_score_args(tas, ix, any_interval, plans, resident, peak, argmax, score, win_out, win_in);
    a.hdr = hdr; a.compact = compact;
    a.ready = ready; a.ready_value = ready_value;
    if (a.n_tab > kTabLds) {
        const size_t need = static_cast<size_t>(blocks) * static_cast<size_t>(a.n_tab);
        const int rc = ws.provide(ws.score_tab, need, "score: block maxima");
        if (rc != TENSILE_OK) return rc;
        a.tab_scratch = ws.score_tab.p;
    }
#define TS_LAUNCH_SCORE(BIG, VEC)                                                                                      \
    do {                                                                                                               \
        if (compact) hipLaunchKernelGGL((score_kernel<BIG, VEC, true>), dim3(blocks), dim3(kThreads), 0, stream, a);   \
        else hipLaunchKernelGGL((score_kernel<BIG, VEC, false>), dim3(blocks), dim3(kThreads), 0, stream, a);          \
    } while (0)
    if (big_t) {
        if (a.vec16) TS_LAUNCH_SCORE(true, true);
        else TS_LAUNCH_SCORE(true, false);
    } else {
        if (a.vec16) TS_LAUNCH_SCORE(false, true);
        else TS_LAUNCH_SCORE(false, false);
    }
#undef TS_LAUNCH_SCORE
    TS_HIP(hipGetLastError());
    return TENSILE_OK;
}

#ifdef TENSILE_SCORE_PROF
extern "C" int tensile_debug_score_prof(unsigned long long *out, int reset) {
    if (out) (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_score_prof), sizeof(g_score_prof));
    if (reset) {
        unsigned long long z[8] = {};
        (void)hipMemcpyToSymbol(HIP_SYMBOL(g_score_prof), z, sizeof(z));
    }
    return 0;
}
#endif

}  // namespace tensile
