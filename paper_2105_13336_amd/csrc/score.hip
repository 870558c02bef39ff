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
//   2. every wavefront streams its own contiguous span of the row, 256 steps at a
//      time, four consecutive steps per lane.  With two wave-level scans it forms,
//      per lane, the running maximum from the span's start up to the lane's steps
//      and the maximum from after them to the end of the 256, and puts both, with
//      the values themselves, in a small LDS buffer of its own; the entries whose
//      o (resp. q) falls inside these 256 steps complete their value from the
//      buffer and fold it into acc (atomic max).  Entries are met in order because
//      the bucket is sorted by o, and a second list is sorted by q; both lists sit
//      in LDS (reloaded only when the bucket changes) and the wavefront takes them
//      up 64 at a time.  The maxima of the 256-step pieces go to a table
//      (LDS), suffix-scanned within the span at the end;
//   3. the plan's own intervals cancel candidates: an interval inside the gap of
//      an entry of its tensor sets acc = +inf (Alg. 2 of the paper only takes tensors
//      that are not swapped out yet).  A per-bucket bit filter over tensors, kept in LDS,
//      turns most intervals away; the others probe the bucket's hash table.  (After
//      the streaming, not before it: +inf survives every max and overwrites one that
//      came first, so the order is free, and the streaming's many independent loads
//      make better use of the time in which the output rows of the plan before are
//      still leaving the CU than this chain of short dependent ones.)  The waves of a
//      workgroup meet at one barrier after this step; nothing before it needs one;
//   4. an entry with o < t* < q and acc != +inf scores
//      P - max( acc, pieces after q's in its span, spans before o's, spans after q's, P - size ).
// Buckets with more entries than acc holds are processed in slices of kMaxLocal
// entries, one full pass per slice; the index keeps the q order and the
// wavefronts' start positions per slice.
#include <atomic>
#include <type_traits>

#include "score_body.h"

namespace tensile {

namespace {

// ---- one iteration of the planner on the device --------------------------------------------------------
// Alg. 3 analyses the peak again after every tensor it schedules.  The planner's row exists already, so an
// iteration is: take the new interval's bytes out of its window of the row; bring the maxima (and their earliest
// steps) of the 256-step blocks the window touches up to date - the table of block maxima is kept in global
// memory from iteration to iteration: it is the block-level form of the prefix / suffix maxima of the row, of
// which only the window's part changes; find the peak and its earliest step from the table; score the candidates
// and hand the host one record per tensor with a window.  One workgroup, one launch.
//
// With the table, the blocks of the row are independent of each other: the maximum of everything before a block
// and of everything after it come from prefix / suffix scans of the table (196 entries for 50,000 steps), so the
// blocks are dealt to the wavefronts round-robin, each block is read once (from L2: the row is 400 KB), and an
// entry whose o (q) lies in a block completes max MF[0..o] (max MF[q..T)) from the block alone.  Which candidates
// the plan has already dealt with is not worked out from the plan's list again either (the list grows with
// every iteration): a flag per gap and per tensor, set as intervals join, says so.  (The batch
// kernel gives every wavefront one contiguous span instead, with boundaries balanced at load time for rows that
// come from HBM; on one L2-resident row that left the slowest wavefront 60 % behind the first.)  Rows of more than
// 131,072 steps, whose table does not fit in LDS next to the lists, take the batch kernel's body in its one-plan
// form.
struct GreedyStepArgs {
    ScoreArgs s;                 // the scoring pass: one plan (all of the interval arrays), hdr / compact / ready set
    int64_t *row;                // [T] the plan's footprint, in/out
    int64_t *blk_max;            // [ceil(T / kMini)] maxima of the row's blocks, in/out
    int32_t *blk_arg;            // [ceil(T / kMini)] earliest step of each block's maximum, in/out
    uint8_t *gap_taken;          // [gaps] the plan holds an interval inside this gap, in/out
    uint8_t *tensor_taken;       // [N] the plan holds an interval of this tensor, in/out
    int32_t new_gap;             // the new interval's gap, or -1
    const int64_t *size;         // [N]
    int32_t rebuild;             // every block's maximum is computed afresh (first launch on a row)
    int32_t has_new;             // an interval joins the plan: applied to the row and written to position plan_n
    int32_t new_tensor, new_out, new_in, plan_n;
    int32_t *plan_t, *plan_o, *plan_r;
    int32_t do_score;            // 0: only the header {peak, peak step, 0} is produced
};

constexpr int kStageRecs = 1024;   // records staged in LDS per round before they leave for the host

struct TabledLds {
    __attribute__((aligned(16))) SpanBuf buf[kWaves];     // 48 KB; after the streaming step: staging of the records
    int64_t pmx[kTabLds + 1];        // pmx[k] = max of the blocks before k (pmx[0] = -inf)
    int64_t smx[kTabLds + 1];        // smx[k] = max of the blocks k .. (smx[n_blk] = -inf)
    int64_t tb[kTabLds];             // the table itself
    int32_t ta[kTabLds];
    int32_t lo_ptr[kTabLds + 1];     // first entry of the o order with o in block k or later
    int32_t hi_ptr[kTabLds + 1];     // the same for the q order
    int64_t acc[kMaxLocal];
    int32_t lo_list[kMaxLocal];
    int2 hi_list[kMaxLocal];
    int32_t n_stage, peak_block;
};
static_assert(sizeof(SpanBuf) * kWaves >= kStageRecs * sizeof(ScoreCand), "the staging area reuses the wavefronts' buffers");

// the compact epilogue: header, then the word the host waits for
__device__ __forceinline__ void publish_header(const ScoreArgs &a, int64_t P, int32_t tstar, int32_t count) {
    *a.hdr = ScoreHeader{P, tstar, count};
    if (a.ready) {
        __threadfence_system();
        __hip_atomic_store(a.ready, a.ready_value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

// The window of the new interval leaves the row, and the table entries of the blocks it touches (of all blocks on a
// fresh row) are recomputed.  One block per wavefront and round, 4 steps per lane.
template <bool kVec>
__device__ __forceinline__ void patch_row_and_table(const GreedyStepArgs &g, int tid) {
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int32_t T = g.s.T, n_blk = g.s.n_tab;
    int64_t *const row = g.row;
    const int32_t i = g.new_tensor, o = g.new_out, r = g.new_in;
    const bool ok = g.has_new && static_cast<uint32_t>(i) < static_cast<uint32_t>(g.s.N) && o >= 0 && r <= T && r > o;
    if (g.has_new && tid == 0) {   // the plan's own arrays learn of the interval here, and so do the flags
        g.plan_t[g.plan_n] = i;
        g.plan_o[g.plan_n] = o;
        g.plan_r[g.plan_n] = r;
        if (ok) {
            g.tensor_taken[i] = 1;
            if (g.new_gap >= 0) g.gap_taken[g.new_gap] = 1;
        }
    }
    const int64_t sz = ok ? g.size[i] : 0;
    const int32_t win_lo = ok ? o + 1 : 0, win_hi = ok ? r : 0;   // steps win_lo .. win_hi - 1 lose sz bytes
    const bool any = win_hi > win_lo;
    const int32_t kb0 = g.rebuild ? 0 : (any ? win_lo / kMini : 0);
    const int32_t kb1 = g.rebuild ? n_blk : (any ? (win_hi - 1) / kMini + 1 : 0);
    for (int32_t k = kb0 + wave; k < kb1; k += kWaves) {   // (wave-uniform)
        const int32_t t = k * kMini + 4 * lane;
        int64_t x[4];
        load_quad<kVec>(row, t, T, x);    // steps beyond T come back as INT64_MIN and lie outside every window
        bool ch[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            ch[j] = t + j >= win_lo && t + j < win_hi;
            x[j] -= ch[j] ? sz : 0;
        }
#pragma unroll
        for (int j = 0; j < 4; j += 2) {
            if (kVec && ch[j] && ch[j + 1]) {
                *reinterpret_cast<ll2 *>(row + t + j) = ll2{x[j], x[j + 1]};
            } else {
                if (ch[j]) row[t + j] = x[j];
                if (ch[j + 1]) row[t + j + 1] = x[j + 1];
            }
        }
        const int64_t lm = max64(max64(x[0], x[1]), max64(x[2], x[3]));
        int32_t lj = 3;
#pragma unroll
        for (int j = 2; j >= 0; --j)
            if (x[j] == lm) lj = j;
        const int64_t m = last_lane(wave_scan_max(lm));
        const uint64_t holders = __builtin_amdgcn_ballot_w64(lm == m);   // (never empty)
        if (lane == __builtin_ctzll(holders)) {
            g.blk_max[k] = m;
            g.blk_arg[k] = t + lj;
        }
    }
}

// kBigT == false: the table-driven scoring pass described above.  kBigT == true: the batch kernel's body.
template <bool kBigT, bool kVec>
__global__ __launch_bounds__(kThreads) void greedy_step_kernel(const GreedyStepArgs g) {
    typedef typename std::conditional<kBigT, ScoreLds<true>, TabledLds>::type Lds;
    __shared__ Lds lds;
    __shared__ int64_t red_v[kWaves];
    __shared__ int32_t red_k[kWaves];
    __shared__ int64_t s_peak;
    __shared__ int32_t s_step;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
#ifdef TENSILE_SCORE_PROF
    unsigned long long prof_t = wall_clock64();
#endif
    const ScoreArgs &a = g.s;
    const int32_t T = a.T, n_blk = a.n_tab;
    patch_row_and_table<kVec>(g, tid);
    // other wavefronts of this workgroup read what these stores wrote (table entries now, the row in the scoring pass)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");

    if constexpr (kBigT) {
        // ---- the peak: largest block maximum, earliest block among equals
        int64_t bv = INT64_MIN;
        int32_t bk = INT32_MAX;
        for (int32_t k = tid; k < n_blk; k += kThreads) {   // (a thread meets its blocks in ascending order)
            const int64_t v = g.blk_max[k];
            if (v > bv) {
                bv = v;
                bk = k;
            }
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            const int64_t ov = __shfl_xor(bv, d, 64);
            const int32_t ok2 = __shfl_xor(bk, d, 64);
            if (ov > bv || (ov == bv && ok2 < bk)) {
                bv = ov;
                bk = ok2;
            }
        }
        if (lane == 0) {
            red_v[wave] = bv;
            red_k[wave] = bk;
        }
        __syncthreads();
        if (tid == 0) {
#pragma unroll
            for (int w = 1; w < kWaves; ++w)
                if (red_v[w] > bv || (red_v[w] == bv && red_k[w] < bk)) {
                    bv = red_v[w];
                    bk = red_k[w];
                }
            s_peak = bv;
            s_step = g.blk_arg[bk];
        }
        __syncthreads();
    } else {
        // ---- the table into LDS; its prefix and suffix maxima; the peak and the first block that holds it
        for (int32_t k = tid; k < n_blk; k += kThreads) {
            lds.tb[k] = g.blk_max[k];
            lds.ta[k] = g.blk_arg[k];
        }
        if (tid == 0) lds.peak_block = INT32_MAX;
        __syncthreads();
        if (wave == 0) {          // pmx[k + 1] = max tb[0..k]
            int64_t run = INT64_MIN;
            if (lane == 0) lds.pmx[0] = INT64_MIN;
            for (int32_t k0 = 0; k0 < n_blk; k0 += 64) {
                const int32_t k = k0 + lane;
                const int64_t incl = max64(wave_scan_max(k < n_blk ? lds.tb[k] : INT64_MIN), run);
                if (k < n_blk) lds.pmx[k + 1] = incl;
                run = last_lane(incl);
            }
            if (lane == 0) s_peak = run;
        } else if (wave == 1) {   // smx[k] = max tb[k..]
            int64_t run = INT64_MIN;
            if (lane == 0) lds.smx[n_blk] = INT64_MIN;
            for (int32_t top = n_blk; top > 0; top -= 64) {
                const int32_t k = top - 1 - lane;
                const int64_t incl = max64(wave_scan_max(k >= 0 ? lds.tb[k] : INT64_MIN), run);
                if (k >= 0) lds.smx[k] = incl;
                run = last_lane(incl);
            }
        }
        __syncthreads();
        for (int32_t k = tid; k < n_blk; k += kThreads)
            if (lds.tb[k] == s_peak) atomicMin(&lds.peak_block, k);
        __syncthreads();
        if (tid == 0) s_step = lds.ta[lds.peak_block];
        __syncthreads();
    }
    const int32_t tstar = __builtin_amdgcn_readfirstlane(s_step);
    const uint32_t p_lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(s_peak));
    const uint32_t p_hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(static_cast<uint64_t>(s_peak) >> 32));
    const int64_t P = static_cast<int64_t>((static_cast<uint64_t>(p_hi) << 32) | p_lo);
#ifdef TENSILE_SCORE_PROF
#define STEP_MARK(k) do { if (tid == 0) { const unsigned long long now_ = wall_clock64(); atomicAdd(&g_score_prof[k], now_ - prof_t); prof_t = now_; } } while (0)
#else
#define STEP_MARK(k) do { } while (0)
#endif
    STEP_MARK(6);
    if (!g.do_score) {
        if (tid == 0) publish_header(a, P, tstar, 0);
        return;
    }
    if constexpr (kBigT) {
        ScoreCarry carry;
#ifdef TENSILE_SCORE_PROF
        carry.prof_t = prof_t;
#endif
        score_plan<true, kVec, true>(a, 0, tstar, P, lds, a.tab_scratch, carry);   // (one workgroup: its scratch table is the first)
    } else {
        const int64_t *const MF = g.row;
        const int32_t bk = tstar >> a.bucket_shift;
        const int32_t e0 = uniform_load(a.bucket_off, bk), n_e = uniform_load(a.bucket_off, bk + 1) - e0;
        int32_t n_out = 0;     // records handed to the host so far (the same in every thread)
        for (int32_t slice_lo = 0; slice_lo < n_e; slice_lo += kMaxLocal) {
            const int32_t n_slice = min(kMaxLocal, n_e - slice_lo);
            __syncthreads();   // the previous slice has finished with the lists, acc and the staging area
            // ---- the slice's lists; per block, where its entries start in each order
            for (int32_t k = tid; k < n_slice; k += kThreads) {
                lds.acc[k] = INT64_MIN;
                lds.lo_list[k] = a.cand_o[e0 + slice_lo + k];
                lds.hi_list[k] = a.qord[e0 + slice_lo + k];
            }
            if (tid == 0) lds.n_stage = 0;
            // this thread's entries for the last step (three at most), requested now: what they are scored from is
            // static, and the flags were set before the barrier above; all of it is on its way while the row streams
            constexpr int kPer = kMaxLocal / kThreads;
            static_assert(kPer * kThreads == kMaxLocal && kStageRecs == kThreads, "one entry per thread and round of the last step");
            int4 my_c[kPer];
            int32_t my_gap[kPer];
            int64_t my_sz[kPer];
#pragma unroll
            for (int j = 0; j < kPer; ++j) {
                const int32_t k = j * kThreads + tid;
                const int32_t e = e0 + slice_lo + (k < n_slice ? k : 0);
                my_c[j] = a.cand[e];
                my_gap[j] = a.cand_gap[e];
                my_sz[j] = a.cand_size[e];
            }
            __syncthreads();
            STEP_MARK(0);
            // lo_ptr[b] / hi_ptr[b]: the first entry of the o / q order whose step lies in block b or later - one
            // binary search per block and order, all blocks at once.  (Walking the entries and filling in the blocks
            // between two of them left the ~100 blocks before the first entry, and as many after the last, to a
            // single thread: 6.7 us of every iteration.)
            for (int32_t bq = tid; bq <= 2 * n_blk + 1; bq += kThreads) {
                const bool hi_order = bq > n_blk;
                const int32_t blk = hi_order ? bq - n_blk - 1 : bq;
                const int32_t bound = blk * kMini;                 // (blk == n_blk: past every step)
                int32_t lo = 0, hi = n_slice;                      // first k with step(k) >= bound
                while (lo < hi) {
                    const int32_t mid = (lo + hi) >> 1;
                    const int32_t step = hi_order ? lds.hi_list[mid].x : lds.lo_list[mid];
                    if (step < bound) lo = mid + 1;
                    else hi = mid;
                }
                if (hi_order) lds.hi_ptr[blk] = lo;
                else lds.lo_ptr[blk] = lo;
            }
            uint8_t my_taken[kPer];
#pragma unroll
            for (int j = 0; j < kPer; ++j) my_taken[j] = a.any_interval ? g.tensor_taken[my_c[j].w] : g.gap_taken[my_gap[j] < 0 ? 0 : my_gap[j]];
            __syncthreads();
            STEP_MARK(1);
            // ---- the row's blocks, dealt round-robin; a block without an endpoint of the slice is not even read.
            // (Taken one by one from a common counter instead - the entries are spread unevenly over the blocks, and
            // the first wavefront waits 3 us for the last - the wait shrinks to 2 us and the step grows by 2: the
            // atomic and its way back into a scalar register sit in front of every request.)
            {
                SpanBuf *const buf = &lds.buf[wave];
                auto wanted = [&](int32_t kb) { return kb < n_blk && (lds.lo_ptr[kb + 1] > lds.lo_ptr[kb] || lds.hi_ptr[kb + 1] > lds.hi_ptr[kb]); };
                auto next_wanted = [&](int32_t kb) {     // (wave-uniform)
                    while (kb < n_blk && !wanted(kb)) kb += kWaves;
                    return kb;
                };
                // The wavefront's blocks are requested kAhead ahead (the row sits in L2; with one request in flight
                // per wavefront every block would cost a full round trip).  The requests live in kAhead fixed sets
                // of registers, taken in turn - rotating them would mean waiting for the youngest - and are always
                // issued, at clamped addresses past the end, so that every wait names an exact count.
                constexpr int kAhead = 4;
                int32_t kq[kAhead];            // the block each set of registers holds (>= n_blk: none)
                int64_t x[kAhead][4];
                int32_t cursor = wave;         // where the search for the wavefront's next block goes on
#pragma unroll
                for (int d = 0; d < kAhead; ++d) {
                    kq[d] = next_wanted(cursor);
                    cursor = kq[d] + kWaves;
                    load_quad<kVec>(MF, (kq[d] < n_blk ? kq[d] : n_blk) * kMini + 4 * lane, T, x[d]);
                }
                for (bool more = true; more;) {
#pragma unroll
                    for (int d = 0; d < kAhead; ++d) {
                        const int32_t kb = kq[d];
                        if (kb >= n_blk) {     // (wave-uniform; the blocks come in ascending order: nothing is left)
                            more = false;
                            break;
                        }
                        const int64_t v0 = x[d][0], v1 = x[d][1], v2 = x[d][2], v3 = x[d][3];
                        kq[d] = next_wanted(cursor);
                        cursor = kq[d] + kWaves;
                        load_quad<kVec>(MF, (kq[d] < n_blk ? kq[d] : n_blk) * kMini + 4 * lane, T, x[d]);
                        const int32_t t0 = kb * kMini;
                        const int64_t before_blk = lds.pmx[kb], after_blk = lds.smx[kb + 1];
                        const int64_t m = max64(max64(v0, v1), max64(v2, v3));
                        // (this pass is bound by its instructions - one CU for the whole row - and the two scans are
                        // most of them: where the block's values share their upper halves, as they nearly always do,
                        // the scans run on the lower ones)
                        int64_t fwd, rs;
                        const int32_t m_hi = static_cast<int32_t>(m >> 32);
                        if (__builtin_amdgcn_ballot_w64(m_hi != __builtin_amdgcn_readfirstlane(m_hi)) == 0) {   // (wave-uniform)
                            const int64_t top = static_cast<int64_t>(static_cast<uint64_t>(static_cast<uint32_t>(m_hi)) << 32);
                            fwd = top | wave_scan_umax32(static_cast<uint32_t>(m));
                            rs = top | wave_rscan_umax32(static_cast<uint32_t>(m), lane);
                        } else {
                            fwd = wave_scan_max(m);
                            rs = wave_rscan_max(m, lane);
                        }
                        const int64_t incl = max64(fwd, before_blk);
                        const int64_t excl = from_prev_lane(incl, before_blk);          // max MF[0 .. t0 + 4 lane - 1]
                        const int64_t rs_next = max64(from_next_lane(rs, INT64_MIN), after_blk);   // max MF[t0 + 4 lane + 4 .. T)
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        reinterpret_cast<ll2 *>(buf->raw)[2 * lane] = ll2{v0, v1};
                        reinterpret_cast<ll2 *>(buf->raw)[2 * lane + 1] = ll2{v2, v3};
                        buf->before[lane] = excl;
                        buf->after[lane] = rs_next;
                        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                        for (int32_t k = lds.lo_ptr[kb] + lane; k < lds.lo_ptr[kb + 1]; k += 64) {
                            const int32_t r = lds.lo_list[k] - t0, l = r >> 2, j = r & 3;
                            int64_t v = max64(buf->before[l], buf->raw[4 * l]);
                            if (j >= 1) v = max64(v, buf->raw[4 * l + 1]);
                            if (j >= 2) v = max64(v, buf->raw[4 * l + 2]);
                            if (j >= 3) v = max64(v, buf->raw[4 * l + 3]);
                            atomicMax(reinterpret_cast<long long *>(lds.acc + k), static_cast<long long>(v));
                        }
                        for (int32_t k = lds.hi_ptr[kb] + lane; k < lds.hi_ptr[kb + 1]; k += 64) {
                            const int2 it = lds.hi_list[k];
                            const int32_t r = it.x - t0, l = r >> 2, j = r & 3;
                            int64_t v = max64(buf->after[l], buf->raw[4 * l + 3]);
                            if (j <= 2) v = max64(v, buf->raw[4 * l + 2]);
                            if (j <= 1) v = max64(v, buf->raw[4 * l + 1]);
                            if (j <= 0) v = max64(v, buf->raw[4 * l]);
                            atomicMax(reinterpret_cast<long long *>(lds.acc + it.y), static_cast<long long>(v));
                        }
                        __builtin_amdgcn_wave_barrier();
                    }
                }
            }
            STEP_MARK(3);
            __syncthreads();
            STEP_MARK(4);
            // ---- scores of the surviving candidates, staged in LDS (where the wavefronts' buffers were) kStageRecs
            // at a time and sent to the host as whole lines
            ScoreCand *const stage = reinterpret_cast<ScoreCand *>(lds.buf);
            int32_t staged_before = 0;     // (n_stage counts the slice's records so far; it is reset at the slice's start)
#pragma unroll
            for (int j = 0; j < kPer; ++j) {
                const int32_t r0 = j * kStageRecs;
                if (r0 >= n_slice) break;      // (block-uniform)
                const int32_t k = r0 + tid;
                if (k < n_slice) {
                    // (a candidate the plan has already dealt with is out: an interval inside the entry's gap - or,
                    // for recomputation, any interval of its tensor - which the flags record as the plan grows)
                    const int4 c = my_c[j];
                    const int32_t gap = my_gap[j];
                    const int64_t sz = my_sz[j];
                    const int64_t v = lds.acc[k];
                    const bool taken = my_taken[j] != 0;
                    if (c.z < tstar && tstar < c.y && !taken)
                        stage[atomicAdd(&lds.n_stage, 1) - staged_before] = ScoreCand{P - max64(v, P - sz), c.w, c.z, c.y, gap};
                }
                __syncthreads();
                STEP_MARK(2);
                const int32_t n_st = lds.n_stage - staged_before;
                const int64_t *src = reinterpret_cast<const int64_t *>(stage);
                int64_t *dst = reinterpret_cast<int64_t *>(a.compact + n_out);
                for (int32_t w = tid; w < 3 * n_st; w += kThreads) dst[w] = src[w];
                n_out += n_st;
                staged_before += n_st;
                __syncthreads();       // the staging area is free again
                STEP_MARK(5);
            }
        }
        // the header travels with the records: one wait for the host's memory instead of two.  The barrier orders every
        // thread's records before thread 0's store of the signal, and that store releases at system scope - which
        // covers what happened before it in other threads too (a system-scope fence in each of the 1024 threads,
        // as it was first written, cost 2 us per iteration more)
        if (tid == 0) *a.hdr = ScoreHeader{P, tstar, n_out};
        __syncthreads();
        if (tid == 0 && a.ready) __hip_atomic_store(a.ready, a.ready_value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        STEP_MARK(7);
    }
#undef STEP_MARK
}

}  // namespace

// One iteration of tensile_greedy_plan on the device (see greedy_step_kernel).  pl: the one plan INCLUDING the new
// interval (n_intervals counts it; its slot in the device arrays is written by the kernel).
int launch_greedy_step(const tensile_tas *tas, Workspace &ws, const CandIndex &ix, bool any_interval, const tensile_plans *pl,
                       int64_t *row, const GreedyTables &tables, bool rebuild, const GreedyNew *fresh, bool do_score,
                       ScoreHeader *hdr, ScoreCand *compact, unsigned long long *ready, unsigned long long ready_value) {
    GreedyStepArgs g{};
    g.s = make_score_args(tas, ix, any_interval, pl, row, nullptr, nullptr, nullptr, nullptr, nullptr);
    g.s.hdr = hdr; g.s.compact = compact; g.s.ready = ready; g.s.ready_value = ready_value;
    g.row = row; g.blk_max = tables.blk_max; g.blk_arg = tables.blk_arg; g.size = tas->d_size.p;
    g.gap_taken = tables.gap_taken; g.tensor_taken = tables.tensor_taken; g.new_gap = -1;
    g.rebuild = rebuild ? 1 : 0;
    g.do_score = (do_score && tas->N > 0) ? 1 : 0;
    if (fresh) {
        g.has_new = 1;
        g.new_tensor = fresh->tensor; g.new_out = fresh->out; g.new_in = fresh->in; g.plan_n = fresh->position;
        g.new_gap = fresh->gap;
        g.plan_t = fresh->plan_t; g.plan_o = fresh->plan_o; g.plan_r = fresh->plan_r;
    }
    const bool big_t = g.s.n_tab > kTabLds;
    if (big_t && g.do_score) {
        const int rc = ws.provide(ws.score_tab, static_cast<size_t>(g.s.n_tab), "greedy: block maxima of the scoring pass");
        if (rc != TENSILE_OK) return rc;
        g.s.tab_scratch = ws.score_tab.p;
    }
    const hipStream_t stream = ws.stream;
    if (big_t) {
        if (g.s.vec16) hipLaunchKernelGGL((greedy_step_kernel<true, true>), dim3(1), dim3(kThreads), 0, stream, g);
        else hipLaunchKernelGGL((greedy_step_kernel<true, false>), dim3(1), dim3(kThreads), 0, stream, g);
    } else {
        if (g.s.vec16) hipLaunchKernelGGL((greedy_step_kernel<false, true>), dim3(1), dim3(kThreads), 0, stream, g);
        else hipLaunchKernelGGL((greedy_step_kernel<false, false>), dim3(1), dim3(kThreads), 0, stream, g);
    }
    TS_HIP(hipGetLastError());
    return TENSILE_OK;
}

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
        unsigned long long z[8 + 2 * 16] = {};
        (void)hipMemcpyToSymbol(HIP_SYMBOL(g_score_prof), z, sizeof(z));
    }
    return 0;
}
#endif

}  // namespace tensile
