// Internal declarations shared by the translation units of libtensile.so.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <map>
#include <memory>
#include <mutex>
#include <string>
#include <vector>

#include "tensile.h"

namespace tensile {

struct GreedyBuffers;   // greedy.hip: what a run of the planner allocates, kept by the handle for the next run

void set_error(const char *fmt, ...) __attribute__((format(printf, 1, 2)));
int hip_fail(hipError_t e, const char *what);

#define TS_HIP(call)                                               \
    do {                                                           \
        hipError_t e_ = (call);                                    \
        if (e_ != hipSuccess) return ::tensile::hip_fail(e_, #call); \
    } while (0)

// Device buffer that frees itself; plain pointer semantics otherwise.
template <typename T>
struct DevBuf {
    T *p = nullptr;
    size_t n = 0;
    bool owned = true;   // false: a view into memory somebody else owns (never freed here)
    DevBuf() = default;
    DevBuf(const DevBuf &) = delete;
    DevBuf &operator=(const DevBuf &) = delete;
    ~DevBuf() { release(); }
    void release() {
        if (p && owned) (void)hipFree(p);
        p = nullptr;
        n = 0;
        owned = true;
    }
    // (Re)allocate to hold at least `count` elements; contents are not kept.  The pointer is valid
    // afterwards even for count == 0 (one element), so kernels may issue clamped loads from it.
    hipError_t reserve(size_t count) {
        if (p && count <= n) return hipSuccess;
        release();
        hipError_t e = hipMalloc(reinterpret_cast<void **>(&p), (count ? count : 1) * sizeof(T));
        if (e == hipSuccess) n = count;
        else p = nullptr;
        return e;
    }
    hipError_t upload(const T *host, size_t count) {
        hipError_t e = reserve(count);
        if (e != hipSuccess || count == 0) return e;
        return hipMemcpy(p, host, count * sizeof(T), hipMemcpyHostToDevice);
    }
};

// Launch geometry of the evaluation kernel (see eval.hip).
constexpr int kEvalThreads = 1024;
constexpr int kEvalTile = 8192;   // steps per LDS difference tile

// Arguments of the fused scatter + scan + reduce kernel.
struct EvalArgs {
    int32_t T, N, B;
    int32_t o_min;                 // smallest admissible out step (0 for plans, -1 when building MF0)
    int64_t n_intervals;
    const int64_t *plan_offsets;
    const int32_t *iv_tensor, *iv_out, *iv_in;
    const int64_t *size;           // [N]
    const uint32_t *size_units;    // [N] size >> size_shift when that is exact and fits 32 bits, else null
    int32_t size_shift;
    const int64_t *MF0;            // [T] unscheduled timeline (read at segment starts only)
    const int64_t *dMF0;           // MF0[t] - MF0[t-1], dMF0[0] = MF0[0]; zero padded to whole tiles plus one tile
    int64_t *resident;             // [B*T] or null
    int64_t tail_threshold;        // plans with more intervals than this belong to the tail kernel
    unsigned long long *tail_flag; // set to `epoch` by the common kernel when it leaves a plan to the tail kernel
    unsigned long long epoch;      // number of this launch (per handle)
    int32_t S;                     // segments per plan
    int32_t tiles_per_seg;
    int64_t *out_max;              // S == 1: peak[B]; else partials [B*S]
    int32_t *out_arg;
    int64_t *out_min;              // may be null when S == 1
    // binned mode (batches of long plans, see eval.hip): the plans' endpoints sorted by tile
    const int2 *recs;              // [2 * n_intervals] {cell in the skewed tile | sign << 31, size units}; plan b's at 2 * offset
    const int32_t *tile_off;       // [B][n_tiles + 1] first record of each tile, relative to the plan's records
    const int64_t *tile_sum;       // [B][n_tiles] sum of the deltas that fall into each tile
    int32_t n_tiles;
};

// Scratch memory of one call chain: partial results, flags and staging that the kernels need beyond the
// caller's inputs and outputs.  A handle keeps one Workspace per HIP stream it has been called with: calls
// enqueued on one stream run one after the other and share it, calls on different streams never touch the
// same memory.  `mu` is held while a call sizes the buffers and enqueues its kernels, so two host threads
// that use the same stream enqueue whole calls, never interleaved ones.  A buffer that has to grow is
// replaced (at least doubled) and the old one is parked in `retired` until the handle is freed: kernels
// enqueued earlier may still read it, and nothing here ever waits for the device.
// fixed_base != null: the workspace lives in a preallocated region of fixed_bytes (see eval.hip, the entry
// point that allocates nothing); buffers are then carved out of it per call and never grow.
struct Workspace {
    std::mutex mu;
    hipStream_t stream = nullptr;
    DevBuf<int64_t> part_max, part_min;   // eval / windowed update: per-segment partials
    DevBuf<int32_t> part_arg;
    DevBuf<unsigned long long> tail_flag;   // eval: see EvalArgs::tail_flag (zero when allocated, then monotone)
    unsigned long long epoch = 0;           // launches of the evaluation kernel through this workspace
    DevBuf<int64_t> score_tab;     // score: per-workgroup sub-span maxima when they do not fit in LDS
    DevBuf<int32_t> job_arg;       // per-job evaluation: peak steps when the caller does not want them
    DevBuf<int2> bin_recs;         // eval, binned mode: see EvalArgs
    DevBuf<int32_t> bin_off;
    DevBuf<int64_t> bin_sum;
    DevBuf<unsigned int> apply_tickets;   // windowed update: finished runs per row (zero between launches)
    DevBuf<int32_t> link_first;    // link: earliest swap-out step per tensor, one row per workgroup (INT32_MAX between plans)
    DevBuf<int32_t> link_acc;      // link: one row per workgroup where the passes of a long plan add up
    std::vector<void *> retired;
    char *fixed_base = nullptr;
    size_t fixed_bytes = 0, fixed_used = 0;
    ~Workspace();
    // Make `b` hold at least `count` elements (contents are not kept).  *fresh, when given, says whether the
    // memory is new (the caller then initialises it on the stream).  TENSILE_OK, or an error code with the
    // message set (TENSILE_E_CAPACITY in a fixed workspace that is too small).
    template <typename T>
    int provide(DevBuf<T> &b, size_t count, const char *what, bool *fresh = nullptr);
    void begin_call() { fixed_used = fixed_base ? 256 : 0; }   // fixed: everything behind the flag's line is carved anew
};

// RAII: the workspace of (handle, stream), locked for the duration of one call's enqueueing.
struct WorkspaceLock {
    Workspace *ws = nullptr;
    std::unique_lock<std::mutex> lock;
    Workspace *operator->() const { return ws; }
    Workspace &operator*() const { return *ws; }
};

// Launch choices that tests and tuning runs may force (tensile_tuning_set); 0 / -1 = the library decides.
// Process-wide; never read from the environment.
struct Tuning {
    int eval_r = 0;            // intervals per thread kept in registers at 1024 threads
    int eval_binned = -1;      // 0 never bin, 1 bin whenever possible
    int eval_threads = 0;      // 256 / 512 / 1024
    int eval_segments = 0;     // segments per plan
    int eval_seg_steps = 0;    // most steps a segment may hold (0: 2^28, what the kernels' 32-bit cell offsets allow)
    int eval_persistent = -1;  // 0 never, 1 whenever possible
    int eval_slots = 0;        // size of the persistent grid
    int eval_nt = -1;          // footprint rows written with nontemporal stores: 0 never, 1 always, -1 by row length
    int score_blocks = 0;      // size of the scoring grid
    int link_packed = 1;       // 0: search C itself even when its packed form exists
    int step_fused = -1;       // tensile_eval_score_plans: 0 = two kernels, 1 = the fused kernel whenever its shape allows
};
extern Tuning g_tuning;

// C for the link kernel's searches (see link.hip): blocks of kLinkCBlock consecutive values, each block's six
// differences packed into 16 bytes, 21 bits each (built when every operator latency is below 2^21 ns).
constexpr int kLinkCBlock = 7;

// Per-job tables of tensile_eval_plans_per_job (see tas.hip), job-major.
struct JobTables {
    bool built = false;
    size_t T_pad = 0;
    DevBuf<int64_t> size, MF0, dMF0;   // [J][N], [J][T], [J][T_pad]
    DevBuf<uint32_t> units;            // [J][N] when the handle has 32-bit size units
};

// Geometry the scoring kernel shares with the index built at load time (see score.hip).
constexpr int kScoreThreads = 1024;
constexpr int kScoreWaves = kScoreThreads / 64;
constexpr int kScoreMaxLocal = 3072;   // bucket entries one pass handles (a "slice"); larger buckets take several
constexpr int kScoreStage = 192;       // tensors whose output (16 bytes each) one wavefront composes in LDS at a time
constexpr int kScoreMini = 256;    // steps one wavefront takes up at a time (4 consecutive steps per lane)

// Candidate index: every gap (p, q) with a feasible earliest swap-out step o, filed under each
// bucket of 2^shift steps that o+1 .. q-1 overlaps.  Per bucket (entries e0 .. e1-1, local
// index = e - e0):
//   cand / cand_size / cand_o   the entries sorted by o; slices are runs of kScoreMaxLocal of them
//   qord                        per slice, its entries as {q, index within the slice} sorted by q
//   tord                        per slice, its entries as {tensor, index within the slice} sorted by tensor
//   wave_ptr[4][kScoreWaves+1]  per slice (slices numbered from slice_first[bucket]): rows 0-2 = first position
//                               within the slice with o (resp. q) >= the w-th span boundary, tensor >= w * tspan,
//                               per order; row 3 = the span boundaries themselves: first step of wavefront w's
//                               part of the row (multiples of kScoreMini, the last one T), placed so that
//                               steps and entries together are spread evenly over the wavefronts
//   hash_dir / hash_slots       open-addressing table tensor -> {tensor, p, q, local | last << 31}
//   filter                      one bit per (tensor mod filter_bits): some entry has this tensor
struct CandIndex {
    int32_t shift = 0, n_buckets = 0;
    int32_t tspan = kScoreStage;   // tensors per wavefront: ceil(N / kScoreWaves) rounded up to kScoreStage
    int32_t filter_words = 0;      // words per bucket, a power of two
    int32_t max_bucket = 0;        // entries in the largest bucket
    DevBuf<int32_t> bucket_off;    // [n_buckets + 1]
    DevBuf<int4> cand;
    DevBuf<int64_t> cand_size;
    DevBuf<int32_t> cand_o;
    DevBuf<int32_t> cand_gap;      // the entry's gap: its number among the gaps of length >= 2 in tensor order
    DevBuf<int2> qord, tord;
    DevBuf<int32_t> slice_first;   // [n_buckets + 1]
    DevBuf<int32_t> wave_ptr;      // [slices][4][kScoreWaves + 1]
    DevBuf<int2> hash_dir;         // [n_buckets] {first slot, log2(slots)}
    DevBuf<int4> hash_slots;
    DevBuf<uint32_t> filter;       // [n_buckets][filter_words]
};

}  // namespace tensile

// The opaque handle of the C ABI.
struct tensile_tas {
    int32_t T = 0, N = 0, J = 1, G = 0;
    int device = 0;
    bool timed = false;
    int64_t base_bytes = 0, link_bytes_per_us = 0;
    int64_t unscheduled_peak = 0;
    int32_t unscheduled_argmax = 0;
    int num_cus = 256;
    // device copies
    tensile::DevBuf<int64_t> d_size, d_MF0, d_dMF0, d_C, d_x, d_touch_off;
    tensile::DevBuf<uint32_t> d_size_units;   // empty when the sizes do not fit (see EvalArgs)
    int32_t size_shift = 0;
    tensile::DevBuf<int32_t> d_touch;
    tensile::DevBuf<uint4> d_Cpack;           // [T / kLinkCBlock + 1] when c_packed
    bool c_packed = false;
    tensile::CandIndex index;                 // swap candidates: o = earliest feasible swap-out step
    // recomputation candidates (every gap, o = p), built by the first tensile_score_recompute
    mutable std::mutex lazy_mu;               // guards the two tables that are built on first use
    mutable tensile::CandIndex recompute_index;
    mutable bool recompute_index_built = false;
    std::vector<int32_t> h_gp, h_gq, h_gt;    // gaps of length >= 2 in tensor order (host)
    std::vector<int32_t> h_gap_first;         // [N+1] first gap of every tensor in those lists
    mutable tensile::JobTables job_tables;    // built by the first tensile_eval_plans_per_job
    // host copies used by the greedy driver and the validator
    std::vector<int64_t> h_size, h_C, h_x, h_touch_off;
    std::vector<int32_t> h_touch, h_job;
    // the buffers of the last tensile_greedy_plan on this handle, for the next one to take (or null)
    mutable std::mutex greedy_mu;
    mutable tensile::GreedyBuffers *greedy_cache = nullptr;
    // one workspace per stream this handle has been called with (see Workspace)
    mutable std::mutex ws_mu;
    mutable std::map<hipStream_t, std::unique_ptr<tensile::Workspace>> workspaces;
};

namespace tensile {

// workspace.hip
// The workspace of (handle, stream), created on first use, locked until the returned object goes away.
WorkspaceLock acquire_workspace(const tensile_tas *tas, hipStream_t stream);
// dst[0..n) = value, 32-bit words, by a small kernel on the stream (not a memset node: callers may capture).
int fill_words(hipStream_t stream, void *dst, size_t n_words, uint32_t value);

// Every launch_* below enqueues on ws.stream and takes its scratch from ws (locked by the caller).
// eval.hip
int launch_eval(const tensile_tas *tas, Workspace &ws, const EvalArgs &proto, int64_t *peak, int32_t *argmax,
                int64_t *min_resident);
int launch_apply(const tensile_tas *tas, Workspace &ws, int32_t B, const int32_t *tensor, const int32_t *out,
                 const int32_t *in, int64_t *resident, int64_t *peak, int32_t *argmax, int64_t *min_resident);
// score.hip
// What one greedy iteration brings back from the device: the peak, its step and the tensors with a window.
struct ScoreHeader {
    int64_t P;
    int32_t tstar, count;
};
struct ScoreCand {
    int64_t score;
    int32_t tensor, wo, wi;
    int32_t gap;                   // number of the candidate's gap (planner's kernel; -1 from the batch kernel's one-plan form)
};
// (any_interval: an interval of the entry's tensor cancels the entry wherever it lies, not only inside the gap.
//  compact != null, B == 1 only: instead of the dense rows, one record per tensor with a window, in no
//  particular order, behind *hdr = {peak, peak step, number of records}; score/win_out/win_in are not touched.
//  hdr and compact may point into pinned host memory; with ready != null the kernel, once all of that is
//  visible to the host, stores ready_value to *ready (system scope), so the host can wait for the word
//  instead of the stream.)
int launch_score(const tensile_tas *tas, Workspace &ws, const CandIndex &ix, bool any_interval, const tensile_plans *plans,
                 const int64_t *resident, const int64_t *peak, const int32_t *argmax, int64_t *score, int32_t *win_out,
                 int32_t *win_in, ScoreHeader *hdr = nullptr, ScoreCand *compact = nullptr,
                 unsigned long long *ready = nullptr, unsigned long long ready_value = 0);
// One iteration of the planner in one launch (score.hip: greedy_step_kernel).  fresh: the interval that joins the plan
// (applied to the row, written to `position` of the plan's device arrays), or null.
struct GreedyNew {
    int32_t tensor, out, in, position;
    int32_t gap;                   // number of the gap the interval lies in (as the candidate's record gave it), or -1
    int32_t *plan_t, *plan_o, *plan_r;
};
// What the planner keeps on the device from iteration to iteration besides the plan and its row.
struct GreedyTables {
    int64_t *blk_max;              // [ceil(T / kScoreMini)] maxima of the row's blocks
    int32_t *blk_arg;              // ... and the earliest step of each
    uint8_t *gap_taken;            // [G] the plan holds an interval inside this gap
    uint8_t *tensor_taken;         // [N] the plan holds an interval of this tensor
};
int launch_greedy_step(const tensile_tas *tas, Workspace &ws, const CandIndex &ix, bool any_interval, const tensile_plans *pl,
                       int64_t *row, const GreedyTables &tables, bool rebuild, const GreedyNew *fresh, bool do_score,
                       ScoreHeader *hdr, ScoreCand *compact, unsigned long long *ready, unsigned long long ready_value);
// step.hip
int launch_step(const tensile_tas *tas, Workspace &ws, const tensile_plans *plans, int64_t *resident, int64_t *peak,
                int32_t *argmax, int64_t *min_resident, int64_t *score, int32_t *win_out, int32_t *win_in);
// link.hip
int launch_link(const tensile_tas *tas, Workspace &ws, const tensile_plans *plans, bool reuse, int32_t *link, int32_t *peak,
                int32_t *argmax, int32_t *overbooked);
// greedy.hip
void drop_greedy_cache(const tensile_tas *tas);   // (at tensile_tas_free)
// tas.hip
int check_plans(const tensile_tas *tas, const tensile_plans *plans, const char *who);   // argument checks shared by the entry points
int build_times_and_index(tensile_tas *tas, const int64_t *step_ns_host);
int ensure_recompute_index(const tensile_tas *tas);

}  // namespace tensile
