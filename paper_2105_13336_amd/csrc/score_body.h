// Candidate scoring of one plan (section IV-C of the paper) as a device function over an LDS struct, and what
// it shares with the kernels built around it.  Included by score.hip (persistent scoring workgroups) and by
// step.hip (evaluation and scoring of a plan in one workgroup).  Everything here has internal linkage.
#pragma once

#include "common.h"
#include "wave_ops.h"

namespace tensile {

namespace {

constexpr int kThreads = kScoreThreads;
constexpr int kWaves = kScoreWaves;
constexpr int kMini = kScoreMini;
constexpr int kMaxLocal = kScoreMaxLocal;   // bucket entries per slice (acc 24 KB, o and q lists 36 KB, tensor order 30 KB)
constexpr int kDepth = 2;           // blocks of kMini steps in flight per wavefront while streaming
constexpr int kTabLds = 512;        // pieces of kMini steps whose maxima fit in LDS (T <= 131072)
constexpr int kFilterWords = 1024;  // largest per-bucket filter (32768 bits)
constexpr int kIvU = 4;             // intervals per thread and round

typedef long long ll2 __attribute__((ext_vector_type(2)));

struct ScoreArgs {
    int32_t T, N, B;
    int32_t tspan;               // tensors per wavefront (a multiple of kScoreStage)
    int32_t n_tab;               // ceil(T / kMini)
    int32_t vec16;               // rows are 16-byte aligned (T even, aligned base)
    int32_t any_interval;        // an interval of the entry's tensor cancels it wherever it lies
    int64_t n_intervals;
    const int64_t *plan_offsets;
    const int32_t *iv_tensor, *iv_out, *iv_in;
    int32_t bucket_shift, filter_words;
    const int32_t *bucket_off;
    const int4 *cand;
    const int64_t *cand_size;
    const int32_t *cand_o;
    const int32_t *cand_gap;
    const int2 *qord, *tord;
    const int32_t *slice_first;
    const int32_t *wave_ptr;
    const int2 *hash_dir;
    const int4 *hash_slots;
    const uint32_t *filter;
    const int64_t *resident;
    const int64_t *peak;
    const int32_t *argmax;
    int64_t *score;
    int32_t *win_out, *win_in;
    int64_t *tab_scratch;        // [gridDim.x][n_tab] when n_tab > kTabLds, else null
    ScoreHeader *hdr;            // compact mode (B == 1): records instead of rows, see launch_score
    ScoreCand *compact;
    unsigned long long *ready;   // compact mode: receives ready_value when header and records are visible system-wide (may be null)
    unsigned long long ready_value;
};

// row[0..n) = v with 16-byte stores where the row allows them
template <typename E>
__device__ __forceinline__ void fill_row(E *row, int32_t n, E v, int tid) {
    constexpr int kPer = 16 / sizeof(E);
    typedef E vec_t __attribute__((ext_vector_type(kPer)));
    const uintptr_t addr = reinterpret_cast<uintptr_t>(row);
    int32_t head = static_cast<int32_t>(((16 - (addr & 15)) & 15) / sizeof(E));
    if (head > n) head = n;
    if (tid < head) row[tid] = v;
    const int32_t n_vec = (n - head) / kPer;
    vec_t *dst = reinterpret_cast<vec_t *>(row + head);
    vec_t vv;
#pragma unroll
    for (int j = 0; j < kPer; ++j) vv[j] = v;
    for (int32_t k = tid; k < n_vec; k += kThreads) dst[k] = vv;
    const int32_t done = head + n_vec * kPer;
    if (done + tid < n) row[done + tid] = v;
}

// Four consecutive steps of the row starting at step t (a multiple of 4; two 16-byte loads when
// the row allows them).  The loads are always issued, at clamped addresses; steps outside
// [0, T) come back as INT64_MIN.
// kStream (the scoring pass over rows of more than 131,072 steps): the row is read once, with nontemporal loads,
// which leave the L2 to the candidate index and the sub-span maxima (rows of 10^6 steps: 2.49 -> 2.40 ms per batch
// of 1024 plans; on rows of 50,000 steps the same loads cost 18 %, on 24,000-step rows 14 %).
template <bool kVec, bool kStream = false>
__device__ __forceinline__ void load_quad(const int64_t *MF, int32_t t, int32_t T, int64_t (&x)[4]) {
    if (kVec) {   // T is even here, so an even step t' < T implies t' + 1 < T
        const ll2 *const at_lo = reinterpret_cast<const ll2 *>(MF + (t < T ? t : T - 2));
        const ll2 *const at_hi = reinterpret_cast<const ll2 *>(MF + (t + 2 < T ? t + 2 : T - 2));
        ll2 lo, hi;
        if constexpr (kStream) {
            lo = __builtin_nontemporal_load(at_lo);
            hi = __builtin_nontemporal_load(at_hi);
        } else {
            lo = *at_lo;
            hi = *at_hi;
        }
        x[0] = lo[0]; x[1] = lo[1]; x[2] = hi[0]; x[3] = hi[1];
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) x[j] = MF[t + j < T ? t + j : T - 1];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (t + j >= T) x[j] = INT64_MIN;
}

// Inclusive max-scan over the 64 lanes from the high end: lane l receives the maximum of lanes
// l .. 63.  Shifts towards lower lanes inside rows of 16, then the totals of the later rows.
__device__ __forceinline__ int64_t wave_rscan_max(int64_t x, int lane) {
    x = max64(x, dpp_move<0x101, 0xf>(x, INT64_MIN));
    x = max64(x, dpp_move<0x102, 0xf>(x, INT64_MIN));
    x = max64(x, dpp_move<0x104, 0xf>(x, INT64_MIN));
    x = max64(x, dpp_move<0x108, 0xf>(x, INT64_MIN));
    const int64_t r3 = lane_value(x, 48);
    const int64_t r2 = max64(lane_value(x, 32), r3);
    const int64_t r1 = max64(lane_value(x, 16), r2);
    const int64_t later = lane < 16 ? r1 : (lane < 32 ? r2 : (lane < 48 ? r3 : INT64_MIN));
    return max64(x, later);
}

// The same two scans over unsigned 32-bit values (a single instruction per step instead of a 64-bit compare and
// two selects): for values that share their upper halves, the maximum is decided by the lower ones.
template <int kCtrl, int kRowMask>
__device__ __forceinline__ uint32_t dpp_umax32(uint32_t x) {
    const uint32_t y = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), kCtrl, kRowMask, 0xf, true));
    return x > y ? x : y;
}
__device__ __forceinline__ uint32_t wave_scan_umax32(uint32_t x) {
    x = dpp_umax32<0x111, 0xf>(x);
    x = dpp_umax32<0x112, 0xf>(x);
    x = dpp_umax32<0x114, 0xf>(x);
    x = dpp_umax32<0x118, 0xf>(x);
    x = dpp_umax32<0x142, 0xa>(x);
    x = dpp_umax32<0x143, 0xc>(x);
    return x;
}
__device__ __forceinline__ uint32_t wave_rscan_umax32(uint32_t x, int lane) {
    x = dpp_umax32<0x101, 0xf>(x);
    x = dpp_umax32<0x102, 0xf>(x);
    x = dpp_umax32<0x104, 0xf>(x);
    x = dpp_umax32<0x108, 0xf>(x);
    const uint32_t r3 = __builtin_amdgcn_readlane(static_cast<int>(x), 48);
    const uint32_t q2 = __builtin_amdgcn_readlane(static_cast<int>(x), 32), r2 = q2 > r3 ? q2 : r3;
    const uint32_t q1 = __builtin_amdgcn_readlane(static_cast<int>(x), 16), r1 = q1 > r2 ? q1 : r2;
    const uint32_t later = lane < 16 ? r1 : (lane < 32 ? r2 : (lane < 48 ? r3 : 0u));
    return x > later ? x : later;
}

// value of the previous / next lane; the first / last lane receives `edge`
__device__ __forceinline__ int64_t from_prev_lane(int64_t x, int64_t edge) { return dpp_move<0x138, 0xf>(x, edge); }   // wave_shr:1
__device__ __forceinline__ int64_t from_next_lane(int64_t x, int64_t edge) { return dpp_move<0x130, 0xf>(x, edge); }   // wave_shl:1

// Step 3 for one wavefront: its span [span_lo, span_hi) of the row.  Returns the span's maximum.
//   lo_k .. lo_end   the wavefront's entries in o order (positions local to the bucket)
//   hi_k .. hi_end   its items of the q order
//   slice_lo, n_slice   the slice of the bucket acc covers
// The span is taken up kMini = 256 steps at a time, four consecutive steps per lane.  Per lane
// the wavefront's buffer in LDS receives the four values, the maximum from the span's start up
// to just before them (before[]) and the maximum from just after them to the end of the 256
// (after[]); an entry completes its value from these:
//   max MF[span_lo .. o]     = max( before[l], the lane's values up to o )     l = (o - t0) / 4
//   max MF[q .. t0 + 255]    = max( after[l],  the lane's values from q on )
// Both lists are met in order.  The wavefront holds a window of 64 consecutive items of each,
// one per lane, and the window after it, requested when the current one was taken up; `pos`
// counts the lanes of the window already served.
struct SpanBuf {
    int64_t raw[kMini];
    int64_t before[64], after[64];
};

template <bool kVec, bool kStream, typename Tab>
__device__ __forceinline__ int64_t stream_span(const ScoreArgs &a, const int64_t *MF, int32_t span_lo, int32_t span_hi,
                                               const int32_t *lo_list, const int2 *hi_list, int32_t lo_k, int32_t lo_end,
                                               int32_t hi_k, int32_t hi_end, int64_t *acc, SpanBuf *buf, Tab tab, int lane) {
    const int32_t n_ms = (span_hi - span_lo + kMini - 1) / kMini;
    int64_t carry = INT64_MIN;
    // one block of kMini steps, its four values per lane already in registers
    auto block = [&](int32_t t0, int64_t v0, int64_t v1, int64_t v2, int64_t v3) {
        const int64_t m = max64(max64(v0, v1), max64(v2, v3));
        const int64_t incl = max64(wave_scan_max(m), carry);
        const int64_t excl = from_prev_lane(incl, carry);         // max MF[span_lo .. t0 + 4 lane - 1]
        const int64_t rs = wave_rscan_max(m, lane);               // max MF[t0 + 4 lane .. t0 + 255]
        const int64_t rs_next = from_next_lane(rs, INT64_MIN);    // max MF[t0 + 4 lane + 4 .. t0 + 255]
        carry = last_lane(incl);
        const int64_t piece = lane_value(rs, 0);
        // (the lanes of a wavefront execute in step and LDS serves a wavefront's accesses in
        // order, so the buffer needs no barrier: the fences only pin the compiler's order)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        reinterpret_cast<ll2 *>(buf->raw)[2 * lane] = ll2{v0, v1};
        reinterpret_cast<ll2 *>(buf->raw)[2 * lane + 1] = ll2{v2, v3};
        buf->before[lane] = excl;
        buf->after[lane] = rs_next;
        if (lane == 0) tab[t0 / kMini] = piece;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        for (;;) {                                      // (wave-uniform)
            const int32_t k = lo_k + lane;
            const int32_t o = k < lo_end ? lo_list[k] : INT32_MAX;
            const bool take = o < t0 + kMini;
            if (take) {
                const int32_t r = o - t0, l = r >> 2, j = r & 3;
                int64_t v = max64(buf->before[l], buf->raw[4 * l]);
                if (j >= 1) v = max64(v, buf->raw[4 * l + 1]);
                if (j >= 2) v = max64(v, buf->raw[4 * l + 2]);
                if (j >= 3) v = max64(v, buf->raw[4 * l + 3]);
                atomicMax(reinterpret_cast<long long *>(acc + k), static_cast<long long>(v));
            }
            const int32_t n = __builtin_popcountll(__builtin_amdgcn_ballot_w64(take));
            lo_k += n;
            if (n < 64) break;
        }
        for (;;) {
            const int32_t k = hi_k + lane;
            const int2 it = k < hi_end ? hi_list[k] : make_int2(INT32_MAX, 0);
            const bool take = it.x < t0 + kMini;
            if (take) {
                const int32_t r = it.x - t0, l = r >> 2, j = r & 3;
                int64_t v = max64(buf->after[l], buf->raw[4 * l + 3]);
                if (j <= 2) v = max64(v, buf->raw[4 * l + 2]);
                if (j <= 1) v = max64(v, buf->raw[4 * l + 1]);
                if (j <= 0) v = max64(v, buf->raw[4 * l]);
                atomicMax(reinterpret_cast<long long *>(acc + it.y), static_cast<long long>(v));
            }
            const int32_t n = __builtin_popcountll(__builtin_amdgcn_ballot_w64(take));
            hi_k += n;
            if (n < 64) break;
        }
        __builtin_amdgcn_wave_barrier();
    };
    // Whole groups of kDepth blocks with the next group's blocks requested one group ahead: the row
    // is the only thing this loop reads from global memory, so the wait before a block is used can
    // leave the younger requests in flight.  The blocks left over are taken one at a time.
    const int32_t n_groups = n_ms / kDepth;
    int64_t x[kDepth][4];
#pragma unroll
    for (int d = 0; d < kDepth; ++d) load_quad<kVec, kStream>(MF, span_lo + d * kMini + 4 * lane, a.T, x[d]);
    for (int32_t g = 0; g < n_groups; ++g) {
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
            const int32_t t0 = span_lo + (g * kDepth + d) * kMini;
            const int64_t v0 = x[d][0], v1 = x[d][1], v2 = x[d][2], v3 = x[d][3];
            load_quad<kVec, kStream>(MF, t0 + kDepth * kMini + 4 * lane, a.T, x[d]);
            block(t0, v0, v1, v2, v3);
        }
    }
    for (int32_t ms = n_groups * kDepth; ms < n_ms; ++ms) {
        const int d = ms - n_groups * kDepth;       // the requests after the last whole group are these blocks
        int64_t v[4] = {x[0][0], x[0][1], x[0][2], x[0][3]};
#pragma unroll
        for (int j = 1; j < kDepth; ++j)
            if (d == j) { v[0] = x[j][0]; v[1] = x[j][1]; v[2] = x[j][2]; v[3] = x[j][3]; }
        block(span_lo + ms * kMini, v[0], v[1], v[2], v[3]);
    }
    // tab[k] = max of the pieces k .. end of this span
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    {
        const int32_t k_lo = span_lo / kMini;
        int64_t run = INT64_MIN;
        for (int32_t top = k_lo + n_ms; top > k_lo; top -= 64) {
            const int32_t k = top - 1 - lane;
            const int64_t v = k >= k_lo ? tab[k] : INT64_MIN;
            const int64_t incl = max64(wave_scan_max(v), run);
            run = last_lane(incl);
            if (k >= k_lo) tab[k] = incl;
        }
    }
    return carry;
}

// Phase timing for tuning, compiled in with -DTENSILE_SCORE_PROF only: thread 0 of every
// workgroup adds the 100 MHz ticks it spent in each phase to g_score_prof.
#ifdef TENSILE_SCORE_PROF
__device__ unsigned long long g_score_prof[8 + 2 * 16];   // phases of thread 0; then per wavefront: streaming, cancelling
#define PROF_MARK(k)                                              \
    do {                                                          \
        if (tid == 0) {                                           \
            const unsigned long long now_ = wall_clock64();       \
            atomicAdd(&g_score_prof[k], now_ - prof_t);           \
            prof_t = now_;                                        \
        }                                                         \
    } while (0)
#else
#define PROF_MARK(k) do { } while (0)
#endif

// kBigT: the table of block maxima does not fit in LDS and lives in global scratch.
// kVec: the footprint rows are 16-byte aligned and T is even (two steps per load).
// A load whose address is the same in every lane, from memory that no kernel writes during this
// launch: through the constant address space it goes to the scalar unit and its result lives in
// scalar registers (as a vector load it would hold one register per lane for as long as the value lives).
template <typename T>
__device__ __forceinline__ T uniform_load(const T *p, int64_t i) {
    typedef const T __attribute__((address_space(4))) *const_ptr;
    return ((const_ptr)p)[i];
}

// A 16-byte piece of an output row.  On long rows (kStream: those of more than 131,072 steps) the store is
// nontemporal: the lines are not read again by this kernel, and left out of the L2 they leave it to the
// candidate index and the sub-span maxima (rows of 10^6 steps: 2.58 -> 2.49 ms per batch of 1024 plans; on rows
// of 50,000 steps it costs 5 %, so short rows keep ordinary stores).
template <bool kStream, typename V>
__device__ __forceinline__ void store_out(V *at, const V v) {
    if constexpr (kStream) __builtin_nontemporal_store(v, at);
    else *at = v;
}

// Step 3 of the scoring pass: the plan's own intervals k0 .. k1-1 cancel candidates of the slice
// [slice_lo, slice_lo + n_slice) of a bucket (acc = +inf): an interval inside the gap of an entry of its tensor
// (any interval of that tensor when a.any_interval).  filter: the bucket's bit filter over tensors, in LDS;
// hd: the bucket's {first slot, log2(slots)} in the hash table.
__device__ __forceinline__ void cancel_by_plan(const ScoreArgs &a, const int64_t k0, const int64_t k1, const int2 hd,
                                               const int32_t slice_lo, const int32_t n_slice, const uint32_t *filter, int64_t *acc,
                                               const int tid) {
    const uint32_t fmask = static_cast<uint32_t>(a.filter_words) * 32 - 1;
    const int hshift = 32 - hd.y;
    const uint32_t hmask = (1u << hd.y) - 1;
    const int4 *slots = a.hash_slots + hd.x;
    for (int64_t kb = k0 + tid; kb < k1; kb += kIvU * kThreads) {
        int32_t i[kIvU], o[kIvU], r[kIvU];
        uint32_t h[kIvU];
        int4 s[kIvU];
        bool go[kIvU];
#pragma unroll
        for (int u = 0; u < kIvU; ++u) {
            const int64_t k = kb + u * kThreads;
            const int64_t kc = k < k1 ? k : k1 - 1;
            i[u] = a.iv_tensor[kc];
            o[u] = a.iv_out[kc];
            r[u] = a.iv_in[kc];
            if (k >= k1) i[u] = -1;
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < kIvU; ++u) {
            go[u] = static_cast<uint32_t>(i[u]) < static_cast<uint32_t>(a.N) && o[u] >= 0 && r[u] <= a.T && r[u] > o[u];
            const uint32_t fb = static_cast<uint32_t>(i[u]) & fmask;
            go[u] = go[u] && ((filter[fb >> 5] >> (fb & 31)) & 1u);
            h[u] = go[u] ? (static_cast<uint32_t>(i[u]) * 2654435769u) >> hshift : 0u;
            s[u] = slots[h[u]];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < kIvU; ++u) {
            while (go[u] && s[u].x >= 0) {      // probe until the tensor's last entry or an empty slot
                if (s[u].x == i[u]) {
                    if (a.any_interval || (s[u].y <= o[u] && r[u] <= s[u].z)) {
                        const uint32_t el = static_cast<uint32_t>((s[u].w & INT32_MAX) - slice_lo);
                        if (el < static_cast<uint32_t>(n_slice)) acc[el] = INT64_MAX;
                    }
                    if (s[u].w < 0) break;
                }
                h[u] = (h[u] + 1) & hmask;
                s[u] = slots[h[u]];
            }
        }
    }
}

// LDS of one scoring workgroup.  A struct, so that a kernel that runs other phases in the same workgroup can
// overlay it with theirs.
template <bool kBigT>
struct ScoreLds {
    // (the wavefronts' buffers first: what the streaming loop addresses most sits in the part of the LDS that an
    // instruction's 16-bit offset reaches from a null base)
    __attribute__((aligned(16))) SpanBuf span_buf[kWaves];
    int64_t span_max[kWaves];
    int32_t span_bound[kWaves + 1];  // first step of every wavefront's span in the slice at hand, then T
    int32_t n_compact;               // records written so far (compact mode)
    int64_t tab_lds[kBigT ? 1 : kTabLds];
    int64_t acc[kMaxLocal];
    int32_t lo_list[kMaxLocal];      // o of the slice's entries (its o order is the entries' own order)
    int2 hi_list[kMaxLocal];         // {q, index within the slice} sorted by q
    uint32_t filter[kFilterWords];
    int32_t t_tensor[kMaxLocal];     // tensors of the slice's entries in ascending order ...
    int32_t q_of[kMaxLocal];         // q of entry el (written per plan, read when the rows are composed)
    uint16_t t_el[kMaxLocal];        // ... and the entries' indices within the slice
};

// What a workgroup carries from plan to plan: which bucket's filter and which slice's lists are in LDS (-1:
// none; a caller that has used the LDS for something else in between says so by resetting them).
struct ScoreCarry {
    int32_t filter_of = -1;      // bucket whose filter is in LDS
    int32_t lists_of = -1;       // slice (numbered over all buckets) whose lists are in LDS
#ifdef TENSILE_SCORE_PROF
    unsigned long long prof_t = 0;
#endif
};

// One plan: b with its peak P at step tstar (given by the caller: read from the evaluation's outputs, or taken
// over from an evaluation in the same workgroup).
// kCompact: one plan, records instead of rows (see launch_score); a separate instantiation so that the
// batch kernel carries none of it (with both in one kernel the register allocator spilled once per plan).
template <bool kBigT, bool kVec, bool kCompact>
__device__ __forceinline__ void score_plan(const ScoreArgs &a, const int32_t b, const int32_t tstar, const int64_t P,
                                           ScoreLds<kBigT> &L, int64_t *const tab_global, ScoreCarry &carry) {
    int64_t *const acc = L.acc, *const tab_lds = L.tab_lds, *const span_max = L.span_max;
    int32_t *const lo_list = L.lo_list, *const t_tensor = L.t_tensor, *const q_of = L.q_of, *const span_bound = L.span_bound;
    int2 *const hi_list = L.hi_list;
    uint16_t *const t_el = L.t_el;
    SpanBuf *const span_buf = L.span_buf;
    uint32_t *const filter = L.filter;
    int32_t &n_compact = L.n_compact;
    int32_t &filter_of = carry.filter_of, &lists_of = carry.lists_of;
#ifdef TENSILE_SCORE_PROF
    unsigned long long &prof_t = carry.prof_t;
#endif
    {
        // (the thread index is made opaque once per plan: everything derived from it is then
        // recomputed where it is used instead of being held in registers across the whole loop)
        int tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
        const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int64_t *MF = a.resident + static_cast<int64_t>(b) * a.T;
        int64_t *score = a.score + static_cast<int64_t>(b) * a.N;
        int32_t *wout = a.win_out ? a.win_out + static_cast<int64_t>(b) * a.N : nullptr;
        int32_t *win = a.win_in ? a.win_in + static_cast<int64_t>(b) * a.N : nullptr;

        // ---- 1: output rows.  A bucket that fits one slice gets its rows composed in LDS and written
        // once, in step 4; otherwise they are cleared here and the candidates written over them.
        const bool has_peak = tstar >= 0 && tstar < a.T;     // else not produced by the evaluator: no candidate
        const int32_t bk = has_peak ? tstar >> a.bucket_shift : 0;
        const int32_t e0 = uniform_load(a.bucket_off, bk), n_e = has_peak ? uniform_load(a.bucket_off, bk + 1) - e0 : 0;
        const bool staged = n_e <= kMaxLocal;
        if (kCompact) {                             // (B == 1: one plan per launch)
            if (tid == 0) n_compact = 0;
            if (n_e == 0 && tid == 0) {
                *a.hdr = ScoreHeader{P, tstar, 0};
                if (a.ready) {
                    __threadfence_system();
                    __hip_atomic_store(a.ready, a.ready_value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
                }
            }
        } else if (n_e == 0 || !staged) {
            fill_row<int64_t>(score, a.N, 0, tid);
            if (wout) fill_row<int32_t>(wout, a.N, -1, tid);
            if (win) fill_row<int32_t>(win, a.N, -1, tid);
        }
        if (n_e == 0) return;                      // no gap around t* can be swapped in time
        const int32_t slice0 = uniform_load(a.slice_first, bk);
        const int32_t *hash_dir = reinterpret_cast<const int32_t *>(a.hash_dir);
        const int2 hd = make_int2(uniform_load(hash_dir, 2 * bk), uniform_load(hash_dir, 2 * bk + 1));
        // (the one plan of the compact form is the whole of the interval arrays: its offsets are not read, so a
        // kernel may append to the plan before it calls this)
        int64_t k0 = kCompact ? 0 : uniform_load(a.plan_offsets, b), k1 = kCompact ? a.n_intervals : uniform_load(a.plan_offsets, b + 1);
        if (k0 < 0) k0 = 0;
        if (k1 > a.n_intervals) k1 = a.n_intervals;
        PROF_MARK(0);

        for (int32_t slice_lo = 0; slice_lo < n_e; slice_lo += kMaxLocal) {
            const int32_t n_slice = min(kMaxLocal, n_e - slice_lo);
            const int32_t slice_id = slice0 + slice_lo / kMaxLocal;
            const int32_t *wp = a.wave_ptr + static_cast<int64_t>(slice_id) * 4 * (kWaves + 1);
            // the wavefronts' spans of the row: the slice's own boundaries (multiples of kMini, the last one T),
            // chosen when the index is built so that steps and entries together are spread evenly
            const int span = wave;   // (which wavefront takes which span is free: span_max is indexed by span)
            const int32_t span_lo = uniform_load(wp, 3 * (kWaves + 1) + span), span_hi = uniform_load(wp, 3 * (kWaves + 1) + span + 1);
            __syncthreads();   // the previous plan or slice has finished with acc, tab, span_max, the filter, the lists
            for (int32_t k = tid; k < n_slice; k += kThreads) acc[k] = INT64_MIN;
            if (lists_of != slice_id) {
                for (int32_t k = tid; k < n_slice; k += kThreads) {
                    lo_list[k] = a.cand_o[e0 + slice_lo + k];
                    hi_list[k] = a.qord[e0 + slice_lo + k];
                    const int2 t = a.tord[e0 + slice_lo + k];
                    t_tensor[k] = t.x;
                    t_el[k] = static_cast<uint16_t>(t.y);
                }
                if (tid <= kWaves) span_bound[tid] = wp[3 * (kWaves + 1) + tid];
                lists_of = slice_id;
            }
            if (filter_of != bk) {
                const uint32_t *src = a.filter + static_cast<int64_t>(bk) * a.filter_words;
                for (int32_t k = tid; k < a.filter_words; k += kThreads) filter[k] = src[k];
                filter_of = bk;
            }
            __syncthreads();
            PROF_MARK(1);

            // ---- 2: stream the row.  It comes before the cancelling because its loads are many and independent: they
            // queue behind the output rows of the plan before (stores that are still leaving the CU) and keep the
            // memory pipeline busy from the moment those are gone, whereas the cancelling is a chain of short
            // dependent loads that would only wait there.  The order does not matter to the result: +inf survives
            // every max, and a max that lands before the +inf is overwritten by it; no barrier in between.
#ifdef TENSILE_SCORE_PROF
            const unsigned long long wave_t0 = wall_clock64();
#endif
            {
                const int32_t lo_begin = uniform_load(wp, span), lo_end = uniform_load(wp, span + 1);
                const int32_t hi_begin = uniform_load(wp, kWaves + 1 + span), hi_end = uniform_load(wp, kWaves + 1 + span + 1);
                int64_t m;
                if (kBigT)
                    m = stream_span<kVec, true>(a, MF, span_lo, span_hi, lo_list, hi_list, lo_begin, lo_end, hi_begin, hi_end,
                                                acc, &span_buf[wave], tab_global, lane);
                else
                    m = stream_span<kVec, false>(a, MF, span_lo, span_hi, lo_list, hi_list, lo_begin, lo_end, hi_begin, hi_end,
                                                 acc, &span_buf[wave], tab_lds, lane);
                if (lane == 0) span_max[span] = m;
            }
#ifdef TENSILE_SCORE_PROF
            const unsigned long long wave_t1 = wall_clock64();
            if (lane == 0) atomicAdd(&g_score_prof[8 + wave], wave_t1 - wave_t0);
#endif
            PROF_MARK(2);

            // ---- 3: the plan's own intervals cancel candidates
            cancel_by_plan(a, k0, k1, hd, slice_lo, n_slice, filter, acc, tid);
#ifdef TENSILE_SCORE_PROF
            if (lane == 0) atomicAdd(&g_score_prof[24 + wave], wall_clock64() - wave_t1);
#endif
            PROF_MARK(3);
            __syncthreads();
            PROF_MARK(4);

            // ---- 4: scores of the surviving candidates
            auto final_score = [&](const int4 &c, int64_t sz, int64_t v) -> int64_t {
                const int32_t q = c.y, o = c.z;
                int32_t w_o = 0, w_q = 0;
#pragma unroll
                for (int w = 1; w < kWaves; ++w) {
                    const int32_t bound = span_bound[w];
                    w_o += o >= bound;
                    w_q += q >= bound;
                }
                int64_t m = max64(v, P - sz);
                const int32_t piece = q / kMini + 1;                          // pieces after q's, inside q's span
                if (piece * kMini < span_bound[w_q + 1]) m = max64(m, kBigT ? tab_global[piece] : tab_lds[piece]);
#pragma unroll
                for (int w = 0; w < kWaves; ++w) {
                    const int64_t sm = span_max[w];
                    if (w < w_o || w > w_q) m = max64(m, sm);
                }
                return P - m;
            };
            if (!staged) {
                for (int32_t k = tid; k < n_slice; k += kThreads) {
                    const int32_t e = e0 + slice_lo + k;
                    const int4 c = a.cand[e];
                    const int64_t sz = a.cand_size[e];
                    const int64_t v = acc[k];
                    if (!(c.z < tstar && tstar < c.y) || v == INT64_MAX) continue;
                    if (kCompact) {
                        a.compact[atomicAdd(&n_compact, 1)] = ScoreCand{final_score(c, sz, v), c.w, c.z, c.y, -1};
                        continue;
                    }
                    score[c.w] = final_score(c, sz, v);
                    if (wout) wout[c.w] = c.z;
                    if (win) win[c.w] = c.y;
                }
            } else {
                // The scores first, entry by entry (in place: acc becomes the score, or -inf for an entry
                // without output).  Then every wavefront composes the output of its own range of tensors,
                // kScoreStage at a time, in its LDS buffer (scores, then the two windows) and writes whole
                // pieces of the rows, so that each output line goes to memory once.  The entries in tensor
                // order, their o and q are all in LDS: this part reads nothing from global memory, and no
                // wait for a load ever holds back the stores queued before it.
                if (kCompact) {
                    for (int32_t k = tid; k < n_e; k += kThreads) {
                        const int4 c = a.cand[e0 + k];
                        const int64_t sz = a.cand_size[e0 + k];
                        const int64_t v = acc[k];
                        if (c.z < tstar && tstar < c.y && v != INT64_MAX)
                            a.compact[atomicAdd(&n_compact, 1)] = ScoreCand{final_score(c, sz, v), c.w, c.z, c.y, -1};
                    }
                    continue;   // (block-uniform; a staged bucket is one slice: this ends the slice loop)
                }
                for (int32_t k = tid; k < n_e; k += kThreads) {
                    const int4 c = a.cand[e0 + k];
                    const int64_t sz = a.cand_size[e0 + k];
                    const int64_t v = acc[k];
                    acc[k] = (c.z < tstar && tstar < c.y && v != INT64_MAX) ? final_score(c, sz, v) : INT64_MIN;
                    q_of[k] = c.y;
                }
                __syncthreads();
                int64_t *st_score = reinterpret_cast<int64_t *>(&span_buf[wave]);
                int32_t *st_wo = reinterpret_cast<int32_t *>(st_score + kScoreStage), *st_wi = st_wo + kScoreStage;
                int32_t tk = wp[2 * (kWaves + 1) + wave];
                const bool wide = ((reinterpret_cast<uintptr_t>(score) | reinterpret_cast<uintptr_t>(wout) |
                                    reinterpret_cast<uintptr_t>(win)) & 15) == 0;
                const int32_t t_end = min((wave + 1) * a.tspan, a.N);
                for (int32_t t0 = wave * a.tspan; t0 < t_end; t0 += kScoreStage) {
                    const int32_t n_t = min(kScoreStage, a.N - t0);
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
#pragma unroll
                    for (int j = 0; j < 3; ++j) {       // 192 vectors of 16 bytes: 96 of scores (0), 96 of windows (-1)
                        const int v = j * 64 + lane;
                        reinterpret_cast<ll2 *>(st_score)[v] = v < kScoreStage / 2 ? ll2{0, 0} : ll2{-1, -1};
                    }
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    for (;;) {                                  // (wave-uniform)
                        const int32_t k = tk + lane;
                        const int32_t tensor = k < n_e ? t_tensor[k] : INT32_MAX;
                        const bool take = tensor < t0 + kScoreStage;
                        if (take) {
                            const int32_t el = t_el[k];
                            const int64_t v = acc[el];
                            if (v != INT64_MIN) {
                                st_score[tensor - t0] = v;
                                st_wo[tensor - t0] = lo_list[el];
                                st_wi[tensor - t0] = q_of[el];
                            }
                        }
                        const int32_t n = __builtin_popcountll(__builtin_amdgcn_ballot_w64(take));
                        tk += n;
                        if (n < 64) break;
                    }
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    if (wide) {
                        typedef int i4 __attribute__((ext_vector_type(4)));
#pragma unroll
                        for (int j = 0; j < 2; ++j) {
                            const int v = j * 64 + lane;            // two scores per vector
                            if (2 * v + 1 < n_t) store_out<kBigT>(reinterpret_cast<ll2 *>(score + t0) + v, reinterpret_cast<const ll2 *>(st_score)[v]);
                            else if (2 * v < n_t) score[t0 + 2 * v] = st_score[2 * v];
                        }
                        if (lane < kScoreStage / 4) {               // four window values per vector
                            if (4 * lane + 3 < n_t) {
                                if (wout) store_out<kBigT>(reinterpret_cast<i4 *>(wout + t0) + lane, reinterpret_cast<const i4 *>(st_wo)[lane]);
                                if (win) store_out<kBigT>(reinterpret_cast<i4 *>(win + t0) + lane, reinterpret_cast<const i4 *>(st_wi)[lane]);
                            } else {
                                for (int32_t k = 4 * lane; k < n_t; ++k) {
                                    if (wout) wout[t0 + k] = st_wo[k];
                                    if (win) win[t0 + k] = st_wi[k];
                                }
                            }
                        }
                    } else {
#pragma unroll
                        for (int j = 0; j < kScoreStage / 64; ++j) {
                            const int32_t k = j * 64 + lane;
                            if (k < n_t) {
                                score[t0 + k] = st_score[k];
                                if (wout) wout[t0 + k] = st_wo[k];
                                if (win) win[t0 + k] = st_wi[k];
                            }
                        }
                    }
                }
            }
            PROF_MARK(5);
        }
        if (kCompact) {
            if (a.ready) __threadfence_system();   // this thread's records, before the barrier that precedes the signal
            __syncthreads();
            if (tid == 0) {
                *a.hdr = ScoreHeader{P, tstar, n_compact};
                if (a.ready) {
                    __threadfence_system();
                    __hip_atomic_store(a.ready, a.ready_value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
                }
            }
        }
    }
}

// Persistent workgroups: workgroup w takes the plans w, w + grid, ...
template <bool kBigT, bool kVec, bool kCompact>
__global__ __launch_bounds__(kThreads) void score_kernel(const ScoreArgs a) {
    __shared__ ScoreLds<kBigT> lds;
    int64_t *tab_global = kBigT ? a.tab_scratch + static_cast<int64_t>(blockIdx.x) * a.n_tab : nullptr;
    ScoreCarry carry;
#ifdef TENSILE_SCORE_PROF
    carry.prof_t = wall_clock64();
#endif
    for (int32_t b = blockIdx.x; b < a.B; b += gridDim.x)
        score_plan<kBigT, kVec, kCompact>(a, b, uniform_load(a.argmax, b), uniform_load(a.peak, b), lds, tab_global, carry);
}

// (host) the arguments of a dense scoring pass; scratch table and compact outputs are left null
inline ScoreArgs make_score_args(const tensile_tas *tas, const CandIndex &ix, bool any_interval, const tensile_plans *plans,
                                 const int64_t *resident, const int64_t *peak, const int32_t *argmax, int64_t *score,
                                 int32_t *win_out, int32_t *win_in) {
    ScoreArgs a;
    a.T = tas->T; a.N = tas->N; a.B = plans->B;
    a.tspan = ix.tspan;
    a.n_tab = (tas->T + kMini - 1) / kMini;
    a.vec16 = (tas->T % 2 == 0) && (reinterpret_cast<uintptr_t>(resident) % 16 == 0);
    a.any_interval = any_interval ? 1 : 0;
    a.n_intervals = plans->n_intervals;
    a.plan_offsets = plans->plan_offsets;
    a.iv_tensor = plans->iv_tensor; a.iv_out = plans->iv_out; a.iv_in = plans->iv_in;
    a.bucket_shift = ix.shift; a.filter_words = ix.filter_words;
    a.bucket_off = ix.bucket_off.p;
    a.cand = ix.cand.p; a.cand_size = ix.cand_size.p; a.cand_o = ix.cand_o.p; a.cand_gap = ix.cand_gap.p; a.qord = ix.qord.p; a.tord = ix.tord.p;
    a.slice_first = ix.slice_first.p; a.wave_ptr = ix.wave_ptr.p; a.hash_dir = ix.hash_dir.p; a.hash_slots = ix.hash_slots.p; a.filter = ix.filter.p;
    a.resident = resident; a.peak = peak; a.argmax = argmax;
    a.score = score; a.win_out = win_out; a.win_in = win_in;
    a.tab_scratch = nullptr;
    a.hdr = nullptr; a.compact = nullptr;
    a.ready = nullptr; a.ready_value = 0;
    return a;
}

}  // namespace

}  // namespace tensile
