// Candidate scoring (section IV-C of the paper): for every plan, how much would
// evicting each tensor that is resident and idle at the peak lower the peak,
// given the earliest swap-out / latest swap-in the host link's speed allows.
//
// score = P - max( max MF[0..o], max MF[q..T), P - size ) needs running maxima of
// the plan's footprint row at scattered positions (o, q).  Writing a full row of
// running maxima would double the traffic of the pass, so the maxima are kept at
// a granularity of kChunk = 8 steps (one 64-byte line of the row).  The row is
// cut into one contiguous span of chunks per wavefront, and inside its span each
// wavefront computes, with wave-level scans only (no workgroup barrier):
//   CM[c]  = max MF[8c .. 8c+7]
//   PMC[c] = max of CM over the chunks of the span up to and including c
//   SMC[c] = max of CM over the chunks of the span from c on
// plus the maximum of the whole span, left in LDS.  A query combines a table
// entry with the span maxima of the other wavefronts and finishes inside its own
// chunk by reading that one line of the row:
//   max MF[0..o]  = max( PMC[(o>>3)-1], spans before that chunk's, MF[8(o>>3) .. o] )
//   max MF[q..T)  = max( SMC[(q>>3)+1], spans after that chunk's,  MF[q .. 8(q>>3)+7] )
// The tables live in a scratch area owned by the workgroup (3*T bytes), which
// stays in L2 / the memory-side cache for the configurations at hand.
//
// Which tensors can be candidates at a peak step t* does not depend on the plan:
// they are the gaps (p, q) of the TAS with a feasible earliest swap-out step o
// (a property of the gap alone: it follows from p, q, the transfer time and the
// cumulative latency) and o < t* < q.  tensile_tas_load files every such gap,
// as {p, q, o, tensor}, under each bucket of 2^shift steps that (o, q) overlaps,
// so a plan looks at the one bucket of its t* instead of all gaps.
//
// One workgroup walks a plan at a time (persistent workgroups, plans dealt
// round-robin):
//   1. the plan's output rows are cleared (score 0, windows -1);
//   2. chunk tables as above;
//   3. every entry of the bucket with o < t* < q puts its index into map[tensor]
//      (a per-workgroup array over tensors, -1 elsewhere);
//   4. the plan's own intervals look their tensor up in the map; an interval
//      inside the candidate gap of its tensor cancels the candidate (map = -2):
//      "tensor has not been swapped out" in the paper's Alg. 2;
//   5. the bucket is walked again: surviving candidates get their score, and every
//      touched map entry is reset to -1 for the next plan.
// No search is needed anywhere: a tensor has at most one gap around t*.
#include "common.h"
#include "wave_ops.h"

namespace tensile {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kChunk = 8;       // steps per chunk = one 64-byte line
constexpr int kFwdU = 4;        // chunks per lane and round of the forward pass
constexpr int kBwdU = 8;        // chunk maxima per lane and round of the backward pass
constexpr int kIvU = 4;         // intervals per thread and round

typedef long long ll2 __attribute__((ext_vector_type(2)));

struct ScoreArgs {
    int32_t T, N, B;
    int32_t n_chunks;            // ceil(T / kChunk)
    int32_t chunks_per_wave;     // span of one wavefront, a multiple of 64
    int64_t n_intervals;
    const int64_t *plan_offsets;
    const int32_t *iv_tensor, *iv_out, *iv_in;
    const int64_t *size;
    const int4 *cand;            // bucketed candidate gaps {p, q, o, tensor}
    const int64_t *cand_size;    // size of each entry's tensor
    const int32_t *bucket_off;   // [n_buckets + 1] into cand
    int32_t bucket_shift;
    const int64_t *resident;
    const int64_t *peak;
    const int32_t *argmax;
    int64_t *score;
    int32_t *win_out, *win_in;
    int64_t *tables;             // [gridDim.x][3][n_chunks]: CM, PMC, SMC of the plan in progress
    int32_t *map;                // [gridDim.x][N]: candidate entry of each tensor for the plan in progress
    int32_t vec16;               // rows are 16-byte aligned (T even, aligned base)
};

// row[0..n) = v with 16-byte stores where the row allows them
template <typename E>
__device__ __forceinline__ void fill_row(E *row, int32_t n, E v) {
    constexpr int kPer = 16 / sizeof(E);
    typedef E vec_t __attribute__((ext_vector_type(kPer)));
    const int tid = threadIdx.x;
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

// Two consecutive steps of the row starting at the even step t (one 16-byte load when the row
// allows it); steps outside [0, T) and masked-off lanes give INT64_MIN.  The load itself is
// always issued, at a clamped address, so that a batch of them can be in flight together.
template <bool kVec>
__device__ __forceinline__ void load_pair(const int64_t *MF, int32_t t, int32_t T, int64_t &x0, int64_t &x1) {
    if (kVec) {   // T is even here, so t < T implies t + 1 < T
        const ll2 x = *reinterpret_cast<const ll2 *>(MF + (t < T ? t : T - 2));
        x0 = x[0];
        x1 = x[1];
    } else {
        x0 = MF[t < T ? t : T - 1];
        x1 = MF[t + 1 < T ? t + 1 : T - 1];
    }
}

// max over the four lanes of each quad, left in all four
__device__ __forceinline__ int64_t quad_max(int64_t x) {
    x = max64(x, dpp_move<0xB1, 0xf>(x, x));   // quad_perm:[1,0,3,2]
    x = max64(x, dpp_move<0x4E, 0xf>(x, x));   // quad_perm:[2,3,0,1]
    return x;
}

__device__ __forceinline__ int64_t permute64(int64_t x, int src_lane) {
    const int lo = __builtin_amdgcn_ds_bpermute(src_lane << 2, static_cast<int>(x));
    const int hi = __builtin_amdgcn_ds_bpermute(src_lane << 2, static_cast<int>(x >> 32));
    return (static_cast<int64_t>(hi) << 32) | static_cast<uint32_t>(lo);
}

// The chunk tables of one wavefront's span [lo, hi) of the row MF; returns the span's maximum.
// A load instruction covers 128 consecutive steps (lane l: steps 2l, 2l+1), i.e. 16 chunks with
// one chunk per quad of lanes; four of them give 64 chunk maxima, which a lane permutation puts
// into chunk order for one wave-level scan and full-width stores.
template <bool kVec>
__device__ __forceinline__ int64_t span_tables(const ScoreArgs &a, const int64_t *MF, int64_t *CM, int64_t *PMC,
                                               int32_t lo, int32_t hi) {
    const int lane = threadIdx.x & 63;
    const int in_order = ((lane & 15) << 2) | (lane >> 4);   // lane holding the maximum of chunk base + lane
    int64_t carry = INT64_MIN;
    for (int32_t base = lo; base < hi; base += 64 * kFwdU) {
        int64_t x[kFwdU][4][2];
#pragma unroll
        for (int u = 0; u < kFwdU; ++u) {
            if (base + u * 64 >= hi) break;     // (wave-uniform)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                load_pair<kVec>(MF, (base + u * 64 + j * 16) * kChunk + 2 * lane, a.T, x[u][j][0], x[u][j][1]);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < kFwdU; ++u) {
            if (base + u * 64 >= hi) break;
            int64_t keep = INT64_MIN;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int32_t t = (base + u * 64 + j * 16) * kChunk + 2 * lane;
                int64_t m = INT64_MIN;
                if (t < a.T) m = x[u][j][0];
                if (t + 1 < a.T) m = max64(m, x[u][j][1]);
                m = quad_max(m);
                if ((lane & 3) == j) keep = m;      // chunk base + 64u + 16j + (lane >> 2)
            }
            const int32_t c = base + u * 64 + lane;
            const int64_t ordered = permute64(keep, in_order);
            const int64_t m = c < hi ? ordered : INT64_MIN;
            const int64_t incl = max64(wave_scan_max(m), carry);
            carry = last_lane(incl);
            if (c < hi) {
                CM[c] = m;
                PMC[c] = incl;
            }
        }
    }
    return carry;
}

// SMC over the span [lo, hi) from the chunk maxima CM
__device__ __forceinline__ void span_suffix(const int64_t *CM, int64_t *SMC, int32_t lo, int32_t hi) {
    const int lane = threadIdx.x & 63;
    int64_t carry = INT64_MIN;
    for (int32_t top = hi; top > lo; top -= 64 * kBwdU) {
        int64_t m[kBwdU];
#pragma unroll
        for (int u = 0; u < kBwdU; ++u) {
            if (top - u * 64 <= lo) break;          // (wave-uniform)
            const int32_t c = top - 1 - (u * 64 + lane);
            m[u] = CM[c >= lo ? c : lo];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < kBwdU; ++u) {
            if (top - u * 64 <= lo) break;
            const int32_t c = top - 1 - (u * 64 + lane);
            const int64_t incl = max64(wave_scan_max(c >= lo ? m[u] : INT64_MIN), carry);
            carry = last_lane(incl);
            if (c >= lo) SMC[c] = incl;
        }
    }
}

// Phase timing for tuning, compiled in with -DTENSILE_SCORE_PROF only: thread 0 of every
// workgroup adds the 100 MHz ticks it spent in each phase to g_score_prof.
#ifdef TENSILE_SCORE_PROF
__device__ unsigned long long g_score_prof[8];
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

__global__ __launch_bounds__(kThreads) void score_kernel(const ScoreArgs a) {
    __shared__ int64_t span_max[kWaves];
    const int tid = threadIdx.x, wave = tid >> 6;
    int64_t *CM = a.tables + static_cast<int64_t>(blockIdx.x) * 3 * a.n_chunks;
    int64_t *PMC = CM + a.n_chunks, *SMC = PMC + a.n_chunks;
    int32_t *map = a.map + static_cast<int64_t>(blockIdx.x) * a.N;
    const int32_t span_lo = min(wave * a.chunks_per_wave, a.n_chunks);
    const int32_t span_hi = min(span_lo + a.chunks_per_wave, a.n_chunks);

    fill_row<int32_t>(map, a.N, -1);
#ifdef TENSILE_SCORE_PROF
    unsigned long long prof_t = wall_clock64();
#endif

    for (int32_t b = blockIdx.x; b < a.B; b += gridDim.x) {
        const int32_t tstar = a.argmax[b];
        const int64_t P = a.peak[b];
        const int64_t *MF = a.resident + static_cast<int64_t>(b) * a.T;
        int64_t *score = a.score + static_cast<int64_t>(b) * a.N;
        int32_t *wout = a.win_out ? a.win_out + static_cast<int64_t>(b) * a.N : nullptr;
        int32_t *win = a.win_in ? a.win_in + static_cast<int64_t>(b) * a.N : nullptr;

        // ---- 1: clear the output rows (independent of everything else)
        fill_row<int64_t>(score, a.N, 0);
        if (wout) fill_row<int32_t>(wout, a.N, -1);
        if (win) fill_row<int32_t>(win, a.N, -1);
        __syncthreads();   // the previous plan has finished with the tables, the map and span_max
        PROF_MARK(0);
        if (tstar < 0 || tstar >= a.T) continue;   // not produced by the evaluator: no candidate
        const int32_t bk = tstar >> a.bucket_shift;
        const int32_t e0 = a.bucket_off[bk], e1 = a.bucket_off[bk + 1];
        if (e0 == e1) continue;                    // no gap around t* can be swapped in time

        // ---- 2: chunk tables of this wavefront's span
        {
            const int64_t m = a.vec16 ? span_tables<true>(a, MF, CM, PMC, span_lo, span_hi)
                                      : span_tables<false>(a, MF, CM, PMC, span_lo, span_hi);
            if ((tid & 63) == 0) span_max[wave] = m;
        }
        PROF_MARK(1);
        // ---- 3: candidate entries -> map[tensor]
        for (int32_t e = e0 + tid; e < e1; e += kThreads) {
            const int4 c = a.cand[e];
            if (c.z < tstar && tstar < c.y) map[c.w] = e;
        }
        __syncthreads();   // CM, the map and span_max are complete
        PROF_MARK(2);
        span_suffix(CM, SMC, span_lo, span_hi);
        PROF_MARK(3);

        // ---- 4: the plan's own intervals cancel candidates
        int64_t k0 = a.plan_offsets[b], k1 = a.plan_offsets[b + 1];
        if (k0 < 0) k0 = 0;
        if (k1 > a.n_intervals) k1 = a.n_intervals;
        for (int64_t kb = k0 + tid; kb < k1; kb += kIvU * kThreads) {
            int32_t i[kIvU], o[kIvU], r[kIvU], e[kIvU];
            int4 c[kIvU];
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
                const bool ok = static_cast<uint32_t>(i[u]) < static_cast<uint32_t>(a.N) && o[u] >= 0 && r[u] <= a.T && r[u] > o[u];
                e[u] = map[ok ? i[u] : 0];
                if (!ok) e[u] = -1;
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < kIvU; ++u) {
                if (e[u] < e0 || e[u] >= e1) e[u] = -1;     // nothing, cancelled, or left by an earlier plan
                c[u] = a.cand[e[u] >= 0 ? e[u] : e0];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < kIvU; ++u)
                if (e[u] >= 0 && c[u].x <= o[u] && r[u] <= c[u].y) map[i[u]] = -2;   // all writers write the same value
        }
        __syncthreads();   // the map and SMC are complete
        PROF_MARK(4);

        // ---- 5: scores of the surviving candidates.  A wavefront takes 64 entries at a time:
        // one entry per lane for the table lookups, then, 16 entries at a time, one entry per
        // quad of lanes for the two 64-byte lines of the row around o and q.
        {
            // maxima of the spans before / after each wavefront's
            int64_t before[kWaves], after[kWaves];
            int64_t run = INT64_MIN;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                before[w] = run;
                run = max64(run, span_max[w]);
            }
            run = INT64_MIN;
#pragma unroll
            for (int w = kWaves - 1; w >= 0; --w) {
                after[w] = run;
                run = max64(run, span_max[w]);
            }
            const int lane = tid & 63;
            for (int32_t eb = e0 + wave * 64; eb < e1; eb += kThreads) {   // (wave-uniform)
                const int32_t e = eb + lane;
                const int32_t ec = e < e1 ? e : e1 - 1;
                const int4 c = a.cand[ec];
                const int32_t q = c.y, o = c.z, i = c.w;
                const int32_t co = o >> 3, cq = q >> 3;
                const int32_t cp = co > 0 ? co - 1 : 0, cs = cq + 1 < a.n_chunks ? cq + 1 : a.n_chunks - 1;
                // every operand is requested before the first is used
                const int32_t owner = map[i];
                const int64_t sz = a.cand_size[ec];
                const int64_t pm = PMC[cp], sm = SMC[cs];
                const bool alive = e < e1 && o < tstar && tstar < q && owner == e;
                const int32_t o_or_none = alive ? o : -1;
                int64_t lines = INT64_MIN;        // max( MF[8co .. o], MF[q .. 8cq+7] ) of this lane's entry
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int src = 16 * r + (lane >> 2);
                    const int32_t o_s = __builtin_amdgcn_ds_bpermute(src << 2, o_or_none);
                    const int32_t q_s = __builtin_amdgcn_ds_bpermute(src << 2, q);
                    int64_t m = INT64_MIN;
                    if (o_s >= 0) {
                        const int32_t t0 = (o_s >> 3) * kChunk + 2 * (lane & 3), t1 = (q_s >> 3) * kChunk + 2 * (lane & 3);
                        int64_t x0, x1, y0, y1;
                        if (a.vec16) {
                            load_pair<true>(MF, t0, a.T, x0, x1);
                            load_pair<true>(MF, t1, a.T, y0, y1);
                        } else {
                            load_pair<false>(MF, t0, a.T, x0, x1);
                            load_pair<false>(MF, t1, a.T, y0, y1);
                        }
                        if (t0 <= o_s) m = max64(m, x0);                     // t0 <= o < T
                        if (t0 + 1 <= o_s) m = max64(m, x1);
                        if (t1 >= q_s && t1 < a.T) m = max64(m, y0);
                        if (t1 + 1 >= q_s && t1 + 1 < a.T) m = max64(m, y1);
                    }
                    m = quad_max(m);
                    const int64_t back = permute64(m, (lane & 15) << 2);   // quad (lane & 15) of round lane >> 4
                    if ((lane >> 4) == r) lines = back;
                }
                if (alive) {
                    int64_t m = max64(P - sz, lines);
                    if (co > 0) {      // whole chunks before o's chunk: this span's, then the earlier spans
                        int64_t x = pm;
                        const int32_t w = cp / a.chunks_per_wave;
#pragma unroll
                        for (int k = 0; k < kWaves; ++k)
                            if (k == w) x = max64(x, before[k]);
                        m = max64(m, x);
                    }
                    if (cq + 1 < a.n_chunks) {
                        int64_t x = sm;
                        const int32_t w = cs / a.chunks_per_wave;
#pragma unroll
                        for (int k = 0; k < kWaves; ++k)
                            if (k == w) x = max64(x, after[k]);
                        m = max64(m, x);
                    }
                    score[i] = P - m;
                    if (wout) wout[i] = o;
                    if (win) win[i] = q;
                }
            }
        }
        PROF_MARK(5);
    }
}

}  // namespace

int launch_score(const tensile_tas *tas, const tensile_plans *plans, const int64_t *resident, const int64_t *peak,
                 const int32_t *argmax, int64_t *score, int32_t *win_out, int32_t *win_in, hipStream_t stream) {
    if (plans->B == 0 || tas->N == 0) return TENSILE_OK;
    // as many workgroups as the device keeps resident, the plans dealt evenly among them
    static int per_cu = 0;
    if (per_cu == 0) {
        int n = 0;
        TS_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, score_kernel, kThreads, 0));
        per_cu = n > 0 ? n : 1;
    }
    const int64_t resident_blocks = static_cast<int64_t>(tas->num_cus) * per_cu;
    const int64_t rounds = (plans->B + resident_blocks - 1) / resident_blocks;
    const int32_t blocks = static_cast<int32_t>((plans->B + rounds - 1) / rounds);
    const int32_t n_chunks = (tas->T + kChunk - 1) / kChunk;
    Scratch &sc = tas->scratch;
    const size_t need = static_cast<size_t>(blocks) * 3 * static_cast<size_t>(n_chunks);
    const size_t need_map = static_cast<size_t>(blocks) * static_cast<size_t>(tas->N);
    if (sc.rowmax.n < need || sc.cand_map.n < need_map) {
        TS_HIP(hipDeviceSynchronize());
        TS_HIP(sc.rowmax.reserve(need));
        TS_HIP(sc.cand_map.reserve(need_map));
    }
    ScoreArgs a;
    a.T = tas->T; a.N = tas->N; a.B = plans->B;
    a.n_chunks = n_chunks;
    a.chunks_per_wave = (n_chunks + kWaves * 64 - 1) / (kWaves * 64) * 64;
    a.n_intervals = plans->n_intervals;
    a.plan_offsets = plans->plan_offsets;
    a.iv_tensor = plans->iv_tensor; a.iv_out = plans->iv_out; a.iv_in = plans->iv_in;
    a.size = tas->d_size.p;
    a.cand = tas->d_cand.p; a.cand_size = tas->d_cand_size.p; a.bucket_off = tas->d_bucket_off.p; a.bucket_shift = tas->bucket_shift;
    a.resident = resident; a.peak = peak; a.argmax = argmax;
    a.score = score; a.win_out = win_out; a.win_in = win_in;
    a.tables = sc.rowmax.p;
    a.map = sc.cand_map.p;
    a.vec16 = (tas->T % 2 == 0) && (reinterpret_cast<uintptr_t>(resident) % 16 == 0);
    hipLaunchKernelGGL(score_kernel, dim3(blocks), dim3(kThreads), 0, stream, a);
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
