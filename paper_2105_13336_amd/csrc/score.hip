// Candidate scoring (section IV-C of the paper): for every plan, how much would
// evicting each tensor that is resident and idle at the peak lower the peak,
// given the earliest swap-out / latest swap-in the host link's speed allows.
//
// score = P - max( max MF[0..o], max MF[q..T), P - size ) needs running maxima of
// the plan's footprint row at scattered positions (o, q).  Writing a full row of
// running maxima would double the traffic of the pass, so the maxima are kept at
// a granularity of kChunk = 8 steps (one 64-byte line of the row):
//   PMC[c] = max MF[0 .. 8c+7]      (prefix, by chunk)
//   SMC[c] = max MF[8c .. T)        (suffix, by chunk)
// and a query finishes inside its own chunk by reading that one line of the row:
//   max MF[0..o]  = max( PMC[(o>>3)-1], max MF[8(o>>3) .. o] )
//   max MF[q..T)  = max( SMC[(q>>3)+1], max MF[q .. 8(q>>3)+7] )
// Neither table depends on the peak step.  Both live in a scratch area owned by
// the workgroup (2*T bytes instead of 8*T), which stays in L2 / the memory-side
// cache for the configurations at hand.
//
// One workgroup walks a plan at a time (persistent workgroups, plans dealt
// round-robin):
//   1. forward over the row: chunk maxima CM and PMC; backward over CM: SMC;
//   2. the plan's output rows are cleared (score 0, windows -1);
//   3. every gap (p, q) of the TAS with p < t* < q whose precomputed earliest
//      swap-out step o (a property of the gap alone: it depends on p, q, the
//      transfer time and the cumulative latency, not on the plan) lies before t*
//      is a candidate: its index goes into map[tensor] (a per-workgroup array over
//      tensors, -1 elsewhere) and onto a list in LDS;
//   4. the plan's own intervals look their tensor up in the map; an interval
//      inside the candidate gap of its tensor cancels the candidate (map = -2):
//      "tensor has not been swapped out" in the paper's Alg. 2;
//   5. the surviving candidates get their score, and every touched map entry is
//      reset to -1 for the next plan.
// No search is needed anywhere: a tensor has at most one gap around t*.
#include "common.h"
#include "wave_ops.h"

namespace tensile {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kChunk = 8;                          // steps per chunk = one 64-byte line
constexpr int kListCap = 4096;                     // candidate gaps kept in LDS (16 KB); more -> rescan

typedef long long ll2 __attribute__((ext_vector_type(2)));

struct ScoreArgs {
    int32_t T, N, B, G;
    int32_t n_chunks;            // ceil(T / kChunk)
    int64_t n_intervals;
    const int64_t *plan_offsets;
    const int32_t *iv_tensor, *iv_out, *iv_in;
    const int64_t *size;
    const int32_t *gp, *gq, *gtensor, *gwin;   // [G] gaps of length >= 2, in tensor order
    const int64_t *resident;
    const int64_t *peak;
    const int32_t *argmax;
    int64_t *score;
    int32_t *win_out, *win_in;
    int64_t *tables;             // [gridDim.x][3][n_chunks]: CM, PMC, SMC of the plan in progress
    int32_t *map;                // [gridDim.x][N]: candidate gap of each tensor for the plan in progress
    int32_t vec16;               // rows are 16-byte aligned (T even, aligned base)
};

// Block-wide inclusive max-scan step: `m` is this thread's value, threads in scan order.
// Returns the inclusive maximum including `carry` (the maximum of everything before this
// round) and updates `carry`.  wave_tot is a double buffer indexed by `buf`.
__device__ __forceinline__ int64_t block_scan_max(int64_t m, int64_t &carry, int64_t (*wave_tot)[kWaves], int &buf) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t incl = wave_scan_max(m);
    if (lane == 63) wave_tot[buf][wave] = incl;
    __syncthreads();
    int64_t pre = carry;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const int64_t tw = wave_tot[buf][w];
        if (w < wave) pre = max64(pre, tw);
        carry = max64(carry, tw);
    }
    buf ^= 1;
    return max64(incl, pre);
}

__device__ __forceinline__ bool is_candidate(const ScoreArgs &a, int32_t g, int32_t tstar) {
    const int32_t p = a.gp[g], q = a.gq[g];
    if (!(p < tstar && tstar < q)) return false;
    const int32_t o = a.gwin[g];
    return o >= 0 && o < tstar;
}

__global__ __launch_bounds__(kThreads) void score_kernel(const ScoreArgs a) {
    __shared__ int32_t list[kListCap];
    __shared__ int32_t list_n;
    __shared__ int64_t wave_tot[2][kWaves];
    const int tid = threadIdx.x;
    int64_t *CM = a.tables + static_cast<int64_t>(blockIdx.x) * 3 * a.n_chunks;
    int64_t *PMC = CM + a.n_chunks, *SMC = PMC + a.n_chunks;
    int32_t *map = a.map + static_cast<int64_t>(blockIdx.x) * a.N;

    for (int32_t i = tid; i < a.N; i += kThreads) map[i] = -1;

    for (int32_t b = blockIdx.x; b < a.B; b += gridDim.x) {
        const int32_t tstar = a.argmax[b];
        const int64_t P = a.peak[b];
        const int64_t *MF = a.resident + static_cast<int64_t>(b) * a.T;
        int64_t *score = a.score + static_cast<int64_t>(b) * a.N;
        int32_t *wout = a.win_out ? a.win_out + static_cast<int64_t>(b) * a.N : nullptr;
        int32_t *win = a.win_in ? a.win_in + static_cast<int64_t>(b) * a.N : nullptr;

        // ---- 2: clear the output rows (independent of everything else)
        for (int32_t i = tid; i < a.N; i += kThreads) {
            score[i] = 0;
            if (wout) wout[i] = -1;
            if (win) win[i] = -1;
        }
        __syncthreads();   // the previous plan has finished with the tables and the list
        if (tid == 0) list_n = 0;   // (read again only after further barriers)
        if (tstar < 0 || tstar >= a.T) continue;   // not produced by the evaluator: no candidate

        // ---- 1a: forward, one chunk (8 steps, 64 bytes) per thread and round; the next round's
        // line is requested before this round's block-wide scan
        {
            int64_t carry = INT64_MIN;
            int buf = 0;
            auto load_chunk = [&](int32_t c, int64_t (&v)[kChunk]) {
                const int32_t t0 = c * kChunk;
                if (c < a.n_chunks && a.vec16 && t0 + kChunk <= a.T) {
                    const ll2 *src = reinterpret_cast<const ll2 *>(MF + t0);
#pragma unroll
                    for (int j = 0; j < kChunk / 2; ++j) {
                        const ll2 x = src[j];
                        v[2 * j] = x[0];
                        v[2 * j + 1] = x[1];
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < kChunk; ++j) v[j] = (c < a.n_chunks && t0 + j < a.T) ? MF[t0 + j] : INT64_MIN;
                }
            };
            int64_t cur[kChunk], nxt[kChunk];
            load_chunk(tid, cur);
            for (int32_t c0 = 0; c0 < a.n_chunks; c0 += kThreads) {
                const int32_t c = c0 + tid;
                load_chunk(c + kThreads, nxt);
                int64_t m = cur[0];
#pragma unroll
                for (int j = 1; j < kChunk; ++j) m = max64(m, cur[j]);
                const int64_t incl = block_scan_max(m, carry, wave_tot, buf);
                if (c < a.n_chunks) {
                    CM[c] = m;
                    PMC[c] = incl;
                }
#pragma unroll
                for (int j = 0; j < kChunk; ++j) cur[j] = nxt[j];
            }
        }
        __syncthreads();   // CM complete
        // ---- 1b: backward over the chunk maxima
        {
            int64_t carry = INT64_MIN;
            int buf = 0;
            for (int32_t r0 = 0; r0 < a.n_chunks; r0 += kThreads) {
                const int32_t r = r0 + tid;                    // position in reverse order
                const int32_t c = a.n_chunks - 1 - r;
                const int64_t m = r < a.n_chunks ? CM[c] : INT64_MIN;
                const int64_t incl = block_scan_max(m, carry, wave_tot, buf);
                if (r < a.n_chunks) SMC[c] = incl;
            }
        }

        // ---- 3: candidate gaps -> map[tensor] and the list
        for (int32_t g = tid; g < a.G; g += kThreads) {
            if (!is_candidate(a, g, tstar)) continue;
            map[a.gtensor[g]] = g;
            const int32_t slot = atomicAdd(&list_n, 1);
            if (slot < kListCap) list[slot] = g;
        }
        __syncthreads();

        // ---- 4: the plan's own intervals cancel candidates
        int64_t k0 = a.plan_offsets[b], k1 = a.plan_offsets[b + 1];
        if (k0 < 0) k0 = 0;
        if (k1 > a.n_intervals) k1 = a.n_intervals;
        if (k1 < k0) k1 = k0;
        for (int64_t k = k0 + tid; k < k1; k += kThreads) {
            const int32_t i = a.iv_tensor[k], o = a.iv_out[k], r = a.iv_in[k];
            if (static_cast<uint32_t>(i) >= static_cast<uint32_t>(a.N) || o < 0 || r > a.T || r <= o) continue;
            const int32_t g = map[i];
            if (g >= 0 && a.gp[g] <= o && r <= a.gq[g]) map[i] = -2;   // all writers write the same value
        }
        __syncthreads();

        // ---- 5: scores of the surviving candidates; reset the map
        auto finish = [&](int32_t g) {
            const int32_t i = a.gtensor[g];
            const bool alive = map[i] == g;
            map[i] = -1;
            if (!alive) return;
            const int32_t o = a.gwin[g], q = a.gq[g];
            int64_t m = P - a.size[i];
            // max MF[0..o]: whole chunks before o's chunk, then the head of that chunk
            const int32_t co = o >> 3;
            if (co > 0) m = max64(m, PMC[co - 1]);
            for (int32_t t = co * kChunk; t <= o; ++t) m = max64(m, MF[t]);
            // max MF[q..T): the tail of q's chunk, then whole chunks after it
            const int32_t cq = q >> 3;
            if (cq + 1 < a.n_chunks) m = max64(m, SMC[cq + 1]);
            const int32_t tail_end = (cq + 1) * kChunk < a.T ? (cq + 1) * kChunk : a.T;
            for (int32_t t = q; t < tail_end; ++t) m = max64(m, MF[t]);
            score[i] = P - m;
            if (wout) wout[i] = o;
            if (win) win[i] = q;
        };
        const int32_t n_cand = list_n;
        if (n_cand <= kListCap) {
            for (int32_t c = tid; c < n_cand; c += kThreads) finish(list[c]);
        } else {   // the list overflowed: find the candidates again
            for (int32_t g = tid; g < a.G; g += kThreads)
                if (is_candidate(a, g, tstar)) finish(g);
        }
    }
}

}  // namespace

int launch_score(const tensile_tas *tas, const tensile_plans *plans, const int64_t *resident, const int64_t *peak,
                 const int32_t *argmax, int64_t *score, int32_t *win_out, int32_t *win_in, hipStream_t stream) {
    if (plans->B == 0 || tas->N == 0) return TENSILE_OK;
    const int32_t want = tas->num_cus * 8;
    const int32_t blocks = plans->B < want ? plans->B : want;
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
    a.T = tas->T; a.N = tas->N; a.B = plans->B; a.G = tas->G;
    a.n_chunks = n_chunks;
    a.n_intervals = plans->n_intervals;
    a.plan_offsets = plans->plan_offsets;
    a.iv_tensor = plans->iv_tensor; a.iv_out = plans->iv_out; a.iv_in = plans->iv_in;
    a.size = tas->d_size.p;
    a.gp = tas->d_gp.p; a.gq = tas->d_gq.p; a.gtensor = tas->d_gtensor.p; a.gwin = tas->d_gwin.p;
    a.resident = resident; a.peak = peak; a.argmax = argmax;
    a.score = score; a.win_out = win_out; a.win_in = win_in;
    a.tables = sc.rowmax.p;
    a.map = sc.cand_map.p;
    a.vec16 = (tas->T % 2 == 0) && (reinterpret_cast<uintptr_t>(resident) % 16 == 0);
    hipLaunchKernelGGL(score_kernel, dim3(blocks), dim3(kThreads), 0, stream, a);
    TS_HIP(hipGetLastError());
    return TENSILE_OK;
}

}  // namespace tensile
