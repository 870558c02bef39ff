// Candidate scoring (section IV-C of the paper): for every plan, how much would
// evicting each tensor that is resident and idle at the peak lower the peak,
// given the earliest swap-out / latest swap-in the host link's speed allows.
//
// One workgroup walks a plan at a time (persistent workgroups, plans dealt
// round-robin), in four phases:
//   1. running maxima of the plan's footprint row: W[t] = max MF[0..t] for
//      t < t*, W[t] = max MF[t..T) for t > t*, written to a scratch row owned by
//      the workgroup (it is read back at scattered positions in phase 4);
//   2. the plan's output rows are cleared (score 0, windows -1);
//   3. the plan's own intervals mark, in an LDS bitmap over tensors, the tensors
//      that already have an interval inside their gap around t*;
//   4. every gap (p, q) of the TAS with p < t* < q whose tensor is not marked and
//      whose precomputed earliest swap-out step o (a property of the gap alone:
//      it depends on p, q, the transfer time and the cumulative latency, not on
//      the plan) lies before t* yields score = P - max(W[o], W[q], P - size).
// Gaps are stored in tensor order, so phase 3/4 can be run per chunk of
// kBitmapBits tensors when N exceeds the bitmap.
#include "common.h"

namespace tensile {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kVpt = 4;
constexpr int kBitmapWords = 8192;                 // 32 KB of LDS
constexpr int kBitmapBits = kBitmapWords * 32;     // tensors per chunk

struct ScoreArgs {
    int32_t T, N, B, G;
    int64_t n_intervals;
    const int64_t *plan_offsets;
    const int32_t *iv_tensor, *iv_out, *iv_in;
    const int64_t *size;
    const int64_t *touch_off;    // [N+1]
    const int32_t *touch;        // alloc step then access steps, per tensor
    const int32_t *gp, *gq, *gtensor, *gwin;   // [G] gaps of length >= 2, in tensor order
    const int64_t *resident;
    const int64_t *peak;
    const int32_t *argmax;
    int64_t *score;
    int32_t *win_out, *win_in;
    int64_t *rowmax;             // [gridDim.x * T]
};

__device__ __forceinline__ int64_t wave_scan_max(int64_t v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int64_t y = __shfl_up(v, d, 64);
        if (lane >= d && y > v) v = y;
    }
    return v;
}

// dst[pos(u)] = max over u' <= u of src[pos(u')], u in [0, n), with pos(u) = start + u*dir.
__device__ void running_max(const int64_t *__restrict__ src, int64_t *__restrict__ dst, int32_t start, int32_t dir,
                            int32_t n, int64_t (*wave_tot)[kWaves]) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int64_t carry = INT64_MIN;
    int buf = 0;
    for (int32_t u0 = 0; u0 < n; u0 += kThreads * kVpt) {
        const int32_t u = u0 + tid * kVpt;
        int64_t v[kVpt];
#pragma unroll
        for (int j = 0; j < kVpt; ++j) v[j] = (u + j < n) ? src[start + (u + j) * dir] : INT64_MIN;
#pragma unroll
        for (int j = 1; j < kVpt; ++j) v[j] = v[j] > v[j - 1] ? v[j] : v[j - 1];
        const int64_t incl = wave_scan_max(v[kVpt - 1], lane);
        int64_t excl = __shfl_up(incl, 1, 64);
        if (lane == 0) excl = INT64_MIN;
        if (lane == 63) wave_tot[buf][wave] = incl;
        __syncthreads();
        int64_t pre = carry;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const int64_t tw = wave_tot[buf][w];
            if (w < wave && tw > pre) pre = tw;
            if (tw > carry) carry = tw;
        }
        if (excl > pre) pre = excl;
#pragma unroll
        for (int j = 0; j < kVpt; ++j)
            if (u + j < n) dst[start + (u + j) * dir] = v[j] > pre ? v[j] : pre;
        buf ^= 1;
    }
}

__global__ __launch_bounds__(kThreads) void score_kernel(const ScoreArgs a) {
    __shared__ uint32_t bitmap[kBitmapWords];
    __shared__ int64_t wave_tot[2][kWaves];
    const int tid = threadIdx.x;
    int64_t *W = a.rowmax + static_cast<int64_t>(blockIdx.x) * a.T;

    for (int32_t b = blockIdx.x; b < a.B; b += gridDim.x) {
        const int32_t tstar = a.argmax[b];
        const int64_t P = a.peak[b];
        const int64_t *MF = a.resident + static_cast<int64_t>(b) * a.T;
        int64_t *score = a.score + static_cast<int64_t>(b) * a.N;
        int32_t *wout = a.win_out ? a.win_out + static_cast<int64_t>(b) * a.N : nullptr;
        int32_t *win = a.win_in ? a.win_in + static_cast<int64_t>(b) * a.N : nullptr;

        // phase 2 first: it has no dependence on the rest
        for (int32_t i = tid; i < a.N; i += kThreads) {
            score[i] = 0;
            if (wout) wout[i] = -1;
            if (win) win[i] = -1;
        }
        if (tstar < 0 || tstar >= a.T) {   // not produced by the evaluator: no candidate
            __syncthreads();
            continue;
        }
        // phase 1
        __syncthreads();   // previous plan's phase 4 has finished reading W
        running_max(MF, W, 0, 1, tstar, wave_tot);
        __syncthreads();
        running_max(MF, W, a.T - 1, -1, a.T - 1 - tstar, wave_tot);

        int64_t k0 = a.plan_offsets[b], k1 = a.plan_offsets[b + 1];
        if (k0 < 0) k0 = 0;
        if (k1 > a.n_intervals) k1 = a.n_intervals;
        if (k1 < k0) k1 = k0;

        for (int32_t cbase = 0; cbase < a.N; cbase += kBitmapBits) {
            const int32_t cend = cbase + kBitmapBits < a.N ? cbase + kBitmapBits : a.N;
            __syncthreads();   // W complete (first chunk) / previous chunk done with the bitmap
            for (int j = tid; j < kBitmapWords; j += kThreads) bitmap[j] = 0;
            __syncthreads();
            // phase 3
            for (int64_t k = k0 + tid; k < k1; k += kThreads) {
                const int32_t i = a.iv_tensor[k], o = a.iv_out[k], r = a.iv_in[k];
                if (i < cbase || i >= cend || o < 0 || r > a.T || r <= o) continue;
                // gap of tensor i around tstar: first touch point >= tstar
                const int64_t lo0 = a.touch_off[i], hi0 = a.touch_off[i + 1];
                int64_t lo = lo0, hi = hi0;
                while (lo < hi) {
                    const int64_t mid = (lo + hi) >> 1;
                    if (a.touch[mid] < tstar) lo = mid + 1;
                    else hi = mid;
                }
                if (lo == lo0 || lo == hi0) continue;          // before the first / after the last touch
                const int32_t q = a.touch[lo];
                if (q == tstar) continue;                      // touched at the peak step
                const int32_t p = a.touch[lo - 1];
                if (p <= o && r <= q) atomicOr(&bitmap[(i - cbase) >> 5], 1u << ((i - cbase) & 31));
            }
            __syncthreads();
            // phase 4: gaps whose tensor lies in [cbase, cend) form a contiguous range
            int32_t g0 = 0, g1 = a.G;
            if (cbase > 0 || cend < a.N) {
                int32_t lo = 0, hi = a.G;
                while (lo < hi) {
                    const int32_t mid = (lo + hi) >> 1;
                    if (a.gtensor[mid] < cbase) lo = mid + 1;
                    else hi = mid;
                }
                g0 = lo;
                hi = a.G;
                while (lo < hi) {
                    const int32_t mid = (lo + hi) >> 1;
                    if (a.gtensor[mid] < cend) lo = mid + 1;
                    else hi = mid;
                }
                g1 = lo;
            }
            for (int32_t g = g0 + tid; g < g1; g += kThreads) {
                const int32_t p = a.gp[g], q = a.gq[g];
                if (!(p < tstar && tstar < q)) continue;
                const int32_t o = a.gwin[g];
                if (o < 0 || o >= tstar) continue;
                const int32_t i = a.gtensor[g];
                if (bitmap[(i - cbase) >> 5] & (1u << ((i - cbase) & 31))) continue;
                int64_t m = P - a.size[i];
                const int64_t left = W[o], right = W[q];
                if (left > m) m = left;
                if (right > m) m = right;
                score[i] = P - m;
                if (wout) wout[i] = o;
                if (win) win[i] = q;
            }
        }
    }
}

}  // namespace

int launch_score(const tensile_tas *tas, const tensile_plans *plans, const int64_t *resident, const int64_t *peak,
                 const int32_t *argmax, int64_t *score, int32_t *win_out, int32_t *win_in, hipStream_t stream) {
    if (plans->B == 0 || tas->N == 0) return TENSILE_OK;
    const int32_t want = tas->num_cus * 4;
    const int32_t blocks = plans->B < want ? plans->B : want;
    Scratch &sc = tas->scratch;
    const size_t need = static_cast<size_t>(blocks) * static_cast<size_t>(tas->T);
    if (sc.rowmax.n < need) {
        TS_HIP(hipDeviceSynchronize());
        TS_HIP(sc.rowmax.reserve(need));
    }
    ScoreArgs a;
    a.T = tas->T; a.N = tas->N; a.B = plans->B; a.G = tas->G;
    a.n_intervals = plans->n_intervals;
    a.plan_offsets = plans->plan_offsets;
    a.iv_tensor = plans->iv_tensor; a.iv_out = plans->iv_out; a.iv_in = plans->iv_in;
    a.size = tas->d_size.p; a.touch_off = tas->d_touch_off.p; a.touch = tas->d_touch.p;
    a.gp = tas->d_gp.p; a.gq = tas->d_gq.p; a.gtensor = tas->d_gtensor.p; a.gwin = tas->d_gwin.p;
    a.resident = resident; a.peak = peak; a.argmax = argmax;
    a.score = score; a.win_out = win_out; a.win_in = win_in;
    a.rowmax = sc.rowmax.p;
    hipLaunchKernelGGL(score_kernel, dim3(blocks), dim3(kThreads), 0, stream, a);
    TS_HIP(hipGetLastError());
    return TENSILE_OK;
}

}  // namespace tensile
