// TAS handle: validation of the description, device copies, and the per-TAS
// tables every plan evaluation shares (unscheduled timeline MF0, cumulative
// latency C, transfer times x, earliest swap-out step per gap).  Also the C-ABI
// entry points that are thin argument checks around the kernels.
#include "common.h"
#include "wave_ops.h"

#include <algorithm>
#include <atomic>
#include <thread>
#include <cstdarg>
#include <cstdio>
#include <new>
#include <unordered_set>

namespace tensile {

namespace {
thread_local std::string g_last_error;
}

void set_error(const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_last_error = buf;
}

int hip_fail(hipError_t e, const char *what) {
    set_error("HIP error %d (%s) in %s", static_cast<int>(e), hipGetErrorString(e), what);
    return e == hipErrorOutOfMemory ? TENSILE_E_NOMEM : TENSILE_E_HIP;
}

namespace {

// x_i = ceil(size_i * 1000 / link_bytes_per_us) ns; 0 without timing information
__global__ void transfer_time_kernel(int32_t N, const int64_t *size, int64_t link_bytes_per_us, int64_t *x) {
    const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N) return;
    x[i] = link_bytes_per_us > 0 ? (size[i] * 1000 + link_bytes_per_us - 1) / link_bytes_per_us : 0;
}

// C[0] = 0, C[t+1] = C[t] + step_ns[t]; one workgroup of 1024 threads, 8192 steps per iteration (8 consecutive
// steps per thread), the next iteration's steps requested before this one's are summed.
__global__ __launch_bounds__(1024) void cumulative_latency_kernel(int32_t T, const int64_t *step_ns, int64_t *C) {
    constexpr int kPer = 8, kChunk = 1024 * kPer, kWavesC = 16;
    __shared__ int64_t wave_tot[2][kWavesC];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int64_t carry = 0;
    int buf = 0;
    if (tid == 0) C[0] = 0;
    auto load = [&](int64_t t, int64_t (&x)[kPer]) {
#pragma unroll
        for (int j = 0; j < kPer; ++j) x[j] = (step_ns && t + j < T) ? step_ns[t + j] : 0;
    };
    int64_t next[kPer];
    load(static_cast<int64_t>(tid) * kPer, next);
    for (int64_t t0 = 0; t0 < T; t0 += kChunk) {
        const int64_t t = t0 + static_cast<int64_t>(tid) * kPer;
        int64_t v[kPer];
#pragma unroll
        for (int j = 0; j < kPer; ++j) v[j] = next[j];
        load(t + kChunk, next);
#pragma unroll
        for (int j = 1; j < kPer; ++j) v[j] += v[j - 1];
        const int64_t incl = wave_scan_add(v[kPer - 1]);
        if (lane == 63) wave_tot[buf][wave] = incl;
        __syncthreads();
        int64_t pre = carry + incl - v[kPer - 1];
#pragma unroll
        for (int w = 0; w < kWavesC; ++w) {
            const int64_t tw = wave_tot[buf][w];
            if (w < wave) pre += tw;
            carry += tw;
        }
#pragma unroll
        for (int j = 0; j < kPer; ++j)
            if (t + j < T) C[t + j + 1] = pre + v[j];
        buf ^= 1;
    }
}

// Earliest feasible swap-out step of every gap (p, q) of tensor i:
//   o = min{ o >= p : C[o+1] - C[p+1] >= x_i }, kept only if C[o+1] + x_i <= C[q]
// (the swap-in, which ends at the start of step q, may not begin before the
// swap-out has ended); -1 otherwise.  C is strictly increasing when timed.
__global__ void gap_window_kernel(int32_t G, int32_t T, const int32_t *gp, const int32_t *gq, const int32_t *gtensor,
                                  const int64_t *C, const int64_t *x, int32_t *gwin) {
    const int32_t g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= G) return;
    const int32_t p = gp[g], q = gq[g];
    const int64_t xi = x[gtensor[g]];
    const int64_t target = C[p + 1] + xi;
    int32_t lo = p, hi = T;          // first o in [p, T) with C[o+1] >= target; T = none
    while (lo < hi) {
        const int32_t mid = lo + ((hi - lo) >> 1);
        if (C[mid + 1] >= target) hi = mid;
        else lo = mid + 1;
    }
    int32_t o = lo;
    if (o >= T || C[o + 1] + xi > C[q]) o = -1;
    gwin[g] = o;
}

// d[t] = MF0[t] - MF0[t-1], d[0] = MF0[0]
__global__ void difference_kernel(int32_t T, const int64_t *MF0, int64_t *d) {
    const int32_t t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < T) d[t] = t > 0 ? MF0[t] - MF0[t - 1] : MF0[0];
}

__global__ void fill_kernel(int64_t n, int64_t value, int64_t *dst) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = value;
}

__global__ void lifetime_intervals_kernel(int32_t N, const int64_t *size, const int32_t *alloc, const int32_t *free_step,
                                          int64_t *neg_size, int32_t *iv_tensor, int32_t *iv_out, int32_t *iv_in) {
    const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N) return;
    neg_size[i] = -size[i];
    iv_tensor[i] = i;
    iv_out[i] = alloc[i] - 1;     // "absent" during alloc .. free with a negated size = present
    iv_in[i] = free_step[i] + 1;
}

int check_latencies(const char *who, int32_t T, int32_t N, const int64_t *size_bytes, const int64_t *step_ns,
                    int64_t link_bytes_per_us) {
    if (!step_ns) return TENSILE_OK;
    if (link_bytes_per_us <= 0) {
        set_error("%s: link_bytes_per_us must be positive when step_ns is given", who);
        return TENSILE_E_INVAL;
    }
    int64_t sum = 0;
    for (int32_t t = 0; t < T; ++t) {
        if (step_ns[t] <= 0) { set_error("%s: step_ns[%d] <= 0", who, t); return TENSILE_E_INVAL; }
        if (__builtin_add_overflow(sum, step_ns[t], &sum)) { set_error("%s: step_ns sums past int64", who); return TENSILE_E_RANGE; }
    }
    if (N > 0 && sum > INT64_MAX / 4) { set_error("%s: total latency too large", who); return TENSILE_E_RANGE; }
    // a transfer time x_i = ceil(size_i * 1000 / link) is added to cumulative latencies: keep it in the same range
    for (int32_t i = 0; i < N; ++i) {
        const int64_t x = (size_bytes[i] * 1000 + link_bytes_per_us - 1) / link_bytes_per_us;   // (size * 1000 fits: checked at load)
        if (x > INT64_MAX / 4) {
            set_error("%s: the transfer of tensor %d over a link of %lld bytes/us takes too long to represent", who, i,
                      static_cast<long long>(link_bytes_per_us));
            return TENSILE_E_RANGE;
        }
    }
    return TENSILE_OK;
}

int validate_desc(const tensile_tas_desc *d) {
    if (!d) { set_error("tas_load: desc is NULL"); return TENSILE_E_INVAL; }
    if (d->T <= 0) { set_error("tas_load: T = %d must be positive", d->T); return TENSILE_E_INVAL; }
    if (d->T > INT32_MAX - (1 << 20)) { set_error("tas_load: T too large"); return TENSILE_E_INVAL; }
    if (d->N < 0) { set_error("tas_load: N = %d is negative", d->N); return TENSILE_E_INVAL; }
    if (d->J < 1) { set_error("tas_load: J = %d must be at least 1", d->J); return TENSILE_E_INVAL; }
    if (d->N > 0 && (!d->size_bytes || !d->alloc_step || !d->free_step || !d->access_offsets)) {
        set_error("tas_load: a required array is NULL");
        return TENSILE_E_INVAL;
    }
    if (d->base_bytes < 0) { set_error("tas_load: base_bytes is negative"); return TENSILE_E_INVAL; }
    if (d->N > 0 && d->access_offsets[0] != 0) { set_error("tas_load: access_offsets[0] != 0"); return TENSILE_E_INVAL; }
    int64_t total = 0;    // the sum of all sizes bounds every footprint: keep it inside int64
    for (int32_t i = 0; i < d->N; ++i) {
        if (d->size_bytes[i] <= 0) { set_error("tas_load: size_bytes[%d] <= 0", i); return TENSILE_E_INVAL; }
        if (d->size_bytes[i] > (INT64_MAX / 1000) - 1) { set_error("tas_load: size_bytes[%d] too large", i); return TENSILE_E_RANGE; }
        if (__builtin_add_overflow(total, d->size_bytes[i], &total) || total > INT64_MAX - d->base_bytes) {
            set_error("tas_load: the sizes sum past int64");
            return TENSILE_E_RANGE;
        }
        const int32_t al = d->alloc_step[i], fr = d->free_step[i];
        if (al < 0 || al >= d->T) { set_error("tas_load: alloc_step[%d] = %d outside [0,T)", i, al); return TENSILE_E_RANGE; }
        if (fr < al || fr >= d->T) { set_error("tas_load: free_step[%d] = %d outside [alloc,T)", i, fr); return TENSILE_E_RANGE; }
        const int64_t a0 = d->access_offsets[i], a1 = d->access_offsets[i + 1];
        if (a1 < a0) { set_error("tas_load: access_offsets not monotone at %d", i); return TENSILE_E_INVAL; }
        if (a1 > a0 && !d->access_steps) { set_error("tas_load: access_steps is NULL"); return TENSILE_E_INVAL; }
        int32_t prev = al;
        for (int64_t k = a0; k < a1; ++k) {
            const int32_t s = d->access_steps[k];
            if (s <= prev || s >= d->T) {
                set_error("tas_load: access %lld of tensor %d (step %d) not after the previous touch point or >= T",
                          static_cast<long long>(k - a0), i, s);
                return TENSILE_E_RANGE;
            }
            prev = s;
        }
        if (prev != fr) { set_error("tas_load: free_step[%d] = %d is not the last touch point %d", i, fr, prev); return TENSILE_E_RANGE; }
        if (d->job_id && (d->job_id[i] < 0 || d->job_id[i] >= d->J)) {
            set_error("tas_load: job_id[%d] outside [0,J)", i);
            return TENSILE_E_RANGE;
        }
    }
    return check_latencies("tas_load", d->T, d->N, d->size_bytes, d->step_ns, d->link_bytes_per_us);
}

// The unscheduled timeline of the tensors with the given sizes on top of a constant `base`, with the
// evaluation kernel: start from the constant and "evict" every tensor with a negated size over its
// lifetime [alloc, free].  MF_out [T]; dMF_out [T rounded up to tiles + 1 tile], zeroed by the caller.
int build_timeline(const tensile_tas *h, const int64_t *d_size, int64_t base_value, const int32_t *d_alloc,
                   const int32_t *d_free, int64_t *MF_out, int64_t *dMF_out, int64_t *peak_host, int32_t *arg_host) {
    const int32_t T = h->T, N = h->N;
    const size_t T_pad = ((static_cast<size_t>(T) + kEvalTile - 1) / kEvalTile + 1) * kEvalTile;
    DevBuf<int64_t> base, dbase, neg, offs, peak, mn;
    DevBuf<int32_t> it, io, ir, arg;
    TS_HIP(base.reserve(T));
    TS_HIP(dbase.reserve(T_pad));     // differences of the constant timeline: base, 0, 0, ...
    TS_HIP(hipMemset(dbase.p, 0, T_pad * sizeof(int64_t)));
    TS_HIP(hipMemcpy(dbase.p, &base_value, sizeof(int64_t), hipMemcpyHostToDevice));
    TS_HIP(neg.reserve(N));
    TS_HIP(it.reserve(N)); TS_HIP(io.reserve(N)); TS_HIP(ir.reserve(N));
    const int64_t h_offs[2] = {0, N};
    TS_HIP(offs.upload(h_offs, 2));
    TS_HIP(peak.reserve(1)); TS_HIP(mn.reserve(1)); TS_HIP(arg.reserve(1));
    hipLaunchKernelGGL(fill_kernel, dim3((T + 255) / 256), dim3(256), 0, 0, static_cast<int64_t>(T), base_value, base.p);
    if (N > 0)
        hipLaunchKernelGGL(lifetime_intervals_kernel, dim3((N + 255) / 256), dim3(256), 0, 0, N, d_size, d_alloc, d_free,
                           neg.p, it.p, io.p, ir.p);
    TS_HIP(hipGetLastError());
    EvalArgs a{};
    a.T = T; a.N = N; a.B = 1; a.o_min = -1; a.n_intervals = N;
    a.plan_offsets = offs.p; a.iv_tensor = it.p; a.iv_out = io.p; a.iv_in = ir.p;
    a.size = neg.p; a.size_units = nullptr; a.MF0 = base.p; a.dMF0 = dbase.p; a.resident = MF_out;
    {
        WorkspaceLock ws = acquire_workspace(h, nullptr);
        const int rc = launch_eval(h, *ws, a, peak.p, arg.p, mn.p);
        if (rc != TENSILE_OK) return rc;
    }
    if (peak_host) TS_HIP(hipMemcpy(peak_host, peak.p, sizeof(int64_t), hipMemcpyDeviceToHost));
    if (arg_host) TS_HIP(hipMemcpy(arg_host, arg.p, sizeof(int32_t), hipMemcpyDeviceToHost));
    hipLaunchKernelGGL(difference_kernel, dim3((T + 255) / 256), dim3(256), 0, 0, T, MF_out, dMF_out);
    TS_HIP(hipGetLastError());
    TS_HIP(hipDeviceSynchronize());     // the temporaries above are freed on return
    return TENSILE_OK;
}

// A gap (p, q) with earliest swap-out step o >= 0 is a scoring candidate at the peak steps
// t* with o < t* < q.  File it under every bucket of 2^shift steps that o+1 .. q-1 overlaps;
// the bucket width starts at 256 steps and doubles while the index would hold more than
// about 16 entries per gap (or its filters more than 256 MiB).  CandIndex (common.h) lists
// what is kept per bucket.
int build_candidate_index(const tensile_tas *h, CandIndex &ix, const std::vector<int32_t> &gp,
                          const std::vector<int32_t> &gq, const std::vector<int32_t> &gt, const std::vector<int32_t> &gwin) {
    const size_t G = gp.size();
    const int32_t T = h->T;
    auto usable = [&](size_t g) { return gwin[g] >= 0 && gwin[g] + 1 <= gq[g] - 1; };
    uint32_t filter_bits = 1024;
    while (filter_bits < 32768 && filter_bits < static_cast<uint32_t>(h->N)) filter_bits <<= 1;
    ix.filter_words = static_cast<int32_t>(filter_bits / 32);
    int32_t shift = 8;
    uint64_t entries;
    for (;; ++shift) {
        entries = 0;
        for (size_t g = 0; g < G; ++g)
            if (usable(g)) entries += ((gq[g] - 1) >> shift) - ((gwin[g] + 1) >> shift) + 1;
        const uint64_t filter_bytes = (static_cast<uint64_t>((T - 1) >> shift) + 1) * (filter_bits / 8);
        if ((entries <= 16 * static_cast<uint64_t>(G) + 4096 && filter_bytes <= (256u << 20)) || (int64_t{1} << shift) >= T) break;
    }
    if (entries > static_cast<uint64_t>(INT32_MAX) / 4) { set_error("tas_load: candidate index too large"); return TENSILE_E_RANGE; }
    const int32_t nb = ((T - 1) >> shift) + 1;
    ix.shift = shift;
    ix.n_buckets = nb;
    ix.tspan = ((h->N + kScoreWaves - 1) / kScoreWaves + kScoreStage - 1) / kScoreStage * kScoreStage;

    std::vector<int32_t> off(static_cast<size_t>(nb) + 1, 0);
    for (size_t g = 0; g < G; ++g)
        if (usable(g))
            for (int32_t b = (gwin[g] + 1) >> shift; b <= (gq[g] - 1) >> shift; ++b) ++off[b + 1];
    for (int32_t b = 0; b < nb; ++b) off[b + 1] += off[b];
    const size_t E = static_cast<size_t>(off[nb]);
    std::vector<int4> cand(E);
    {
        std::vector<int32_t> fill(off.begin(), off.end() - 1);
        for (size_t g = 0; g < G; ++g)
            if (usable(g))
                for (int32_t b = (gwin[g] + 1) >> shift; b <= (gq[g] - 1) >> shift; ++b)
                    cand[fill[b]++] = make_int4(gp[g], gq[g], gwin[g], gt[g]);
    }
    std::vector<int64_t> cand_size(E);
    std::vector<int32_t> cand_o(E), cand_gap(E);
    std::vector<int2> qord(E), tord(E);
    std::vector<int32_t> slice_first(static_cast<size_t>(nb) + 1, 0);
    for (int32_t b = 0; b < nb; ++b)
        slice_first[b + 1] = slice_first[b] + (off[b + 1] - off[b] + kScoreMaxLocal - 1) / kScoreMaxLocal;
    std::vector<int32_t> wave_ptr(static_cast<size_t>(slice_first[nb]) * 4 * (kScoreWaves + 1));
    std::vector<int2> hash_dir(static_cast<size_t>(nb));
    std::vector<uint32_t> filter(static_cast<size_t>(nb) * ix.filter_words, 0u);
    // every bucket's hash table has its place before any is filled: the buckets are then independent of each
    // other and are worked on by several host threads (the sorts dominate the time this takes)
    ix.max_bucket = 0;
    size_t hash_total = 0;
    for (int32_t b = 0; b < nb; ++b) {
        const int32_t n = off[b + 1] - off[b];
        ix.max_bucket = std::max(ix.max_bucket, n);
        int bits = 1;
        while ((int64_t{1} << bits) < 2 * static_cast<int64_t>(n)) ++bits;
        hash_dir[b] = make_int2(static_cast<int32_t>(hash_total), n > 0 ? bits : 0);
        if (n > 0) hash_total += size_t{1} << bits;
        if (hash_total > static_cast<size_t>(INT32_MAX)) { set_error("tas_load: candidate index too large"); return TENSILE_E_RANGE; }
    }
    std::vector<int4> hash_slots(hash_total, make_int4(-1, 0, 0, 0));
    auto do_bucket = [&](int32_t b, std::vector<int32_t> &order) {
        const int32_t e0 = off[b], n = off[b + 1] - off[b];
        int4 *c = cand.data() + e0;
        std::sort(c, c + n, [](const int4 &x, const int4 &y) {
            return x.z != y.z ? x.z < y.z : (x.w != y.w ? x.w < y.w : x.x < y.x);
        });
        for (int32_t k = 0; k < n; ++k) {
            cand_size[e0 + k] = h->h_size[c[k].w];
            cand_o[e0 + k] = c[k].z;
            // the gap's number: its place among the tensor's gaps, which are listed by ascending first step
            const int32_t *g0 = gp.data() + h->h_gap_first[c[k].w], *g1 = gp.data() + h->h_gap_first[c[k].w + 1];
            cand_gap[e0 + k] = static_cast<int32_t>(std::lower_bound(g0, g1, c[k].x) - gp.data());
        }
        for (int32_t s0 = 0, sl = slice_first[b]; s0 < n; s0 += kScoreMaxLocal, ++sl) {
            const int32_t ns = std::min(kScoreMaxLocal, n - s0);
            order.resize(ns);
            for (int32_t k = 0; k < ns; ++k) order[k] = k;
            std::sort(order.begin(), order.end(),
                      [&](int32_t x, int32_t y) { return c[s0 + x].y != c[s0 + y].y ? c[s0 + x].y < c[s0 + y].y : x < y; });
            for (int32_t k = 0; k < ns; ++k) qord[e0 + s0 + k] = make_int2(c[s0 + order[k]].y, order[k]);
            std::sort(order.begin(), order.end(),
                      [&](int32_t x, int32_t y) { return c[s0 + x].w != c[s0 + y].w ? c[s0 + x].w < c[s0 + y].w : x < y; });
            for (int32_t k = 0; k < ns; ++k) tord[e0 + s0 + k] = make_int2(c[s0 + order[k]].w, order[k]);
            int32_t *wp = wave_ptr.data() + static_cast<size_t>(sl) * 4 * (kScoreWaves + 1);
            // The wavefronts' spans of the row.  A wavefront's time in the streaming pass is about one unit per
            // block of kScoreMini steps plus one per kEntriesPerBlock entries whose o or q it meets (measured:
            // 1.05 us per block, 7 ns per entry), so the boundaries are put where the running cost
            // blocks * kEntriesPerBlock + entries passes w/16 of the total (boundaries on whole blocks).
            int32_t *sb = wp + 3 * (kScoreWaves + 1);
            {
                constexpr int64_t kEntriesPerBlock = 150;
                const int64_t nblk = (static_cast<int64_t>(T) + kScoreMini - 1) / kScoreMini;
                auto cost_before = [&](int64_t blk) {   // cost of the blocks [0, blk)
                    const int64_t step = blk * kScoreMini;
                    const int64_t n_o = std::lower_bound(c + s0, c + s0 + ns, step, [](const int4 &e, int64_t v) { return e.z < v; }) - (c + s0);
                    const int2 *qo = qord.data() + e0 + s0;
                    const int64_t n_q = std::lower_bound(qo, qo + ns, step, [](const int2 &e, int64_t v) { return e.x < v; }) - qo;
                    return blk * kEntriesPerBlock + n_o + n_q;
                };
                const int64_t total = cost_before(nblk);
                sb[0] = 0;
                for (int w = 1; w < kScoreWaves; ++w) {
                    const int64_t want = (total * w + kScoreWaves - 1) / kScoreWaves;
                    int64_t lo_b = sb[w - 1] / kScoreMini, hi_b = nblk;       // smallest block count with cost >= want
                    while (lo_b < hi_b) {
                        const int64_t mid = (lo_b + hi_b) / 2;
                        if (cost_before(mid) >= want) hi_b = mid;
                        else lo_b = mid + 1;
                    }
                    sb[w] = static_cast<int32_t>(std::min<int64_t>(lo_b * kScoreMini, T));
                }
                sb[kScoreWaves] = T;
            }
            int32_t ko = 0, kq = 0, kt = 0;
            for (int w = 0; w <= kScoreWaves; ++w) {
                const int64_t bound = sb[w], tbound = static_cast<int64_t>(w) * ix.tspan;
                while (ko < ns && c[s0 + ko].z < bound) ++ko;
                while (kq < ns && qord[e0 + s0 + kq].x < bound) ++kq;
                while (kt < ns && tord[e0 + s0 + kt].x < tbound) ++kt;
                wp[w] = w == kScoreWaves ? ns : ko;
                wp[kScoreWaves + 1 + w] = w == kScoreWaves ? ns : kq;
                wp[2 * (kScoreWaves + 1) + w] = w == kScoreWaves ? ns : kt;
            }
        }
        // hash table: the entries of one tensor are inserted one after the other, the last flagged
        if (n == 0) return;
        const size_t base = static_cast<size_t>(hash_dir[b].x);
        const int bits = hash_dir[b].y;
        order.resize(n);
        for (int32_t k = 0; k < n; ++k) order[k] = k;
        std::sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return c[x].w != c[y].w ? c[x].w < c[y].w : x < y; });
        const uint32_t mask = (1u << bits) - 1;
        for (int32_t k = 0; k < n; ++k) {
            const int4 &en = c[order[k]];
            const bool last = k + 1 == n || c[order[k + 1]].w != en.w;
            uint32_t s = (static_cast<uint32_t>(en.w) * 2654435769u) >> (32 - bits);
            while (hash_slots[base + s].x >= 0) s = (s + 1) & mask;
            hash_slots[base + s] = make_int4(en.w, en.x, en.y, order[k] | (last ? INT32_MIN : 0));
            const uint32_t fb = static_cast<uint32_t>(en.w) & (filter_bits - 1);
            filter[static_cast<size_t>(b) * ix.filter_words + (fb >> 5)] |= 1u << (fb & 31);
        }
    };
    {
        unsigned n_threads = std::thread::hardware_concurrency();
        n_threads = n_threads < 1 ? 1 : n_threads > 16 ? 16 : n_threads;
        if (E < 50000 || nb < 4) n_threads = 1;
        if (n_threads > static_cast<unsigned>(nb)) n_threads = static_cast<unsigned>(nb);
        std::atomic<int32_t> next_bucket{0};
        std::atomic<bool> failed{false};
        auto worker = [&]() {
            try {
                std::vector<int32_t> order;
                for (int32_t b; (b = next_bucket.fetch_add(1)) < nb;) do_bucket(b, order);
            } catch (...) {
                failed = true;
            }
        };
        std::vector<std::thread> pool;
        try {
            for (unsigned k = 1; k < n_threads; ++k) pool.emplace_back(worker);
        } catch (...) {   // (no more threads to be had: the ones there and this one do the work)
        }
        worker();
        for (std::thread &t : pool) t.join();
        if (failed) throw std::bad_alloc();
    }
    TS_HIP(ix.bucket_off.upload(off.data(), off.size()));
    TS_HIP(ix.cand.upload(cand.data(), E));
    TS_HIP(ix.cand_size.upload(cand_size.data(), E));
    TS_HIP(ix.cand_o.upload(cand_o.data(), E));
    TS_HIP(ix.cand_gap.upload(cand_gap.data(), E));
    TS_HIP(ix.qord.upload(qord.data(), E));
    TS_HIP(ix.tord.upload(tord.data(), E));
    TS_HIP(ix.slice_first.upload(slice_first.data(), slice_first.size()));
    TS_HIP(ix.wave_ptr.upload(wave_ptr.data(), wave_ptr.size()));
    TS_HIP(ix.hash_dir.upload(hash_dir.data(), hash_dir.size()));
    TS_HIP(ix.hash_slots.upload(hash_slots.data(), hash_slots.size()));
    TS_HIP(ix.filter.upload(filter.data(), filter.size()));
    return TENSILE_OK;
}

int build(tensile_tas *h, const tensile_tas_desc *d) {
    const int32_t T = d->T, N = d->N;
    TS_HIP(hipGetDevice(&h->device));
    hipDeviceProp_t prop;
    TS_HIP(hipGetDeviceProperties(&prop, h->device));
    h->num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    h->T = T; h->N = N; h->J = d->J;
    h->timed = d->step_ns != nullptr;
    h->base_bytes = d->base_bytes;
    h->link_bytes_per_us = h->timed ? d->link_bytes_per_us : 0;

    // host copies: sizes, touch points (alloc then accesses), jobs
    h->h_size.assign(d->size_bytes, d->size_bytes + N);
    h->h_job.assign(static_cast<size_t>(N), 0);
    if (d->job_id) h->h_job.assign(d->job_id, d->job_id + N);
    h->h_touch_off.resize(static_cast<size_t>(N) + 1);
    const int64_t n_acc = N > 0 ? d->access_offsets[N] : 0;
    h->h_touch.resize(static_cast<size_t>(n_acc + N));
    std::vector<int32_t> gp, gq, gt;
    for (int32_t i = 0; i < N; ++i) {
        const int64_t a0 = d->access_offsets[i], a1 = d->access_offsets[i + 1];
        int64_t w = a0 + i;
        h->h_touch_off[i] = w;
        h->h_touch[w++] = d->alloc_step[i];
        for (int64_t k = a0; k < a1; ++k) {
            const int32_t prev = h->h_touch[w - 1], s = d->access_steps[k];
            if (s - prev >= 2) {          // a shorter gap has no step strictly inside
                gp.push_back(prev);
                gq.push_back(s);
                gt.push_back(i);
            }
            h->h_touch[w++] = s;
        }
    }
    h->h_touch_off[N] = n_acc + N;
    if (gp.size() > static_cast<size_t>(INT32_MAX)) { set_error("tas_load: too many gaps"); return TENSILE_E_RANGE; }
    h->G = static_cast<int32_t>(gp.size());

    TS_HIP(h->d_size.upload(h->h_size.data(), N));
    TS_HIP(h->d_touch_off.upload(h->h_touch_off.data(), static_cast<size_t>(N) + 1));
    TS_HIP(h->d_touch.upload(h->h_touch.data(), h->h_touch.size()));
    // whole tiles plus one: the evaluation kernel prefetches one tile ahead unconditionally
    const size_t T_pad = ((static_cast<size_t>(T) + kEvalTile - 1) / kEvalTile + 1) * kEvalTile;
    TS_HIP(h->d_MF0.reserve(T));
    TS_HIP(h->d_dMF0.reserve(T_pad));
    TS_HIP(hipMemset(h->d_dMF0.p, 0, T_pad * sizeof(int64_t)));
    {   // sizes as 32-bit multiples of their common power of two, when they fit
        uint64_t all = 0, mx = 0;
        for (int32_t i = 0; i < N; ++i) {
            all |= static_cast<uint64_t>(d->size_bytes[i]);
            mx = std::max<uint64_t>(mx, static_cast<uint64_t>(d->size_bytes[i]));
        }
        const int shift = all ? __builtin_ctzll(all) : 0;
        if (N > 0 && (mx >> shift) <= 0xffffffffULL) {
            std::vector<uint32_t> units(static_cast<size_t>(N));
            for (int32_t i = 0; i < N; ++i) units[i] = static_cast<uint32_t>(static_cast<uint64_t>(d->size_bytes[i]) >> shift);
            TS_HIP(h->d_size_units.upload(units.data(), units.size()));
            h->size_shift = shift;
        }
    }
    TS_HIP(h->d_C.reserve(static_cast<size_t>(T) + 1));
    TS_HIP(h->d_x.reserve(N));

    // ---- MF0 and its differences
    {
        DevBuf<int32_t> alloc, fr;
        TS_HIP(alloc.upload(d->alloc_step, N));
        TS_HIP(fr.upload(d->free_step, N));
        int rc = build_timeline(h, h->d_size.p, d->base_bytes, alloc.p, fr.p, h->d_MF0.p, h->d_dMF0.p, &h->unscheduled_peak,
                                &h->unscheduled_argmax);
        if (rc != TENSILE_OK) return rc;
    }

    h->h_gap_first.assign(static_cast<size_t>(N) + 1, 0);
    for (int32_t t : gt) ++h->h_gap_first[t + 1];
    for (int32_t i = 0; i < N; ++i) h->h_gap_first[i + 1] += h->h_gap_first[i];
    h->h_gp = std::move(gp);
    h->h_gq = std::move(gq);
    h->h_gt = std::move(gt);
    return build_times_and_index(h, d->step_ns);
}

}  // namespace

// Everything that depends on the operator latencies and the link speed: cumulative latency C,
// transfer times x, every gap's earliest swap-out step, and the swap-candidate index built from
// them.  step_ns is a HOST array or null (no latencies: all transfer times 0).
int build_times_and_index(tensile_tas *h, const int64_t *step_ns) {
    const int32_t T = h->T, N = h->N;
    const std::vector<int32_t> &gp = h->h_gp, &gq = h->h_gq, &gt = h->h_gt;
    {
        DevBuf<int64_t> step;
        if (h->timed) TS_HIP(step.upload(step_ns, T));
        hipLaunchKernelGGL(cumulative_latency_kernel, dim3(1), dim3(1024), 0, 0, T, h->timed ? step.p : nullptr, h->d_C.p);
        if (N > 0)
            hipLaunchKernelGGL(transfer_time_kernel, dim3((N + 255) / 256), dim3(256), 0, 0, N, h->d_size.p,
                               h->link_bytes_per_us, h->d_x.p);
        DevBuf<int32_t> d_gp, d_gq, d_gt, d_gwin;
        TS_HIP(d_gp.upload(gp.data(), gp.size()));
        TS_HIP(d_gq.upload(gq.data(), gq.size()));
        TS_HIP(d_gt.upload(gt.data(), gt.size()));
        TS_HIP(d_gwin.reserve(gp.size()));
        if (h->G > 0)
            hipLaunchKernelGGL(gap_window_kernel, dim3((h->G + 255) / 256), dim3(256), 0, 0, h->G, T, d_gp.p, d_gq.p,
                               d_gt.p, h->d_C.p, h->d_x.p, d_gwin.p);
        TS_HIP(hipGetLastError());
        TS_HIP(hipDeviceSynchronize());
        std::vector<int32_t> gwin(gp.size());
        if (h->G > 0) TS_HIP(hipMemcpy(gwin.data(), d_gwin.p, gwin.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
        int rc = build_candidate_index(h, h->index, gp, gq, gt, gwin);
        if (rc != TENSILE_OK) return rc;
    }
    h->h_C.resize(static_cast<size_t>(T) + 1);
    h->h_x.resize(static_cast<size_t>(N));
    TS_HIP(hipMemcpy(h->h_C.data(), h->d_C.p, (static_cast<size_t>(T) + 1) * sizeof(int64_t), hipMemcpyDeviceToHost));
    if (N > 0) TS_HIP(hipMemcpy(h->h_x.data(), h->d_x.p, static_cast<size_t>(N) * sizeof(int64_t), hipMemcpyDeviceToHost));
    // C packed for the link kernel: block b holds, 21 bits each, C[7b+1]-C[7b] .. C[7b+6]-C[7b+5] (0 past C[T])
    h->c_packed = false;
    if (h->timed) {
        constexpr int kBits = 21;
        const std::vector<int64_t> &C = h->h_C;
        bool fits = true;
        for (int32_t t = 0; t < T && fits; ++t) fits = C[t + 1] - C[t] < (int64_t{1} << kBits);
        if (fits) {
            std::vector<uint4> rec(static_cast<size_t>(T) / kLinkCBlock + 1);
            for (size_t b = 0; b < rec.size(); ++b) {
                unsigned __int128 bits = 0;
                for (int j = 0; j + 1 < kLinkCBlock; ++j) {
                    const int64_t k = static_cast<int64_t>(b) * kLinkCBlock + j;
                    const uint64_t d = k + 1 <= T ? static_cast<uint64_t>(C[k + 1] - C[k]) : 0;
                    bits |= static_cast<unsigned __int128>(d) << (kBits * j);
                }
                rec[b] = make_uint4(static_cast<uint32_t>(bits), static_cast<uint32_t>(bits >> 32), static_cast<uint32_t>(bits >> 64),
                                    static_cast<uint32_t>(bits >> 96));
            }
            TS_HIP(h->d_Cpack.upload(rec.data(), rec.size()));
            h->c_packed = true;
        }
    }
    return TENSILE_OK;
}

// The index of the recomputation candidates: every gap, released right after the access that
// opens it (o = p).  Built on first use, by whichever caller comes first (the others wait).
int ensure_recompute_index(const tensile_tas *tas) {
    std::lock_guard<std::mutex> once(tas->lazy_mu);
    if (tas->recompute_index_built) return TENSILE_OK;
    try {
        int rc = build_candidate_index(tas, tas->recompute_index, tas->h_gp, tas->h_gq, tas->h_gt, tas->h_gp);
        if (rc != TENSILE_OK) return rc;
    } catch (const std::bad_alloc &) {
        set_error("score_recompute: out of host memory");
        return TENSILE_E_NOMEM;
    }
    tas->recompute_index_built = true;
    return TENSILE_OK;
}

// Per-job copies of the tables the evaluation kernel reads: sizes with the other jobs' tensors set to
// zero (an interval on such a tensor then changes nothing), and each job's own unscheduled timeline
// without the base bytes.  Built on first use (see ensure_recompute_index about concurrency).
int ensure_job_tables(const tensile_tas *tas) {
    std::lock_guard<std::mutex> once(tas->lazy_mu);
    JobTables &jt = tas->job_tables;
    if (jt.built) return TENSILE_OK;
    const int32_t T = tas->T, N = tas->N, J = tas->J;
    jt.T_pad = ((static_cast<size_t>(T) + kEvalTile - 1) / kEvalTile + 1) * kEvalTile;
    try {
        std::vector<int64_t> sizes(static_cast<size_t>(J) * N, 0);
        std::vector<uint32_t> units;
        const bool narrow = tas->d_size_units.p != nullptr;
        if (narrow) units.assign(static_cast<size_t>(J) * N, 0u);
        std::vector<int32_t> alloc(static_cast<size_t>(N)), fr(static_cast<size_t>(N));
        for (int32_t i = 0; i < N; ++i) {
            const int32_t j = tas->h_job.empty() ? 0 : tas->h_job[i];
            sizes[static_cast<size_t>(j) * N + i] = tas->h_size[i];
            if (narrow) units[static_cast<size_t>(j) * N + i] = static_cast<uint32_t>(static_cast<uint64_t>(tas->h_size[i]) >> tas->size_shift);
            alloc[i] = tas->h_touch[tas->h_touch_off[i]];
            fr[i] = tas->h_touch[tas->h_touch_off[i + 1] - 1];
        }
        TS_HIP(jt.size.upload(sizes.data(), sizes.size()));
        if (narrow) TS_HIP(jt.units.upload(units.data(), units.size()));
        TS_HIP(jt.MF0.reserve(static_cast<size_t>(J) * T));
        TS_HIP(jt.dMF0.reserve(static_cast<size_t>(J) * jt.T_pad));
        TS_HIP(hipMemset(jt.dMF0.p, 0, static_cast<size_t>(J) * jt.T_pad * sizeof(int64_t)));
        DevBuf<int32_t> d_alloc, d_free;
        TS_HIP(d_alloc.upload(alloc.data(), alloc.size()));
        TS_HIP(d_free.upload(fr.data(), fr.size()));
        for (int32_t j = 0; j < J; ++j) {
            int rc = build_timeline(tas, jt.size.p + static_cast<size_t>(j) * N, 0, d_alloc.p, d_free.p,
                                    jt.MF0.p + static_cast<size_t>(j) * T, jt.dMF0.p + static_cast<size_t>(j) * jt.T_pad, nullptr,
                                    nullptr);
            if (rc != TENSILE_OK) return rc;
        }
    } catch (const std::bad_alloc &) {
        set_error("eval_plans_per_job: out of host memory");
        return TENSILE_E_NOMEM;
    }
    jt.built = true;
    return TENSILE_OK;
}

namespace {

// sum_peak[b] = base + sum over jobs of job_peak[j*B + b]
__global__ void sum_job_peaks_kernel(int32_t B, int32_t J, int64_t base, const int64_t *job_peak, int64_t *sum_peak) {
    const int32_t b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int64_t s = base;
    for (int32_t j = 0; j < J; ++j) s += job_peak[static_cast<int64_t>(j) * B + b];
    sum_peak[b] = s;
}

}  // namespace

int check_plans(const tensile_tas *tas, const tensile_plans *plans, const char *who) {
    if (!tas || !plans) { set_error("%s: NULL handle or plans", who); return TENSILE_E_INVAL; }
    if (plans->B < 0 || plans->n_intervals < 0) { set_error("%s: negative B or n_intervals", who); return TENSILE_E_INVAL; }
    if (plans->B > 0 && !plans->plan_offsets) { set_error("%s: plan_offsets is NULL", who); return TENSILE_E_INVAL; }
    if (plans->n_intervals > 0 && (!plans->iv_tensor || !plans->iv_out || !plans->iv_in)) {
        set_error("%s: an interval array is NULL", who);
        return TENSILE_E_INVAL;
    }
    return TENSILE_OK;
}

}  // namespace tensile

using namespace tensile;

extern "C" {

const char *tensile_last_error(void) { return g_last_error.c_str(); }

int tensile_version(void) { return 100; }

int tensile_tas_load(const tensile_tas_desc *desc, tensile_tas **out) {
    if (!out) { set_error("tas_load: out is NULL"); return TENSILE_E_INVAL; }
    *out = nullptr;
    int rc = validate_desc(desc);
    if (rc != TENSILE_OK) return rc;
    tensile_tas *h = new (std::nothrow) tensile_tas();
    if (!h) { set_error("tas_load: out of host memory"); return TENSILE_E_NOMEM; }
    try {
        rc = build(h, desc);
    } catch (const std::bad_alloc &) {
        set_error("tas_load: out of host memory");
        rc = TENSILE_E_NOMEM;
    }
    if (rc != TENSILE_OK) {
        delete h;
        return rc;
    }
    *out = h;
    return TENSILE_OK;
}

void tensile_tas_free(tensile_tas *tas) {
    if (!tas) return;
    (void)hipDeviceSynchronize();
    drop_greedy_cache(tas);
    delete tas;
}

int tensile_tas_update_latencies(tensile_tas *tas, const int64_t *step_ns, int64_t link_bytes_per_us) {
    if (!tas) { set_error("tas_update_latencies: NULL handle"); return TENSILE_E_INVAL; }
    int rc = check_latencies("tas_update_latencies", tas->T, tas->N, tas->h_size.data(), step_ns, link_bytes_per_us);
    if (rc != TENSILE_OK) return rc;
    TS_HIP(hipDeviceSynchronize());     // earlier launches may still read the tables replaced below
    tas->timed = step_ns != nullptr;
    tas->link_bytes_per_us = tas->timed ? link_bytes_per_us : 0;
    try {
        return build_times_and_index(tas, step_ns);
    } catch (const std::bad_alloc &) {
        set_error("tas_update_latencies: out of host memory");
        return TENSILE_E_NOMEM;
    }
}

int tensile_tas_info(const tensile_tas *tas, int64_t *unscheduled_peak, int32_t *argmax) {
    if (!tas) { set_error("tas_info: NULL handle"); return TENSILE_E_INVAL; }
    if (unscheduled_peak) *unscheduled_peak = tas->unscheduled_peak;
    if (argmax) *argmax = tas->unscheduled_argmax;
    return TENSILE_OK;
}

int tensile_tas_base_timeline(const tensile_tas *tas, int64_t *mf0_host) {
    if (!tas || !mf0_host) { set_error("tas_base_timeline: NULL argument"); return TENSILE_E_INVAL; }
    TS_HIP(hipMemcpy(mf0_host, tas->d_MF0.p, static_cast<size_t>(tas->T) * sizeof(int64_t), hipMemcpyDeviceToHost));
    return TENSILE_OK;
}

int tensile_eval_plans(const tensile_tas *tas, const tensile_plans *plans, int64_t *resident, int64_t *peak,
                       int32_t *argmax, int64_t *min_resident, void *hip_stream) {
    int rc = check_plans(tas, plans, "eval_plans");
    if (rc != TENSILE_OK) return rc;
    if (plans->B == 0) return TENSILE_OK;
    if (!peak || !argmax) { set_error("eval_plans: peak and argmax are required"); return TENSILE_E_INVAL; }
    EvalArgs a{};
    a.T = tas->T; a.N = tas->N; a.B = plans->B; a.o_min = 0; a.n_intervals = plans->n_intervals;
    a.plan_offsets = plans->plan_offsets;
    a.iv_tensor = plans->iv_tensor; a.iv_out = plans->iv_out; a.iv_in = plans->iv_in;
    a.size = tas->d_size.p; a.size_units = tas->d_size_units.p; a.size_shift = tas->size_shift;
    a.MF0 = tas->d_MF0.p; a.dMF0 = tas->d_dMF0.p; a.resident = resident;
    WorkspaceLock ws = acquire_workspace(tas, static_cast<hipStream_t>(hip_stream));
    return launch_eval(tas, *ws, a, peak, argmax, min_resident);
}

int tensile_eval_plans_per_job(const tensile_tas *tas, const tensile_plans *plans, int64_t *job_peak, int32_t *job_argmax,
                               int64_t *sum_peak, void *hip_stream) {
    int rc = check_plans(tas, plans, "eval_plans_per_job");
    if (rc != TENSILE_OK) return rc;
    if (plans->B == 0) return TENSILE_OK;
    if (!job_peak) { set_error("eval_plans_per_job: job_peak is required"); return TENSILE_E_INVAL; }
    rc = ensure_job_tables(tas);
    if (rc != TENSILE_OK) return rc;
    const JobTables &jt = tas->job_tables;
    const int32_t B = plans->B, J = tas->J;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    WorkspaceLock ws = acquire_workspace(tas, stream);
    if (!job_argmax) {
        rc = ws->provide(ws->job_arg, static_cast<size_t>(J) * B, "eval_plans_per_job: peak steps");
        if (rc != TENSILE_OK) return rc;
        job_argmax = ws->job_arg.p;
    }
    for (int32_t j = 0; j < J; ++j) {      // one pass of the evaluation kernel per job, footprint rows not written
        EvalArgs a{};
        a.T = tas->T; a.N = tas->N; a.B = B; a.o_min = 0; a.n_intervals = plans->n_intervals;
        a.plan_offsets = plans->plan_offsets;
        a.iv_tensor = plans->iv_tensor; a.iv_out = plans->iv_out; a.iv_in = plans->iv_in;
        a.size = jt.size.p + static_cast<size_t>(j) * tas->N;
        a.size_units = jt.units.p ? jt.units.p + static_cast<size_t>(j) * tas->N : nullptr;
        a.size_shift = tas->size_shift;
        a.MF0 = jt.MF0.p + static_cast<size_t>(j) * tas->T;
        a.dMF0 = jt.dMF0.p + static_cast<size_t>(j) * jt.T_pad;
        a.resident = nullptr;
        rc = launch_eval(tas, *ws, a, job_peak + static_cast<size_t>(j) * B, job_argmax + static_cast<size_t>(j) * B, nullptr);
        if (rc != TENSILE_OK) return rc;
    }
    if (sum_peak) {
        hipLaunchKernelGGL(sum_job_peaks_kernel, dim3((B + 255) / 256), dim3(256), 0, stream, B, J, tas->base_bytes, job_peak,
                           sum_peak);
        TS_HIP(hipGetLastError());
    }
    return TENSILE_OK;
}

int tensile_apply_intervals(const tensile_tas *tas, int32_t B, const int32_t *tensor, const int32_t *out_step,
                            const int32_t *in_step, int64_t *resident, int64_t *peak, int32_t *argmax,
                            int64_t *min_resident, void *hip_stream) {
    if (!tas) { set_error("apply_intervals: NULL handle"); return TENSILE_E_INVAL; }
    if (B < 0) { set_error("apply_intervals: negative B"); return TENSILE_E_INVAL; }
    if (B == 0) return TENSILE_OK;
    if (!tensor || !out_step || !in_step || !resident || !peak || !argmax) {
        set_error("apply_intervals: tensor, out_step, in_step, resident, peak and argmax are required");
        return TENSILE_E_INVAL;
    }
    WorkspaceLock ws = acquire_workspace(tas, static_cast<hipStream_t>(hip_stream));
    return launch_apply(tas, *ws, B, tensor, out_step, in_step, resident, peak, argmax, min_resident);
}

int tensile_eval_link(const tensile_tas *tas, const tensile_plans *plans, int32_t reuse_host_copies, int32_t *link,
                      int32_t *link_peak, int32_t *link_argmax, int32_t *overbooked, void *hip_stream) {
    int rc = check_plans(tas, plans, "eval_link");
    if (rc != TENSILE_OK) return rc;
    if (plans->B == 0) return TENSILE_OK;
    if (!link_peak) { set_error("eval_link: link_peak is required"); return TENSILE_E_INVAL; }
    WorkspaceLock ws = acquire_workspace(tas, static_cast<hipStream_t>(hip_stream));
    return launch_link(tas, *ws, plans, reuse_host_copies != 0, link, link_peak, link_argmax, overbooked);
}

int tensile_score_candidates(const tensile_tas *tas, const tensile_plans *plans, const int64_t *resident,
                             const int64_t *peak, const int32_t *argmax, int64_t *score, int32_t *win_out,
                             int32_t *win_in, void *hip_stream) {
    int rc = check_plans(tas, plans, "score_candidates");
    if (rc != TENSILE_OK) return rc;
    if (plans->B == 0) return TENSILE_OK;
    if (!resident || !peak || !argmax || !score) {
        set_error("score_candidates: resident, peak, argmax and score are required");
        return TENSILE_E_INVAL;
    }
    WorkspaceLock ws = acquire_workspace(tas, static_cast<hipStream_t>(hip_stream));
    return launch_score(tas, *ws, tas->index, false, plans, resident, peak, argmax, score, win_out, win_in);
}

int tensile_score_recompute(const tensile_tas *tas, const tensile_plans *plans, const int64_t *resident,
                            const int64_t *peak, const int32_t *argmax, int64_t *score, int32_t *win_out,
                            int32_t *win_in, void *hip_stream) {
    int rc = check_plans(tas, plans, "score_recompute");
    if (rc != TENSILE_OK) return rc;
    if (plans->B == 0) return TENSILE_OK;
    if (!resident || !peak || !argmax || !score) {
        set_error("score_recompute: resident, peak, argmax and score are required");
        return TENSILE_E_INVAL;
    }
    rc = ensure_recompute_index(tas);
    if (rc != TENSILE_OK) return rc;
    WorkspaceLock ws = acquire_workspace(tas, static_cast<hipStream_t>(hip_stream));
    return launch_score(tas, *ws, tas->recompute_index, true, plans, resident, peak, argmax, score, win_out, win_in);
}

int tensile_validate_plans(const tensile_tas *tas, const tensile_plans *plans, int64_t *first_bad, int32_t *reason) {
    int rc = check_plans(tas, plans, "validate_plans");
    if (rc != TENSILE_OK) return rc;
    if (!first_bad) { set_error("validate_plans: first_bad is NULL"); return TENSILE_E_INVAL; }
    *first_bad = -1;
    if (reason) *reason = 0;
    const int32_t B = plans->B;
    const int64_t K = plans->n_intervals;
    try {
        std::vector<int64_t> offs(static_cast<size_t>(B) + 1);
        std::vector<int32_t> it(K), io(K), ir(K);
        if (B > 0) TS_HIP(hipMemcpy(offs.data(), plans->plan_offsets, offs.size() * 8, hipMemcpyDeviceToHost));
        if (K > 0) {
            TS_HIP(hipMemcpy(it.data(), plans->iv_tensor, K * 4, hipMemcpyDeviceToHost));
            TS_HIP(hipMemcpy(io.data(), plans->iv_out, K * 4, hipMemcpyDeviceToHost));
            TS_HIP(hipMemcpy(ir.data(), plans->iv_in, K * 4, hipMemcpyDeviceToHost));
        }
        auto fail = [&](int64_t k, int32_t why) {
            *first_bad = k;
            if (reason) *reason = why;
            return TENSILE_OK;
        };
        std::unordered_set<int64_t> used;
        for (int32_t b = 0; b < B; ++b) {
            if (offs[b] < 0 || offs[b + 1] < offs[b] || offs[b + 1] > K) return fail(offs[b] < 0 ? 0 : offs[b], 4);
            used.clear();
            for (int64_t k = offs[b]; k < offs[b + 1]; ++k) {
                const int32_t i = it[k], o = io[k], r = ir[k];
                if (i < 0 || i >= tas->N || o < 0 || r > tas->T || r <= o) return fail(k, 1);
                // gap with p_g <= o < p_{g+1}
                const int32_t *tp = tas->h_touch.data();
                int64_t lo = tas->h_touch_off[i], hi = tas->h_touch_off[i + 1];
                const int64_t first = lo, last = hi;
                while (lo < hi) {
                    const int64_t mid = (lo + hi) >> 1;
                    if (tp[mid] <= o) lo = mid + 1;
                    else hi = mid;
                }
                if (lo == first || lo == last || r > tp[lo]) return fail(k, 2);
                if (!used.insert(lo).second) return fail(k, 3);
            }
        }
    } catch (const std::bad_alloc &) {
        set_error("validate_plans: out of host memory");
        return TENSILE_E_NOMEM;
    }
    return TENSILE_OK;
}

}  // extern "C"
