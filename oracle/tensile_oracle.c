/* TEST INFRASTRUCTURE - not part of the product.
 *
 * Plain, slow, single-threaded CPU statement of what the batched plan evaluator
 * computes, written from the paper (TENSILE, arXiv 2105.13336).  Only tests,
 * the smoke check and the benchmark's cpu_baseline leg may call it.  It shares
 * no code with the HIP path.  All arithmetic is int64; there is no floating
 * point.
 *
 * Step-indexed model (the discretisation of the paper's continuous time axis):
 *   step t in [0,T) is one operator-execution slot of the merged timeline
 *   (section III-A, "Workload": accesses ordered by execution order).
 *   Tensor i: size[i] bytes, resident from its tensor-generating access
 *   alloc[i] (section IV-B situation 2, Alg. 1 "output_access" branch) through
 *   free[i], the step of its last tensor-using access (activity analysis,
 *   section IV-E: released when its last TUA finishes; Alg. 1 releases a tensor
 *   once the traversal has passed the tensor's end time).
 *   A plan interval (i, o, r, kind): tensor i is NOT resident during steps
 *   o+1 .. r-1.  o is the last step it is still resident (the footprint drops
 *   at the end of the swap-out, or of the using access if that ends later -
 *   situation 4; or the release after an access for recomputation - situation
 *   5); r is the step at which its bytes are back (the swap-in's finishing
 *   point is when the footprint rises - situation 3).
 *
 * Intervals that cannot be applied (tensor outside [0,N), o < 0, r > T,
 * r <= o) are skipped everywhere, in the same way as the evaluator's header
 * states; plan offsets are clamped to [0, n_intervals].
 *
 * Pins (tests/test_oracle_*.py): literal membership sums in numpy, numpy.cumsum
 * on the difference array, a hand-worked example, closed-form staircases,
 * invariants, brute force over all swap subsets on tiny sequences.
 * oracle_greedy: closeness to the optimum is a heuristic property -> "parity
 * unpinned" beyond monotonicity, validity, idempotence and the brute-force
 * bounds.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define OR_OK 0
#define OR_E_INVAL (-1)
#define OR_E_NOMEM (-3)

static int interval_applies(int32_t N, int32_t T, int32_t i, int32_t o, int32_t r) {
    return i >= 0 && i < N && o >= 0 && r <= T && r > o;
}

static void plan_range(const int64_t *plan_offsets, int64_t b, int64_t n_intervals, int64_t *k0, int64_t *k1) {
    int64_t a = plan_offsets[b], e = plan_offsets[b + 1];
    if (a < 0) a = 0;
    if (e > n_intervals) e = n_intervals;
    if (e < a) e = a;
    *k0 = a;
    *k1 = e;
}

/* Eq. 1 with no scheduling events: MF0[t] = base + sum of size[i] over tensors
 * with alloc[i] <= t <= free[i].  Written as the running sum of Mem(a) over the
 * accesses in time order: +size at the TGA, -size right after the last TUA. */
int oracle_base_timeline(int32_t T, int32_t N, const int64_t *size, const int32_t *alloc, const int32_t *free_step,
                         int64_t base_bytes, int64_t *MF0) {
    if (T <= 0 || N < 0) return OR_E_INVAL;
    int64_t *D = (int64_t *)calloc((size_t)T + 1, sizeof(int64_t));
    if (!D) return OR_E_NOMEM;
    for (int32_t i = 0; i < N; ++i) {
        D[alloc[i]] += size[i];
        D[free_step[i] + 1] -= size[i];
    }
    int64_t memory_used = base_bytes;
    for (int32_t t = 0; t < T; ++t) {
        memory_used += D[t];
        MF0[t] = memory_used;
    }
    free(D);
    return OR_OK;
}

/* One plan: Eq. 1 (footprint after every step) and Eq. 2 (its maximum), with
 * Alg. 1's strict '>' update so the earliest step attaining the maximum is the
 * peak time.  MF[T] is written; D is a caller-provided scratch of T+1 words. */
static void eval_one(int32_t T, int32_t N, const int64_t *size, const int64_t *MF0, int64_t k0, int64_t k1,
                     const int32_t *iv_tensor, const int32_t *iv_out, const int32_t *iv_in, int64_t *D, int64_t *MF,
                     int64_t *peak, int32_t *argmax, int64_t *min_resident) {
    memset(D, 0, ((size_t)T + 1) * sizeof(int64_t));
    for (int64_t k = k0; k < k1; ++k) {
        int32_t i = iv_tensor[k], o = iv_out[k], r = iv_in[k];
        if (!interval_applies(N, T, i, o, r)) continue;
        D[o + 1] -= size[i];            /* swap-out / release: Mem(x) = -size */
        if (r < T) D[r] += size[i];     /* swap-in / recompute: Mem(x) = +size */
    }
    int64_t run = 0;
    for (int32_t t = 0; t < T; ++t) {
        run += D[t];
        MF[t] = MF0[t] + run;
    }
    int64_t memory_peak = MF[0], mn = MF[0];
    int32_t MPTime = 0;
    for (int32_t t = 1; t < T; ++t) {
        if (MF[t] > memory_peak) {
            memory_peak = MF[t];
            MPTime = t;
        }
        if (MF[t] < mn) mn = MF[t];
    }
    *peak = memory_peak;
    *argmax = MPTime;
    *min_resident = mn;
}

/* B plans.  resident may be NULL (then only peak/argmax/min are produced). */
int oracle_eval(int32_t T, int32_t N, const int64_t *size, const int64_t *MF0, int64_t B, const int64_t *plan_offsets,
                int64_t n_intervals, const int32_t *iv_tensor, const int32_t *iv_out, const int32_t *iv_in,
                int64_t *resident, int64_t *peak, int32_t *argmax, int64_t *min_resident) {
    if (T <= 0 || N < 0 || B < 0) return OR_E_INVAL;
    int64_t *D = (int64_t *)malloc(((size_t)T + 1) * sizeof(int64_t));
    int64_t *row = resident ? NULL : (int64_t *)malloc((size_t)T * sizeof(int64_t));
    if (!D || (!resident && !row)) {
        free(D);
        free(row);
        return OR_E_NOMEM;
    }
    for (int64_t b = 0; b < B; ++b) {
        int64_t k0, k1;
        plan_range(plan_offsets, b, n_intervals, &k0, &k1);
        int64_t *MF = resident ? resident + b * (int64_t)T : row;
        eval_one(T, N, size, MF0, k0, k1, iv_tensor, iv_out, iv_in, D, MF, &peak[b], &argmax[b], &min_resident[b]);
    }
    free(D);
    free(row);
    return OR_OK;
}

/* One more interval per plan, applied to footprint rows that already exist (Alg. 3
 * analyses the peak again after every scheduled tensor, section IV-C; only the
 * steps o+1 .. r-1 of the row change when (i, o, r) joins the plan).  Row b loses
 * size[i_b] during those steps if the interval can be applied (otherwise it stays
 * as it is); peak, earliest peak step (strict '>' as in Alg. 1) and minimum are
 * taken over the whole row again. */
int oracle_apply_intervals(int32_t T, int32_t N, const int64_t *size, int64_t B, const int32_t *tensor,
                           const int32_t *out, const int32_t *in, int64_t *resident, int64_t *peak, int32_t *argmax,
                           int64_t *min_resident) {
    if (T <= 0 || N < 0 || B < 0) return OR_E_INVAL;
    for (int64_t b = 0; b < B; ++b) {
        int64_t *row = resident + b * (int64_t)T;
        if (interval_applies(N, T, tensor[b], out[b], in[b]))
            for (int32_t t = out[b] + 1; t < in[b]; ++t) row[t] -= size[tensor[b]];
        int64_t mx = row[0], mn = row[0];
        int32_t arg = 0;
        for (int32_t t = 1; t < T; ++t) {
            if (row[t] > mx) {
                mx = row[t];
                arg = t;
            }
            if (row[t] < mn) mn = row[t];
        }
        peak[b] = mx;
        argmax[b] = arg;
        if (min_resident) min_resident[b] = mn;
    }
    return OR_OK;
}

/* Per-workload peaks (section III-A): the footprint MF_j of workload W_j sums
 * Mem over the accesses and schedule events of that workload only, MP_j is its
 * maximum, and for workloads that run asynchronously the global peak is taken as
 * the sum of the MP_j.  Here: job j owns the tensors with job_id[i] == j; its
 * timeline counts those tensors (generated at alloc, released after free) and the
 * plan's intervals on them; the job-independent base_bytes belongs to no job and
 * is left to the caller.  job_peak[j*B + b], job_arg[j*B + b] (earliest step of
 * the maximum, strict comparison as in Alg. 1). */
int oracle_eval_per_job(int32_t T, int32_t N, int32_t J, const int64_t *size, const int32_t *alloc,
                        const int32_t *free_step, const int32_t *job_id, int64_t B, const int64_t *plan_offsets,
                        int64_t n_intervals, const int32_t *iv_tensor, const int32_t *iv_out, const int32_t *iv_in,
                        int64_t *job_peak, int32_t *job_arg) {
    if (T <= 0 || N < 0 || J <= 0 || B < 0) return OR_E_INVAL;
    int64_t *D = (int64_t *)malloc(((size_t)T + 1) * sizeof(int64_t));
    if (!D) return OR_E_NOMEM;
    for (int64_t b = 0; b < B; ++b) {
        int64_t k0, k1;
        plan_range(plan_offsets, b, n_intervals, &k0, &k1);
        for (int32_t j = 0; j < J; ++j) {
            memset(D, 0, ((size_t)T + 1) * sizeof(int64_t));
            for (int32_t i = 0; i < N; ++i) {
                if ((job_id ? job_id[i] : 0) != j) continue;
                D[alloc[i]] += size[i];
                D[free_step[i] + 1] -= size[i];
            }
            for (int64_t k = k0; k < k1; ++k) {
                int32_t i = iv_tensor[k], o = iv_out[k], r = iv_in[k];
                if (!interval_applies(N, T, i, o, r) || (job_id ? job_id[i] : 0) != j) continue;
                D[o + 1] -= size[i];
                if (r < T) D[r] += size[i];
            }
            int64_t run = D[0], peak = D[0];
            int32_t arg = 0;
            for (int32_t t = 1; t < T; ++t) {
                run += D[t];
                if (run > peak) {
                    peak = run;
                    arg = t;
                }
            }
            job_peak[(int64_t)j * B + b] = peak;
            if (job_arg) job_arg[(int64_t)j * B + b] = arg;
        }
    }
    free(D);
    return OR_OK;
}

/* Cumulative operator latency C[0..T] (C[0] = 0) and transfer time
 * x_i = ceil(size_i * 1000 / link_bytes_per_us) in ns.  step_ns == NULL means
 * no timing information: C == 0 and x == 0 (every window is the whole gap). */
int oracle_times(int32_t T, int32_t N, const int64_t *size, const int64_t *step_ns, int64_t link_bytes_per_us,
                 int64_t *C, int64_t *x) {
    if (T <= 0 || N < 0) return OR_E_INVAL;
    C[0] = 0;
    for (int32_t t = 0; t < T; ++t) C[t + 1] = C[t] + (step_ns ? step_ns[t] : 0);
    for (int32_t i = 0; i < N; ++i) {
        if (!step_ns)
            x[i] = 0;
        else {
            if (link_bytes_per_us <= 0) return OR_E_INVAL;
            x[i] = (size[i] * 1000 + link_bytes_per_us - 1) / link_bytes_per_us;
        }
    }
    return OR_OK;
}

/* Occupancy of the host link by the transfers of each plan, step by step (section
 * IV-C, "Swap Event Scheduling": transfers use the PCIe channel exclusively, so
 * only one tensor is in flight at a time; a plan respects that iff no step is
 * occupied twice).  The plan format stores, for a swap (kind 0) of tensor i, only
 * o (last resident step) and r (step the bytes are back); the transfers are read
 * in their canonical, shortest form:
 *   - the swap-out finishes with step o: it occupies the steps s..o for the
 *     LATEST s with C[o+1] - C[s] >= x_i (step 0 if even that is too short);
 *   - the swap-in finishes right before step r (section IV-B situation 3): it
 *     occupies s'..r-1 for the latest s' with C[r] - C[s'] >= x_i (likewise).
 * Any real placement that ends at the same steps occupies at least these steps.
 * Recomputation intervals (kind != 0) use no link; without latencies (x == 0)
 * nothing is occupied.  Inapplicable intervals are skipped as everywhere.
 * reuse != 0: the copy in host memory stays until the tensor's last access
 * (section III-C, "Swap Event"), so of several swap-outs of one tensor in a plan
 * only the earliest (smallest o) transfers anything; every swap-in transfers.
 * Out, per plan: link[b*T + t] (may be NULL), peak[b] = max_t, argmax[b] = earliest
 * step of the maximum, overbooked[b] = number of steps occupied more than once. */
int oracle_link_occupancy(int32_t T, int32_t N, const int64_t *size, const int64_t *step_ns, int64_t link_bytes_per_us,
                          int64_t B, const int64_t *plan_offsets, int64_t n_intervals, const int32_t *iv_tensor,
                          const int32_t *iv_out, const int32_t *iv_in, const uint8_t *iv_kind, int32_t reuse,
                          int32_t *link, int32_t *peak, int32_t *argmax, int32_t *overbooked) {
    if (T <= 0 || N < 0 || B < 0) return OR_E_INVAL;
    int64_t *C = (int64_t *)malloc(((size_t)T + 1) * sizeof(int64_t));
    int64_t *x = (int64_t *)malloc(((size_t)N + 1) * sizeof(int64_t));
    int32_t *L = (int32_t *)malloc((size_t)T * sizeof(int32_t));
    int32_t *first_o = (int32_t *)malloc(((size_t)N + 1) * sizeof(int32_t));
    int rc = OR_E_NOMEM;
    if (!C || !x || !L || !first_o) goto done;
    if ((rc = oracle_times(T, N, size, step_ns, link_bytes_per_us, C, x)) != OR_OK) goto done;
    for (int64_t b = 0; b < B; ++b) {
        int64_t k0, k1;
        plan_range(plan_offsets, b, n_intervals, &k0, &k1);
        for (int32_t t = 0; t < T; ++t) L[t] = 0;
        for (int32_t i = 0; i < N; ++i) first_o[i] = INT32_MAX;
        for (int64_t k = k0; k < k1; ++k) {
            int32_t i = iv_tensor[k], o = iv_out[k], r = iv_in[k];
            if (!interval_applies(N, T, i, o, r) || iv_kind[k] != 0) continue;
            if (o < first_o[i]) first_o[i] = o;
        }
        for (int64_t k = k0; k < k1; ++k) {
            int32_t i = iv_tensor[k], o = iv_out[k], r = iv_in[k];
            if (!interval_applies(N, T, i, o, r) || iv_kind[k] != 0 || x[i] == 0) continue;
            if (!reuse || o == first_o[i]) {
                int32_t s = o;                                   /* walk back until the run is long enough */
                while (s > 0 && C[o + 1] - C[s] < x[i]) --s;
                for (int32_t t = s; t <= o; ++t) ++L[t];
            }
            int32_t s = r - 1;
            while (s > 0 && C[r] - C[s] < x[i]) --s;
            for (int32_t t = s; t <= r - 1; ++t) ++L[t];
        }
        int32_t mx = L[0], arg = 0, over = 0;
        for (int32_t t = 0; t < T; ++t) {
            if (L[t] > mx) {
                mx = L[t];
                arg = t;
            }
            if (L[t] >= 2) ++over;
            if (link) link[b * (int64_t)T + t] = L[t];
        }
        peak[b] = mx;
        if (argmax) argmax[b] = arg;
        if (overbooked) overbooked[b] = over;
    }
    rc = OR_OK;
done:
    free(C); free(x); free(L); free(first_o);
    return rc;
}

/* Candidate score of every tensor for ONE plan whose footprint MF, peak P and
 * peak time tstar are given (section IV-C: the candidates are the tensors that
 * are in GPU memory at the peak, MPTensor of Alg. 1; the paper ranks them by
 * size, here the exact peak reduction of the maximal feasible eviction window
 * is computed, which equals the size when the peak is isolated).
 *   1. gap g of tensor i with p_g < tstar < p_{g+1} (touch points p = alloc,
 *      accesses); a tensor touched at tstar is in use and cannot be swapped
 *      (a swap event may not coincide with an access of its own tensor).
 *   2. zero if the plan already holds an interval of i inside that gap
 *      (Alg. 2 only takes tensors not swapped out yet).
 *   3. swap-out starts right after the access p_g (as early as it can be):
 *      o_i = min{ o >= p_g : C[o+1] - C[p_g+1] >= x_i }.
 *   4. swap-in ends right before the using access (as late as it can be):
 *      r_i = p_{g+1}, using the link during [C[r_i]-x_i, C[r_i]).
 *   5. feasible iff o_i exists, C[o_i+1] + x_i <= C[r_i] (swap-in not earlier
 *      than the swap-out) and o_i < tstar < r_i (swapped out before the peak).
 *   6. score = P - max(PM[o_i], SM[r_i], P - size_i), PM/SM prefix/suffix maxima.
 * win_out/win_in receive (o_i, r_i), or -1 when the tensor is no candidate. */
int oracle_score_plan(int32_t T, int32_t N, const int64_t *size, const int32_t *alloc, const int64_t *access_offsets,
                      const int32_t *access_steps, const int64_t *C, const int64_t *x, int64_t K,
                      const int32_t *iv_tensor, const int32_t *iv_out, const int32_t *iv_in, const int64_t *MF,
                      int64_t P, int32_t tstar, int64_t *score, int32_t *win_out, int32_t *win_in) {
    if (T <= 0 || N < 0) return OR_E_INVAL;
    int64_t *PM = (int64_t *)malloc((size_t)T * sizeof(int64_t));
    int64_t *SM = (int64_t *)malloc((size_t)T * sizeof(int64_t));
    if (!PM || !SM) {
        free(PM);
        free(SM);
        return OR_E_NOMEM;
    }
    PM[0] = MF[0];
    for (int32_t t = 1; t < T; ++t) PM[t] = MF[t] > PM[t - 1] ? MF[t] : PM[t - 1];
    SM[T - 1] = MF[T - 1];
    for (int32_t t = T - 2; t >= 0; --t) SM[t] = MF[t] > SM[t + 1] ? MF[t] : SM[t + 1];

    for (int32_t i = 0; i < N; ++i) {
        score[i] = 0;
        if (win_out) win_out[i] = -1;
        if (win_in) win_in[i] = -1;
        /* 1: touch points p_0 = alloc, p_1.. = accesses */
        int64_t a0 = access_offsets[i], a1 = access_offsets[i + 1];
        int64_t n_touch = 1 + (a1 - a0);
        int32_t pg = -1, pg1 = -1;
        for (int64_t g = 0; g + 1 < n_touch; ++g) {
            int32_t lo = g == 0 ? alloc[i] : access_steps[a0 + g - 1];
            int32_t hi = access_steps[a0 + g];
            if (lo < tstar && tstar < hi) {
                pg = lo;
                pg1 = hi;
                break;
            }
        }
        if (pg < 0) continue;
        /* 2 */
        int blocked = 0;
        for (int64_t k = 0; k < K; ++k) {
            if (iv_tensor[k] != i || !interval_applies(N, T, iv_tensor[k], iv_out[k], iv_in[k])) continue;
            if (pg <= iv_out[k] && iv_in[k] <= pg1) blocked = 1;
        }
        if (blocked) continue;
        /* 3 */
        int32_t oi = -1;
        for (int32_t o = pg; o < T; ++o) {
            if (C[o + 1] - C[pg + 1] >= x[i]) {
                oi = o;
                break;
            }
        }
        if (oi < 0) continue;
        /* 4, 5 */
        int32_t ri = pg1;
        if (!(C[oi + 1] + x[i] <= C[ri])) continue;
        if (!(oi < tstar && tstar < ri)) continue;
        /* 6 */
        int64_t m = P - size[i];
        if (PM[oi] > m) m = PM[oi];
        if (SM[ri] > m) m = SM[ri];
        score[i] = P - m;
        if (win_out) win_out[i] = oi;
        if (win_in) win_in[i] = ri;
    }
    free(PM);
    free(SM);
    return OR_OK;
}

/* Recomputation candidates of ONE plan (section IV-D, "Recomputation
 * Scheduling"): a tensor may be released after an access and regenerated right
 * before its next access, but only if it was never released before, read here as:
 * the plan holds no interval of this tensor at all, in any gap (a tensor already
 * swapped or recomputed somewhere stays out, so that the plan built so far is
 * not disturbed).
 *   1. gap g of tensor i with p_g < tstar < p_{g+1}, as for swapping.
 *   2. zero if the plan holds any applicable interval of tensor i.
 *   3. the window is the whole gap: o = p_g, r = p_{g+1} (no transfer, no link).
 *   4. memory saving = P - max(PM[p_g], SM[p_{g+1}], P - size_i).
 * win_out/win_in receive (p_g, p_{g+1}), or -1 when the tensor is no candidate. */
int oracle_score_recompute_plan(int32_t T, int32_t N, const int64_t *size, const int32_t *alloc,
                                const int64_t *access_offsets, const int32_t *access_steps, int64_t K,
                                const int32_t *iv_tensor, const int32_t *iv_out, const int32_t *iv_in, const int64_t *MF,
                                int64_t P, int32_t tstar, int64_t *score, int32_t *win_out, int32_t *win_in) {
    if (T <= 0 || N < 0) return OR_E_INVAL;
    for (int32_t i = 0; i < N; ++i) {
        score[i] = 0;
        if (win_out) win_out[i] = -1;
        if (win_in) win_in[i] = -1;
        int64_t a0 = access_offsets[i], a1 = access_offsets[i + 1];
        int32_t pg = -1, pg1 = -1, prev = alloc[i];
        for (int64_t k = a0; k < a1; ++k) {
            if (prev < tstar && tstar < access_steps[k]) {
                pg = prev;
                pg1 = access_steps[k];
            }
            prev = access_steps[k];
        }
        if (pg < 0) continue;
        int released = 0;
        for (int64_t k = 0; k < K; ++k)
            if (iv_tensor[k] == i && interval_applies(N, T, iv_tensor[k], iv_out[k], iv_in[k])) released = 1;
        if (released) continue;
        /* maxima outside the window, by direct search */
        int64_t m = P - size[i];
        for (int32_t t = 0; t <= pg; ++t)
            if (MF[t] > m) m = MF[t];
        for (int32_t t = pg1; t < T; ++t)
            if (MF[t] > m) m = MF[t];
        score[i] = P - m;
        if (win_out) win_out[i] = pg;
        if (win_in) win_in[i] = pg1;
    }
    return OR_OK;
}

/* Options of the greedy planner (Alg. 3's hyper-parameters). */
typedef struct {
    int32_t max_iters;        /* hard cap on accepted intervals */
    int32_t min_iters;        /* the paper's 100: the stall rule only applies after it */
    int32_t stop_at_budget;   /* stop once the peak is within the budget */
    int32_t J;                /* jobs, for the swapping-rate limit (0 = off) */
    const int32_t *job_id;    /* [N] */
    const int64_t *msr_num;   /* [J] max swapping rate of job j = msr_num[j]/msr_den */
    int64_t msr_den;
    int32_t recompute;        /* run the recomputation phase while the peak exceeds the budget */
} oracle_greedy_opts;

typedef struct {
    int32_t tensor;
    int64_t score, size;
    int64_t time;             /* recomputation phase only: latency of the generating operator */
} cand_t;

static int cand_cmp(const void *pa, const void *pb) {
    const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
    if (a->score != b->score) return a->score > b->score ? -1 : 1;
    if (a->size != b->size) return a->size > b->size ? -1 : 1;
    return a->tensor < b->tensor ? -1 : (a->tensor > b->tensor ? 1 : 0);
}

/* Recomputation candidates in the order of their value MSPS = memory saving /
 * recomputation time (section IV-D), largest first; the quotients are compared
 * exactly by cross-multiplication.  Ties: larger saving, larger tensor, lower id. */
static int msps_cmp(const void *pa, const void *pb) {
    const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
    __int128 l = (__int128)a->score * b->time, r = (__int128)b->score * a->time;
    if (l != r) return l > r ? -1 : 1;
    return cand_cmp(pa, pb);
}

/* Swap phase of Alg. 3 with Alg. 2's placement, one interval per iteration:
 * analyse the peak (Alg. 1), order the candidates by (score desc, size desc,
 * tensor id asc), place the swap-out as early and the swap-in as late as the
 * exclusive host link allows at step resolution, accept the first candidate
 * whose placed window still contains the peak step; stop when nothing is
 * accepted, at max_iters, at the budget if asked, or when the last three
 * iterations lowered the peak by less than 0.05% after min_iters iterations.
 * With opt->recompute, once no swap is accepted and while the peak is above the
 * budget, recomputation intervals (kind 1) are added one per iteration, the
 * candidate with the largest MSPS first (oracle_score_recompute_plan, msps_cmp),
 * under the same stop rules.
 * The first n_initial entries of the interval arrays are a plan to extend (kept
 * as they are; their transfers are not entered into the link timeline).
 * peak_trace[k] is the peak before the k-th newly accepted interval
 * (peak_trace[*n_out - n_initial] = final peak).  xfer_out_start/xfer_in_start
 * (optional, indexed like the intervals) receive the first link step of the
 * swap-out and of the swap-in of each new interval, -1 if it needs no link time. */
int oracle_greedy(int32_t T, int32_t N, const int64_t *size, const int32_t *alloc, const int32_t *free_step,
                  const int64_t *access_offsets, const int32_t *access_steps, const int64_t *step_ns,
                  int64_t base_bytes, int64_t link_bytes_per_us, int64_t budget, const oracle_greedy_opts *opt,
                  int32_t capacity, int32_t n_initial, int32_t *iv_tensor, int32_t *iv_out, int32_t *iv_in,
                  uint8_t *iv_kind, int32_t *n_out, int64_t *peak_trace, int64_t *final_peak,
                  int32_t *xfer_out_start, int32_t *xfer_in_start) {
    if (T <= 0 || N < 0 || capacity < 0 || n_initial < 0 || n_initial > capacity) return OR_E_INVAL;
    int rc = OR_OK;
    int64_t *MF0 = malloc((size_t)T * 8), *MF = malloc((size_t)T * 8), *D = malloc(((size_t)T + 1) * 8);
    int64_t *C = malloc(((size_t)T + 1) * 8), *x = malloc((size_t)(N + 1) * 8), *score = malloc((size_t)(N + 1) * 8);
    int32_t *wo = malloc((size_t)(N + 1) * 4), *wi = malloc((size_t)(N + 1) * 4);
    cand_t *cand = malloc((size_t)(N + 1) * sizeof(cand_t));
    uint8_t *link_busy = calloc((size_t)T, 1);
    int64_t *hist = malloc(((size_t)capacity + 2) * 8);
    int64_t *SON = calloc((size_t)(opt->J > 0 ? opt->J : 1), 8);
    if (!MF0 || !MF || !D || !C || !x || !score || !wo || !wi || !cand || !link_busy || !hist || !SON) {
        rc = OR_E_NOMEM;
        goto done;
    }
    if ((rc = oracle_base_timeline(T, N, size, alloc, free_step, base_bytes, MF0)) != OR_OK) goto done;
    if ((rc = oracle_times(T, N, size, step_ns, link_bytes_per_us, C, x)) != OR_OK) goto done;

    int32_t iter = n_initial;
    int64_t P = 0, son_total = 0;
    int swap_phase = 1;
    for (;;) {
        int32_t tstar;
        int64_t mn;
        eval_one(T, N, size, MF0, 0, iter, iv_tensor, iv_out, iv_in, D, MF, &P, &tstar, &mn);
        const int32_t it = iter - n_initial;     /* Alg. 3's iteration counter */
        hist[it] = P;
        if (peak_trace) peak_trace[it] = P;
        if (it >= opt->max_iters || iter >= capacity) break;
        if (opt->stop_at_budget && P <= budget) break;
        if (it > opt->min_iters && it >= 3 && (hist[it - 3] - P) * 10000 < 5 * hist[it - 3]) break;

        int accepted = 0;
        int32_t nc = 0;
        if (swap_phase) {
            rc = oracle_score_plan(T, N, size, alloc, access_offsets, access_steps, C, x, iter, iv_tensor, iv_out, iv_in,
                                   MF, P, tstar, score, wo, wi);
            if (rc != OR_OK) goto done;
            for (int32_t i = 0; i < N; ++i) {
                if (wo[i] < 0) continue;
                if (opt->J > 0 && opt->msr_num) {   /* per-job max swapping rate (section IV-C) */
                    int32_t j = opt->job_id[i];
                    int64_t tot = son_total > 1 ? son_total : 1;
                    if (!(SON[j] * opt->msr_den <= opt->msr_num[j] * tot)) continue;
                }
                cand[nc].tensor = i;
                cand[nc].score = score[i];
                cand[nc].size = size[i];
                cand[nc].time = 1;
                ++nc;
            }
            qsort(cand, (size_t)nc, sizeof(cand_t), cand_cmp);
            for (int32_t c = 0; c < nc && !accepted; ++c) {
                int32_t i = cand[c].tensor;
                /* the gap around tstar: p_g is the last touch point before it, p_{g+1} = wi[i] */
                int32_t pg1 = wi[i], pg = alloc[i];
                for (int64_t k = access_offsets[i]; k < access_offsets[i + 1]; ++k)
                    if (access_steps[k] < tstar) pg = access_steps[k];
                int32_t o_placed, r_placed, a = -1, cc = -1, d = -1;
                if (x[i] == 0) {
                    o_placed = pg;
                    r_placed = pg1;
                } else {
                    /* swap-out: earliest run of free steps [a..o'] from p_g+1 on with C[o'+1]-C[a] >= x */
                    o_placed = -1;
                    int32_t s = pg + 1;
                    while (s <= pg1 - 1 && o_placed < 0) {
                        if (link_busy[s]) {
                            ++s;
                            continue;
                        }
                        int32_t e = s;
                        while (e <= pg1 - 1 && !link_busy[e] && C[e + 1] - C[s] < x[i]) ++e;
                        if (e <= pg1 - 1 && !link_busy[e]) {
                            a = s;
                            o_placed = e;
                        } else
                            s = e + 1;      /* ran into a busy step or the end of the gap */
                    }
                    if (o_placed < 0) continue;
                    /* swap-in: latest run of free steps [c..d], d <= p_{g+1}-1, c > o' */
                    r_placed = -1;
                    int32_t e2 = pg1 - 1;
                    while (e2 > o_placed && r_placed < 0) {
                        if (link_busy[e2]) {
                            --e2;
                            continue;
                        }
                        int32_t s2 = e2;
                        while (s2 > o_placed && !link_busy[s2] && C[e2 + 1] - C[s2] < x[i]) --s2;
                        if (s2 > o_placed && !link_busy[s2]) {
                            cc = s2;
                            d = e2;
                            r_placed = e2 + 1;
                        } else
                            e2 = s2 - 1;
                    }
                    if (r_placed < 0) continue;
                }
                if (!(o_placed < tstar && tstar < r_placed)) continue;
                if (x[i] != 0) {
                    for (int32_t t = a; t <= o_placed; ++t) link_busy[t] = 1;
                    for (int32_t t = cc; t <= d; ++t) link_busy[t] = 1;
                }
                iv_tensor[iter] = i;
                iv_out[iter] = o_placed;
                iv_in[iter] = r_placed;
                iv_kind[iter] = 0;
                if (xfer_out_start) xfer_out_start[iter] = x[i] != 0 ? a : -1;
                if (xfer_in_start) xfer_in_start[iter] = x[i] != 0 ? cc : -1;
                if (opt->J > 0 && opt->job_id) {
                    ++SON[opt->job_id[i]];
                    ++son_total;
                }
                ++iter;
                accepted = 1;
            }
            if (accepted) continue;
            swap_phase = 0;      /* an iteration without a swap event ends swapping for good (Alg. 3) */
        }

        /* Recomputation phase (Alg. 3: only while the peak does not fit; section IV-D): release the
         * candidate with the largest MSPS over its whole gap.  Candidates that save nothing are left out. */
        if (!(opt->recompute && P > budget)) break;
        rc = oracle_score_recompute_plan(T, N, size, alloc, access_offsets, access_steps, iter, iv_tensor, iv_out, iv_in,
                                         MF, P, tstar, score, wo, wi);
        if (rc != OR_OK) goto done;
        nc = 0;
        for (int32_t i = 0; i < N; ++i) {
            if (wo[i] < 0 || score[i] <= 0) continue;
            cand[nc].tensor = i;
            cand[nc].score = score[i];
            cand[nc].size = size[i];
            cand[nc].time = step_ns ? step_ns[alloc[i]] : 1;
            ++nc;
        }
        if (nc == 0) break;
        qsort(cand, (size_t)nc, sizeof(cand_t), msps_cmp);
        iv_tensor[iter] = cand[0].tensor;
        iv_out[iter] = wo[cand[0].tensor];
        iv_in[iter] = wi[cand[0].tensor];
        iv_kind[iter] = 1;
        if (xfer_out_start) xfer_out_start[iter] = -1;
        if (xfer_in_start) xfer_in_start[iter] = -1;
        ++iter;
    }
    *n_out = iter;
    *final_peak = P;
done:
    free(MF0); free(MF); free(D); free(C); free(x); free(score); free(wo); free(wi); free(cand); free(link_busy);
    free(hist); free(SON);
    return rc;
}
