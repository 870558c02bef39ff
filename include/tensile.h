/* tensile.h - batched evaluation of GPU-memory footprint timelines over a tensor
 * access sequence (TAS) for candidate swap/recompute plans, on one AMD MI355X.
 *
 * This is the data-parallel core of the plan generation of TENSILE (arXiv
 * 2105.13336): the GPU memory peak analysis (section IV-B, Alg. 1), which the
 * paper re-runs after every scheduled tensor, the choice of the candidate
 * tensor among those resident at the peak (section IV-C) and the greedy loop
 * around them (Alg. 2, Alg. 3).  All quantities are integers; results are
 * exact.
 *
 * Step model.  The paper's time axis is continuous; here it is indexed by
 * steps t in [0,T), one operator-execution slot each, in execution order
 * (section III-A "Workload").  Tensor i is resident from the step of its
 * tensor-generating access, alloc_step[i], through free_step[i], the step of
 * its last tensor-using access (activity analysis, section IV-E), or
 * alloc_step[i] if nobody reads it.  Its touch points are p_0 = alloc_step[i],
 * p_1.. = its access steps.
 *   MF0[t]  = base_bytes + sum_i size[i] * [alloc_step[i] <= t <= free_step[i]]      (Eq. 1, no events)
 * A plan is a set of intervals (tensor i, out o, in r, kind): tensor i is NOT
 * resident during steps o+1 .. r-1.  o is the last step the bytes are still
 * there (end of the swap-out, or of the using access if later - situation 4 of
 * section IV-B; release after an access for recomputation - situation 5); r is
 * the step the bytes are back (the swap-in's finishing point - situation 3).
 *   MF_b[t] = MF0[t] - sum_{(i,o,r) in plan b} size[i] * [o < t < r]                 (Eq. 1)
 *   peak_b  = max_t MF_b[t]                                                          (Eq. 2)
 *   argmax_b = the smallest t attaining it (Alg. 1 updates on a strict '>').
 * An interval that cannot be applied (i outside [0,N), o < 0, r > T, r <= o)
 * is skipped by every entry point; an endpoint at r == T is dropped.  Offsets
 * in plan_offsets are clamped to [0, n_intervals].  Apart from that, plan
 * semantics (interval inside one gap of its tensor, one interval per gap) are
 * NOT checked on the fast path: the arithmetic above is applied as written and
 * min_resident < 0 is the cheap tell-tale; tensile_validate_plans checks them.
 *
 * Conventions.  Every function returns TENSILE_OK (0) or a negative error
 * code, never throws or aborts; tensile_last_error() gives a thread-local
 * message for the last failure.  "HOST" / "DEVICE" says where a pointer must
 * live.  Device buffers are caller-owned (any HIP allocation, e.g. a torch
 * tensor's data_ptr()).  eval/score/link/apply are asynchronous: they enqueue
 * on the given HIP stream (hipStream_t passed as void*, NULL = the default
 * stream) and return; they never wait for the device.
 *
 * Concurrency.  A loaded handle is read-only for every entry point except
 * tensile_tas_update_latencies and tensile_tas_free: any number of host
 * threads may call the others on one handle at the same time, on the same or
 * on different streams.  Scratch memory (partial results, flags, staging) is
 * kept per (handle, stream): calls on one stream run in order and share it,
 * calls on different streams use different memory.  A call that needs more
 * scratch than any earlier call on its stream allocates it (hipMalloc; the
 * memory it replaces is kept until the handle is freed, since kernels enqueued
 * earlier may still use it); a caller that cannot allocate at some point (a
 * stream being captured into a graph, say) first makes one call of the largest
 * shape on that stream, or uses tensile_eval_plans_static.  The two tables
 * that are built on first use (tensile_score_recompute,
 * tensile_eval_plans_per_job) are built by whichever thread comes first while
 * the others wait.  A stream must outlive the calls enqueued on it.
 */
#ifndef TENSILE_H
#define TENSILE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TENSILE_OK 0
#define TENSILE_E_INVAL (-1)    /* NULL pointer, non-positive size, inconsistent arguments        */
#define TENSILE_E_RANGE (-2)    /* an index or step outside its range in a TAS description         */
#define TENSILE_E_NOMEM (-3)    /* host or device allocation failed                                */
#define TENSILE_E_HIP (-4)      /* a HIP runtime call failed (message has the HIP error string)    */
#define TENSILE_E_CAPACITY (-5) /* an output buffer of the stated capacity is too small            */

/* Thread-local description of the last error on this thread ("" if none). */
const char *tensile_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int tensile_version(void);

/* ------------------------------------------------------------------ TAS */

typedef struct tensile_tas tensile_tas; /* opaque; owns device copies and scratch */

/* Problem statement of section III-A in structure-of-arrays form.  All
 * pointers are HOST pointers; the arrays are copied, the caller keeps them. */
typedef struct {
    int32_t T, N, J;               /* steps, tensors, jobs (J >= 1)                                  */
    const int64_t *size_bytes;     /* [N]   > 0                                                      */
    const int32_t *alloc_step;     /* [N]   in [0,T)                                                 */
    const int32_t *free_step;      /* [N]   == last access step, or alloc_step if no access          */
    const int64_t *access_offsets; /* [N+1] CSR over tensors into access_steps, offsets[0] == 0      */
    const int32_t *access_steps;   /* per tensor strictly increasing, every one > alloc_step, < T    */
    const int32_t *job_id;         /* [N] in [0,J), or NULL (all job 0)                              */
    const int64_t *step_ns;        /* [T] operator latency > 0, or NULL: no timing, transfers free   */
    int64_t base_bytes;            /* initial space of the runtime libraries (section IV-B sit. 1)   */
    int64_t link_bytes_per_us;     /* host link bandwidth (64 GB/s = 64000); > 0 if step_ns != NULL  */
} tensile_tas_desc;

/* Validates the description (E_INVAL / E_RANGE name the first violation in
 * tensile_last_error), copies it to the current HIP device and builds there:
 * MF0[T] (same scatter + scan kernels as plan evaluation), the cumulative
 * latency C[T+1], the transfer times x_i = ceil(size_i*1000/link_bytes_per_us)
 * ns, and for every gap between touch points its earliest feasible swap-out
 * step (section IV-C: swap-out as early as possible after the previous access,
 * swap-in as late as possible before the next one, the two must not overlap).
 * Synchronous.  *out is NULL on failure. */
int tensile_tas_load(const tensile_tas_desc *desc, tensile_tas **out);

/* Releases the handle and everything it owns (synchronises the device). NULL is allowed. */
void tensile_tas_free(tensile_tas *tas);

/* Peak and earliest peak step of the unscheduled timeline MF0 (either output may be NULL). */
int tensile_tas_info(const tensile_tas *tas, int64_t *unscheduled_peak, int32_t *argmax);

/* New operator latencies for a loaded sequence (section IV-E, "Scheduling Plan
 * Updating": when the measured latencies have drifted, the plan is regenerated
 * from the corrected sequence).  Latencies do not enter the footprint, so only
 * what depends on them is rebuilt: cumulative latency, transfer times, every
 * gap's earliest swap-out step and the swap-candidate index; footprints that were
 * evaluated before stay valid and can be scored again.  step_ns: HOST [T], all
 * > 0, or NULL for "no latencies"; link_bytes_per_us > 0 when step_ns is given.
 * Synchronous (waits for the device first).  The caller must not run any other
 * call on this handle at the same time. */
int tensile_tas_update_latencies(tensile_tas *tas, const int64_t *step_ns, int64_t link_bytes_per_us);

/* Copies MF0 into a HOST buffer of T words (synchronous). */
int tensile_tas_base_timeline(const tensile_tas *tas, int64_t *mf0_host);

/* ---------------------------------------------------------------- plans */

/* A batch of B plans in CSR form.  DEVICE pointers, caller-owned, read-only.
 * Intervals of plan b are entries plan_offsets[b] .. plan_offsets[b+1]-1, in
 * any order.  Performance note: the kernels size their per-thread interval
 * lists from n_intervals / B, the only length the host knows without reading
 * the offsets back.  A batch that is a window into larger arrays (offsets that
 * start far above 0 or end far below n_intervals) is still evaluated exactly,
 * but with lists sized for plans it does not hold; pass the window's own
 * arrays and rebased offsets instead. */
typedef struct {
    int32_t B;                   /* plans, >= 0                                                     */
    int64_t n_intervals;         /* length of the four interval arrays (host-known)                 */
    const int64_t *plan_offsets; /* [B+1]                                                           */
    const int32_t *iv_tensor;    /* [n_intervals] tensor index                                      */
    const int32_t *iv_out;       /* [n_intervals] o: last resident step                             */
    const int32_t *iv_in;        /* [n_intervals] r: step the bytes are back                        */
    const uint8_t *iv_kind;      /* [n_intervals] 0 swap, 1 recompute; may be NULL (all swap).      *
                                  * The kind does not change the footprint (Alg. 1 treats a release  *
                                  * for recomputation like a swap-out).                              */
} tensile_plans;

/* Memory peak analysis of B plans at once (Eq. 1, Eq. 2, Alg. 1).
 *   resident     DEVICE [B*T] row-major, t fastest: MF_b[t]; may be NULL (peaks only)
 *   peak         DEVICE [B]   max_t MF_b[t]
 *   argmax       DEVICE [B]   earliest t with MF_b[t] == peak[b]
 *   min_resident DEVICE [B]   min_t MF_b[t]; may be NULL
 * Asynchronous on hip_stream.  B == 0 is a no-op. */
int tensile_eval_plans(const tensile_tas *tas, const tensile_plans *plans, int64_t *resident, int64_t *peak,
                       int32_t *argmax, int64_t *min_resident, void *hip_stream);

/* tensile_eval_plans for callers that cannot allocate: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same results, same kernels; the scratch memory (per-segment
 * partial results, the launch flag, the sorted endpoint records of batches of
 * long plans) lives in a 16 MiB device array that is part of the library's
 * code object instead of the handle's per-stream workspaces, and the call makes
 * no allocation of any kind on host or device paths of the HIP runtime
 * (no hipMalloc / hipFree / allocating library routine).  Every GPU the library
 * runs on holds its own copy of the array until the process ends.
 *   Limits: the per-segment partials (20 bytes per plan and segment, only when
 *   a plan is split into several segments: batches of fewer plans than the GPU
 *   has compute units, or rows of millions of steps) must fit the 16 MiB, else
 *   TENSILE_E_CAPACITY with the sizes in tensile_last_error() and nothing is
 *   enqueued.  Batches whose average plan exceeds about 5,400 intervals are
 *   sorted by tile first when the records (16 bytes per interval + 12 bytes per
 *   plan and 8192 steps) fit what is left; otherwise they are evaluated from
 *   their lists as they are, exactly but more slowly.
 *   The handle must live on the current device (TENSILE_E_INVAL otherwise).
 *   All calls on one GPU share that GPU's array, whatever the handle or stream:
 *   calls that may overlap in time on one GPU (different streams, or different
 *   host threads without a common stream order) race on it and give wrong
 *   results; order them on one stream.  Nothing in the array needs to start
 *   at zero between calls.
 * Asynchronous on hip_stream.  B == 0 is a no-op. */
int tensile_eval_plans_static(const tensile_tas *tas, const tensile_plans *plans, int64_t *resident, int64_t *peak,
                              int32_t *argmax, int64_t *min_resident, void *hip_stream);

/* Per-workload peaks (section III-A: the footprint MF_j of workload W_j counts
 * the accesses and schedule events of that workload alone, MP_j is its maximum,
 * and the global peak of workloads that run asynchronously is the sum of the
 * MP_j).  Job j owns the tensors with job_id[i] == j; base_bytes belongs to no
 * job.  For every plan b and job j:
 *   MF_{b,j}[t] = sum of size_i over job j's tensors resident at t under plan b
 *   job_peak[j*B + b]   = max_t MF_{b,j}[t]           (job-major layout)
 *   job_argmax[j*B + b] = earliest step attaining it  (may be NULL)
 *   sum_peak[b]         = base_bytes + sum_j job_peak[j*B + b]   (may be NULL)
 * With one job, sum_peak equals tensile_eval_plans' peak.  sum_peak >= peak
 * always.  DEVICE outputs.  Runs the evaluation kernel once per job without
 * writing footprint rows; the first call on a handle builds per-job tables
 * (synchronous, allocates), later calls are asynchronous on hip_stream. */
int tensile_eval_plans_per_job(const tensile_tas *tas, const tensile_plans *plans, int64_t *job_peak,
                               int32_t *job_argmax, int64_t *sum_peak, void *hip_stream);

/* Per-tensor candidate scores for every plan (section IV-C: the candidates are
 * the tensors resident and idle at the peak; the paper orders them by size,
 * this returns the exact peak reduction, which is the size when the peak is
 * isolated).  For plan b with t* = argmax[b], P = peak[b], tensor i:
 *   1. gap g with p_g < t* < p_{g+1}; none -> 0 (not resident, or in use at t*)
 *   2. plan b already has an applicable interval of i with p_g <= o and r <= p_{g+1} -> 0
 *   3. o_i = min{ o >= p_g : C[o+1] - C[p_g+1] >= x_i }   (swap-out as early as possible)
 *   4. r_i = p_{g+1}                                     (swap-in as late as possible)
 *   5. feasible iff o_i exists, C[o_i+1] + x_i <= C[r_i] and o_i < t* < r_i; else 0
 *   6. score = P - max( max_{t<=o_i} MF_b[t], max_{t>=r_i} MF_b[t], P - size_i )
 *            = P - peak(plan b + (i, o_i, r_i)),  0 <= score <= size_i.
 * Exclusive use of the link is not considered here (only transfer duration);
 * tensile_greedy_plan places transfers on the link.
 *   resident, peak, argmax  DEVICE, as produced by tensile_eval_plans for the same plans
 *   score    DEVICE [B*N]
 *   win_out  DEVICE [B*N] o_i, or -1 where steps 1, 2 or 5 reject; may be NULL
 *   win_in   DEVICE [B*N] r_i, or -1; may be NULL
 * Asynchronous on hip_stream. */
int tensile_score_candidates(const tensile_tas *tas, const tensile_plans *plans, const int64_t *resident,
                             const int64_t *peak, const int32_t *argmax, int64_t *score, int32_t *win_out,
                             int32_t *win_in, void *hip_stream);

/* Peak analysis and candidate scores of B plans in one call: the body of the
 * loop of Alg. 3, where the memory peak analysis (Alg. 1) is immediately
 * followed by the choice among the tensors resident at the peak (section IV-C).
 * Outputs and their meaning are exactly those of tensile_eval_plans followed by
 * tensile_score_candidates on the same batch (resident is required here, the
 * scores are computed from it); the two kernels are enqueued back to back
 * under one lock of the stream's workspace.  Asynchronous on hip_stream.
 * B == 0 is a no-op. */
int tensile_eval_score_plans(const tensile_tas *tas, const tensile_plans *plans, int64_t *resident, int64_t *peak,
                             int32_t *argmax, int64_t *min_resident, int64_t *score, int32_t *win_out, int32_t *win_in,
                             void *hip_stream);

/* Recomputation savings for every plan (section IV-D, "Recomputation
 * Scheduling": recomputation is applied only to tensors that have never been
 * released, and valued by the memory it saves).  Tensor i may be dropped after
 * an access and regenerated right before the next one; no transfer is involved,
 * so the window is the whole gap.  For plan b with t* = argmax[b], P = peak[b]:
 *   1. gap g with p_g < t* < p_{g+1}; none -> 0
 *   2. plan b holds any applicable interval of tensor i (any gap, any kind) -> 0
 *   3. score = P - max( max_{t<=p_g} MF_b[t], max_{t>=p_{g+1}} MF_b[t], P - size_i )
 *            = P - peak(plan b + (i, p_g, p_{g+1}))
 * Arguments as for tensile_score_candidates; win_out/win_in receive p_g and
 * p_{g+1}, or -1.  The first call on a handle builds a second candidate index
 * (synchronous, allocates); later calls are asynchronous on hip_stream. */
int tensile_score_recompute(const tensile_tas *tas, const tensile_plans *plans, const int64_t *resident,
                            const int64_t *peak, const int32_t *argmax, int64_t *score, int32_t *win_out,
                            int32_t *win_in, void *hip_stream);

/* Slow semantic check of a batch (synchronous; copies the plans to the host).
 * Valid means: applicable (see top), p_g <= o and r <= p_{g+1} for one gap g of
 * the tensor (section IV-C: a swap may not overlap the tensor's own accesses;
 * swap-in not later than the using access), and at most one interval per
 * (plan, tensor, gap).  *first_bad (HOST) receives the index of the first
 * offending interval or -1; *reason (HOST, may be NULL) 1 = not applicable,
 * 2 = not inside one gap, 3 = second interval in a gap, 4 = bad plan_offsets. */
int tensile_validate_plans(const tensile_tas *tas, const tensile_plans *plans, int64_t *first_bad, int32_t *reason);

/* Windowed re-evaluation: plan b gains ONE interval (tensor[b], out_step[b],
 * in_step[b]) and its footprint row, which exists already, is brought up to
 * date in place.  Alg. 3 analyses the peak again after every tensor it
 * schedules (section IV-C); only the steps out_step+1 .. in_step-1 of the row
 * change, so nothing but that window is written and the plan's other
 * intervals are not read again.  The result is the one tensile_eval_plans
 * gives for the extended plan.
 *   tensor, out_step, in_step  DEVICE [B]; an interval that cannot be applied
 *                (see tensile_eval_plans) leaves its row as it is
 *   resident     DEVICE [B*T] in/out: rows as tensile_eval_plans wrote them
 *   peak, argmax DEVICE [B] out: of the updated rows
 *   min_resident DEVICE [B] out; may be NULL
 * Asynchronous on hip_stream.  B == 0 is a no-op. */
int tensile_apply_intervals(const tensile_tas *tas, int32_t B, const int32_t *tensor, const int32_t *out_step,
                            const int32_t *in_step, int64_t *resident, int64_t *peak, int32_t *argmax,
                            int64_t *min_resident, void *hip_stream);

/* Occupancy of the host link by the transfers of each plan (section IV-C, "Swap
 * Event Scheduling": a transfer occupies the PCIe channel exclusively, only one
 * tensor can be on its way at a time).  A swap interval (i, o, r) of a timed
 * sequence is read as two transfers of x_i ns in their shortest form: the
 * swap-out ends with step o and occupies s..o for the latest s with
 * C[o+1] - C[s] >= x_i, the swap-in ends right before step r and occupies
 * s'..r-1 for the latest s' with C[r] - C[s'] >= x_i (C = cumulative step
 * latency; from step 0 if the past is too short).  Any real placement that ends
 * at the same steps occupies at least these steps, so link_peak[b] <= 1 is
 * necessary for plan b to respect the exclusive channel, and sufficient for the
 * placement of tensile_greedy_plan, whose plans always satisfy it.
 * Recomputation intervals (kind 1) and sequences without latencies occupy nothing.
 *   reuse_host_copies  non-zero: the copy in host memory stays until the tensor's
 *                last access (section III-C, "Swap Event"), so of several swap-outs
 *                of one tensor in a plan only the earliest (smallest o) transfers
 *   link         DEVICE [B*T] int32 row-major: transfers on the link at step t; may be NULL
 *   link_peak    DEVICE [B]   max_t link_b[t]
 *   link_argmax  DEVICE [B]   earliest step of the maximum; may be NULL
 *   overbooked   DEVICE [B]   number of steps with link_b[t] >= 2; may be NULL
 * Inapplicable intervals are skipped as in tensile_eval_plans.  Sequences of
 * more than 2^28 steps are refused (TENSILE_E_RANGE).
 * Asynchronous on hip_stream.  B == 0 is a no-op. */
int tensile_eval_link(const tensile_tas *tas, const tensile_plans *plans, int32_t reuse_host_copies, int32_t *link,
                      int32_t *link_peak, int32_t *link_argmax, int32_t *overbooked, void *hip_stream);

/* --------------------------------------------------------------- greedy */

/* Hyper-parameters of the complete scheduling algorithm (Alg. 3). */
typedef struct {
    int32_t max_iters;      /* at most this many new intervals (<= 0: no limit)                      */
    int32_t min_iters;      /* the stall rule applies only after this many iterations (paper: 100)   */
    int32_t stop_at_budget; /* non-zero: stop as soon as peak <= budget_bytes                        */
    const int64_t *msr_num; /* HOST [J] max swapping rate of job j = msr_num[j]/msr_den (section     *
                             * IV-C); a tensor of job j is a candidate while                         *
                             * swapped[j]*msr_den <= msr_num[j]*max(1, total swapped). NULL = off.   */
    int64_t msr_den;
    int32_t recompute;      /* non-zero: once no swap is accepted and while peak > budget_bytes, add *
                             * recomputation intervals (kind 1), see tensile_greedy_plan             */
} tensile_greedy_opts;

/* Swap phase of Alg. 3 with the placement of Alg. 2, one interval per
 * iteration: evaluate the current plan (tensile_eval_plans, B = 1), score the
 * candidates (tensile_score_candidates), order them by (score desc, size desc,
 * tensor asc), and for each in turn place the swap-out on the earliest run of
 * consecutive free link steps after p_g whose duration covers x_i and the
 * swap-in on the latest such run before p_{g+1} (the link carries one transfer
 * at a time, section IV-C); accept the first candidate whose placed window
 * (o', d+1) still has o' < t* < d+1.  Stops when no candidate is accepted, at
 * max_iters, at capacity, at the budget if asked, or when, after min_iters
 * iterations, the last three lowered the peak by less than 0.05 %.
 * Recomputation branch of Alg. 3 (opts->recompute): when an iteration accepts no
 * swap, swapping is over; from then on, while peak > budget_bytes, each iteration
 * scores the tensors with tensile_score_recompute, leaves out those that save
 * nothing, and appends (i, p_g, p_{g+1}, kind 1) for the one with the largest
 * MSPS = saving / recomputation time (section IV-D), the time being the latency
 * step_ns[alloc_i] of the operator that generates the tensor (1 without
 * latencies); quotients are compared exactly by cross-multiplication, ties by
 * (saving desc, size desc, tensor asc).  The same stop rules apply.
 * Synchronous; uses the default stream.
 *   capacity    length of the four HOST interval arrays
 *   n_initial   the first n_initial entries are an existing plan to extend (kept; their
 *               transfers are not entered into the link timeline)
 *   n_intervals HOST out: total number of intervals (>= n_initial)
 *   peak_trace  HOST [capacity - n_initial + 1] or NULL: peak before each new interval, last = final
 *   final_peak  HOST out */
int tensile_greedy_plan(const tensile_tas *tas, int64_t budget_bytes, const tensile_greedy_opts *opts,
                        int32_t capacity, int32_t n_initial, int32_t *iv_tensor, int32_t *iv_out, int32_t *iv_in,
                        uint8_t *iv_kind, int32_t *n_intervals, int64_t *peak_trace, int64_t *final_peak);

/* --------------------------------------------------- testing and tuning aids */

/* Forces a launch choice that the library otherwise makes from the shape of the
 * batch (results never depend on it; used by the parity tests to reach every
 * kernel variant on small inputs, and by tuning runs).  Process-wide; set it
 * while no call is in flight.  The library never reads the environment.
 *   "eval_threads"    256 / 512 / 1024: workgroup geometry of the evaluation kernel (0 = automatic)
 *   "eval_segments"   segments per plan (0 = automatic)
 *   "eval_seg_steps"  most steps a segment may hold: rows longer than this are cut, whatever else was chosen
 *                     (0 = 2^28, the kernels' limit; a smaller value only serves to exercise the rule)
 *   "eval_binned"     0 never sort a batch's endpoints by tile first, 1 whenever possible (-1 = automatic)
 *   "eval_persistent" 0 never use the persistent grid, 1 whenever possible (-1 = automatic)
 *   "eval_slots"      size of the persistent grid (0 = automatic)
 *   "eval_nt"         footprint rows written with nontemporal stores: 0 never, 1 whenever compiled for the
 *                     kernel at hand, -1 (default) for rows whose unscheduled timeline exceeds 1 MiB
 *   "eval_r"          intervals per thread kept in registers (0 = automatic)
 *   "score_blocks"    size of the scoring grid (0 = automatic)
 *   "link_packed"     0: search the cumulative latencies themselves even when their packed form exists (1 = automatic)
 *   "step_fused"      1: tensile_eval_score_plans takes each plan through evaluation and scoring in ONE kernel when the
 *                     batch has the shape for it (sizes in 32-bit units, T even and at most 131,072, 16-byte aligned
 *                     rows, plans of at most about 5,400 intervals on average); measured slower than the two kernels,
 *                     hence never chosen automatically (0 / -1: two kernels)
 * TENSILE_E_INVAL for an unknown name. */
int tensile_tuning_set(const char *knob, int value);

/* Back to the automatic choices. */
void tensile_tuning_reset(void);

#ifdef __cplusplus
}
#endif
#endif /* TENSILE_H */
