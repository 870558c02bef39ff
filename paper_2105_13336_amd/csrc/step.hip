// Peak analysis and candidate scores of a batch in one call (the body of the paper's Alg. 3 loop: the memory
// peak analysis of Alg. 1 immediately followed by the choice among the tensors resident at the peak, section
// IV-C): the evaluation kernel and the scoring kernel enqueued back to back, or - on request only - one fused
// kernel.
//
// The fused kernel.  Evaluated and scored by two kernels, the footprint rows travel to HBM and back: the
// scoring kernel re-reads 8 bytes per plan-timestep that the evaluation kernel has just written, and the
// interval lists a second time.  In step_kernel a persistent workgroup takes a plan through both phases back
// to back: the evaluation body (eval_body.h) writes the row and leaves the peak and its step in LDS, the scoring
// body (score_body.h) streams the same row back while it is still in the memory-side cache; the two phases'
// LDS structs share one union (150 KB).  Plain streaming loops of the same shape (16,384 rows of 400 KB, 320 KB
// of output per row, one workgroup per CU) say what there is to gain: write rows + read cold rows + write
// outputs 3.6 ms, write rows + read the row just written + write outputs 2.7 ms.  The real phases do not get
// there: on that batch the fused kernel takes 4.75 ms against 1.68 + 2.80 ms for the two kernels.  A plan's
// phases are paced by instruction issue and by chains of dependent loads inside the one workgroup a CU holds
// (evaluation: about 6,100 cycles per 8192-step tile before any store; scoring: a lone plan takes longer than a
// plan of a full batch), not by HBM, so serving the re-read from cache buys little, while the fusion adds what
// the separate kernels hide: the next plan's cold start (offsets, intervals, sizes: three dependent latencies)
// no longer overlaps the previous workgroup's draining stores, the stores must have landed before the row is
// read back, and the candidate lists and filter that a scoring-only workgroup keeps in LDS from plan to plan
// are reloaded for every plan because the evaluation phase has used the space.  Overlapping the two phases of
// different plans would need two workgroups per CU, i.e. both phases in half the LDS (a second index layout for
// scoring with 8 wavefronts); not built.  The kernel is kept, tested, behind the "step_fused" tuning knob.
#include "eval_body.h"
#include "score_body.h"

namespace tensile {

namespace {

constexpr int kStepThr = 1024;

union StepLds {
    EvalLds<kStepThr> eval;
    ScoreLds<false> score;
};

// R: intervals per thread the evaluation phase keeps in registers; a plan with more than R * 1024 goes through
// the form of the evaluation body that re-reads what does not fit (8192 in registers) per tile.
template <int R, bool kNarrow>
__global__ __launch_bounds__(kStepThr) __attribute__((amdgpu_waves_per_eu(4, 4))) void step_kernel(const EvalArgs ea, const ScoreArgs sa) {
    __shared__ StepLds lds;
    __shared__ Best result;   // the evaluation's (peak, peak step, minimum) on its way to the scoring phase
    ScoreCarry carry;
    typedef const int64_t __attribute__((address_space(4))) *const_i64_ptr;   // (the batch is not written during the launch)
    const const_i64_ptr plan_offsets = (const_i64_ptr)(ea.plan_offsets);
    for (int32_t b = blockIdx.x; b < ea.B; b += gridDim.x) {
        int64_t k0 = plan_offsets[b], k1 = plan_offsets[b + 1];
        if (k0 < 0) k0 = 0;
        if (k1 > ea.n_intervals) k1 = ea.n_intervals;
        if (k1 < k0) k1 = k0;
        if (k1 - k0 <= ea.tail_threshold) eval_body<kStepThr, R, false, kNarrow, 2>(ea, b, 0, lds.eval, &result);
        else eval_body<kStepThr, kCapTail / kStepThr, true, kNarrow, 2>(ea, b, 0, lds.eval, &result);
        // the row this workgroup has written is read back by other wavefronts of it: their loads come after
        // everybody's stores; the barrier also ends the evaluation's use of the LDS
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        const int32_t tstar = __builtin_amdgcn_readfirstlane(result.arg);
        const uint32_t p_lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(result.mx));
        const uint32_t p_hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(static_cast<uint64_t>(result.mx) >> 32));
        const int64_t P = static_cast<int64_t>((static_cast<uint64_t>(p_hi) << 32) | p_lo);
        carry.filter_of = -1;    // (the evaluation has overwritten lists and filter)
        carry.lists_of = -1;
        score_plan<false, true, false>(sa, b, tstar, P, lds.score, nullptr, carry);
        __syncthreads();   // the scoring phase has finished with the LDS (and with `result`)
    }
}

}  // namespace

// The fused pass, or the two kernels one after the other (see the top of the file).
int launch_step(const tensile_tas *tas, Workspace &ws, const tensile_plans *plans, int64_t *resident, int64_t *peak,
                int32_t *argmax, int64_t *min_resident, int64_t *score, int32_t *win_out, int32_t *win_in) {
    const int32_t B = plans->B, T = tas->T;
    EvalArgs ea{};
    ea.T = T; ea.N = tas->N; ea.B = B; ea.o_min = 0; ea.n_intervals = plans->n_intervals;
    ea.plan_offsets = plans->plan_offsets;
    ea.iv_tensor = plans->iv_tensor; ea.iv_out = plans->iv_out; ea.iv_in = plans->iv_in;
    ea.size = tas->d_size.p; ea.size_units = tas->d_size_units.p; ea.size_shift = tas->size_shift;
    ea.MF0 = tas->d_MF0.p; ea.dMF0 = tas->d_dMF0.p; ea.resident = resident;
    const int64_t avg_k = (plans->n_intervals + B - 1) / B;
    const int64_t need = avg_k + avg_k / 8;      // (as the evaluation's own launch sizes its registers)
    const bool vec16 = (T % 2 == 0) && (reinterpret_cast<uintptr_t>(resident) % 16 == 0);
    // (B >= 2: a workgroup's plans are then never neighbours in memory, so no cache line of a row it reads back
    // was ever fetched by its CU before the row was written)
    const bool shape_ok = B >= 2 && tas->N > 0 && ea.size_units != nullptr && vec16 && (T + kMini - 1) / kMini <= kTabLds && need <= kCapBig;
    const bool fused = shape_ok && g_tuning.step_fused == 1;   // (slower than the two kernels where measured: on request only)
    if (!fused) {
        int rc = launch_eval(tas, ws, ea, peak, argmax, min_resident);
        if (rc != TENSILE_OK) return rc;
        return launch_score(tas, ws, tas->index, false, plans, resident, peak, argmax, score, win_out, win_in);
    }
    const int cap = need <= kCapSmall ? kCapSmall : need <= kCapMid ? kCapMid : kCapBig;
    ea.S = 1;
    ea.tiles_per_seg = static_cast<int32_t>((static_cast<int64_t>(T) + kEvalTile - 1) / kEvalTile);
    ea.out_max = peak; ea.out_arg = argmax; ea.out_min = min_resident;
    ea.tail_threshold = cap;
    ea.tail_flag = nullptr;   // (never raised: the kernel takes long plans itself)
    ea.epoch = 0;
    const ScoreArgs sa = make_score_args(tas, tas->index, false, plans, resident, peak, argmax, score, win_out, win_in);
    const int64_t slots = tas->num_cus;       // one workgroup per CU (150 KB of LDS), the plans dealt evenly
    const int64_t rounds = (B + slots - 1) / slots;
    const dim3 grid(static_cast<uint32_t>((B + rounds - 1) / rounds)), block(kStepThr);
    const hipStream_t stream = ws.stream;
    if (cap == kCapSmall) hipLaunchKernelGGL((step_kernel<kCapSmall / kStepThr, true>), grid, block, 0, stream, ea, sa);
    else if (cap == kCapMid) hipLaunchKernelGGL((step_kernel<kCapMid / kStepThr, true>), grid, block, 0, stream, ea, sa);
    else hipLaunchKernelGGL((step_kernel<kCapBig / kStepThr, true>), grid, block, 0, stream, ea, sa);
    TS_HIP(hipGetLastError());
    return TENSILE_OK;
}

}  // namespace tensile

using namespace tensile;

extern "C" int tensile_eval_score_plans(const tensile_tas *tas, const tensile_plans *plans, int64_t *resident, int64_t *peak,
                                        int32_t *argmax, int64_t *min_resident, int64_t *score, int32_t *win_out,
                                        int32_t *win_in, void *hip_stream) {
    int rc = check_plans(tas, plans, "eval_score_plans");
    if (rc != TENSILE_OK) return rc;
    if (plans->B == 0) return TENSILE_OK;
    if (!resident || !peak || !argmax || !score) {
        set_error("eval_score_plans: resident, peak, argmax and score are required");
        return TENSILE_E_INVAL;
    }
    WorkspaceLock ws = acquire_workspace(tas, static_cast<hipStream_t>(hip_stream));
    return launch_step(tas, *ws, plans, resident, peak, argmax, min_resident, score, win_out, win_in);
}
