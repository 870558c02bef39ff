// The fused scatter + scan + reduce body of the evaluation kernels (Eq. 1, Eq. 2 and Alg. 1 of the paper)
// and what it shares with the kernels built around it.  Included by eval.hip (one workgroup per plan and
// segment, persistent and binned forms) and by step.hip (evaluation and scoring of a plan in one workgroup).
// Everything here has internal linkage.
#pragma once

#include "common.h"
#include "wave_ops.h"

#include <type_traits>

namespace tensile {

namespace {

constexpr int kVpt = 8;   // steps per lane per tile: the scan below is written for 8
// intervals per plan held in registers: three sizes for the common kernel, 8192 for the kernel that takes longer plans
constexpr int kCapSmall = 2048, kCapMid = 4096, kCapBig = 6144, kCapTail = 8192;
constexpr int kTailU = 4;   // intervals per thread and round where a long plan's list is re-read (see eval_body)
// LDS layouts are skewed: 16-byte granule g lives at granule g + (g >> 4), i.e. cell u at
// u + 2 * (u >> 5).  A lane's four granules stay contiguous (they never straddle a multiple of 16).
constexpr int kStageCells = 64 * kVpt + 2 * ((64 * kVpt) >> 5) + 2;    // 546 per wave, rounded up below
constexpr int kStageStride = (kStageCells + 7) / 8 * 8;               // 552
// Geometry of a workgroup with kThr threads
template <int kThr>
struct Geom {
    static constexpr int kWaves = kThr / 64;
    static constexpr int kTile = kThr * kVpt;                          // steps per LDS difference tile
    static constexpr int kTileCells = kTile + 2 * (kTile >> 5);
    static_assert(kWaves <= 16 && kTile <= kEvalTile, "wave totals are scanned by 16 lanes; dMF0 is padded for kEvalTile");
};
__device__ __forceinline__ uint32_t skew(uint32_t u) { return u + ((u >> 5) << 1); }
// An interval's endpoints are kept as BYTE offsets of their cells from the segment's first cell (skew is monotone, and
// additive over multiples of 32, so the offset inside a tile is this minus the tile's own).  Segments have at most
// 2^28 + one tile of steps (the host cuts longer rows), so an offset stays below 2.3e9, and kNoCell - for an endpoint
// outside the segment, an interval that is not applied or an empty slot - minus any tile's offset, like the
// wrapped difference of an endpoint before the tile, lies far above the 70 KB of a tile: one unsigned minimum
// with the lane's trash cell sends all of them there.
constexpr uint32_t kNoCell = 0xfffffff8u;
__device__ __forceinline__ uint32_t cell_bytes(int32_t step, int32_t seg_lo, int32_t seg_hi) {
    return step >= seg_lo && step < seg_hi ? skew(static_cast<uint32_t>(step - seg_lo)) * 8u : kNoCell;
}

// LDS of one workgroup of the evaluation body.  A struct, so that a kernel that runs other phases in the
// same workgroup can overlay it with theirs.
template <int kThr>
struct EvalLds {
    // the tile, followed by 64 "trash" cells: a lane whose endpoint lies outside the tile adds to
    // trash[lane] instead (never read), which keeps the scatter free of branches and of
    // execution-mask changes
    __attribute__((aligned(16))) int64_t delta[Geom<kThr>::kTileCells + 64];
    __attribute__((aligned(16))) int64_t stage_all[Geom<kThr>::kWaves * kStageStride];
    int64_t wave_tot[Geom<kThr>::kWaves];
    int64_t carry_part[Geom<kThr>::kWaves];
    int64_t red_mx[Geom<kThr>::kWaves], red_mn[Geom<kThr>::kWaves];
    int32_t red_arg[Geom<kThr>::kWaves];
};

// Workgroup w of a launch -> (plan, segment).  XCD-aware: block w runs on XCD w % 8; XCD x gets the plans
// = x (mod 8), and all segments of a plan run on the same XCD.  False past the end of the batch.
__device__ __forceinline__ bool decode_block(const EvalArgs &a, int64_t w, int32_t &plan, int32_t &seg) {
    const int32_t xcd = static_cast<int32_t>(w & 7);
    const int64_t q = w >> 3;
    const int64_t plan64 = (q / a.S) * 8 + xcd;
    seg = static_cast<int32_t>(q % a.S);
    if (plan64 >= a.B) return false;
    plan = static_cast<int32_t>(plan64);
    return true;
}

struct Best {
    int64_t mx, mn;
    int32_t arg;
};

// (value desc, step asc): the earliest step wins among equal values
__device__ __forceinline__ void best_merge(Best &a, int64_t mx, int32_t arg, int64_t mn) {
    if (mx > a.mx || (mx == a.mx && arg < a.arg)) {
        a.mx = mx;
        a.arg = arg;
    }
    if (mn < a.mn) a.mn = mn;
}

typedef long long ll2 __attribute__((ext_vector_type(2)));

// Sizes are kept in registers either as int64 (kNarrow == false) or, when every
// size is a multiple of 2^size_shift and fits 32 bits after the shift, as uint32
// units (one register less per interval).
template <bool kNarrow>
struct SizeReg;
template <>
struct SizeReg<false> {
    typedef int64_t type;
    static __device__ __forceinline__ type load(const EvalArgs &a, int32_t i) { return a.size[i]; }
    static __device__ __forceinline__ int64_t bytes(const EvalArgs &, type s) { return s; }
};
template <>
struct SizeReg<true> {
    typedef uint32_t type;
    static __device__ __forceinline__ type load(const EvalArgs &a, int32_t i) { return a.size_units[i]; }
    static __device__ __forceinline__ int64_t bytes(const EvalArgs &a, type s) {
        return static_cast<int64_t>(static_cast<uint64_t>(s) << a.size_shift);
    }
};

// Phase timing for tuning, compiled in with -DTENSILE_EVAL_PROF only: thread 0 of every workgroup adds the
// 100 MHz ticks it spent in each part of a tile to g_eval_prof (lane 0 of every wavefront, per wavefront).
#ifdef TENSILE_EVAL_PROF
__device__ unsigned long long g_eval_prof[16 * 8];   // [wavefront][part]
#define EVAL_MARK(k)                                              \
    do {                                                          \
        const unsigned long long now_ = wall_clock64();           \
        prof_acc[k] += now_ - prof_t;                             \
        prof_t = now_;                                            \
    } while (0)
#else
#define EVAL_MARK(k) do { } while (0)
#endif

__device__ __forceinline__ void opaque(uint32_t &x) { asm volatile("" : "+v"(x)); }
__device__ __forceinline__ void opaque(int64_t &x) { asm volatile("" : "+v"(x)); }

__device__ __forceinline__ void lds_add(int64_t *p, int64_t v) {
    __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void lds_sub(int64_t *p, int64_t v) {
    __hip_atomic_fetch_sub(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

__device__ __forceinline__ bool applies(const EvalArgs &a, int32_t i, int32_t o, int32_t r) {
    return static_cast<uint32_t>(i) < static_cast<uint32_t>(a.N) && o >= a.o_min && r <= a.T && r > o;
}

// kTail == false: the common kernel.  It only takes plans whose intervals all fit the registers
// (at most R per thread) and has no memory loads in its tile loop besides the dMF0 prefetch, so
// the compiler can wait for that prefetch with an exact counter value instead of draining every
// outstanding store.  kTail == true: the kernel for the remaining (longer) plans, which re-reads
// the intervals beyond the registers from memory for every tile.  Both are launched for every
// batch; a workgroup whose plan belongs to the other kernel exits at once.
// kOut: 0 = no footprint rows are written (peaks only), 1 = rows written with 8-byte stores
// (odd T or unaligned buffer), 2 = with 16-byte stores, 3 = with nontemporal 16-byte stores (long rows,
// see launch_eval).  A compile-time property so that every path through the tile loop issues the
// same memory operations: the compiler's waits for the loop's loads count the stores issued after
// them only when no branch surrounds those stores.
// kBinned: the batch went through bin_kernel first; nothing is kept in registers (R is 1 and unused),
// every tile reads its own records.  Every plan of the batch is taken.
// kBinFast (with kBinned): no tile of the segment holds more than kBinFastRecs * kThr records, so a tile's
// records are two unconditional loads per thread, requested one tile ahead, and the tile offsets come
// through the scalar unit: the tile loop then issues a fixed set of memory instructions like the common
// kernel's, instead of waiting for two dependent loads (and with them for every store) in every tile.
constexpr int kBinFastRecs = 2;
constexpr int kBinAhead = 4;   // tiles between the request for a tile's records and their use
// result (may be null): an LDS word triple that receives the segment's (max, earliest argmax, min) as well; it
// is complete after the next workgroup barrier.
template <int kThr, int R, bool kTail, bool kNarrow, int kOut, bool kBinned = false, bool kBinFast = false>
__device__ __forceinline__ void eval_body(const EvalArgs &a, const int32_t plan, const int32_t seg, EvalLds<kThr> &L,
                                          Best *result = nullptr) {
    static_assert(!kBinFast || kBinned, "kBinFast is a form of the binned kernel");
    constexpr bool kStore = kOut != 0, kVec16 = kOut >= 2;
    constexpr int kWaves = Geom<kThr>::kWaves, kTile = Geom<kThr>::kTile, kTileCells = Geom<kThr>::kTileCells;
    int64_t *const delta = L.delta, *const stage_all = L.stage_all, *const wave_tot = L.wave_tot, *const carry_part = L.carry_part;
    int64_t *const red_mx = L.red_mx, *const red_mn = L.red_mn;
    int32_t *const red_arg = L.red_arg;
    typedef SizeReg<kNarrow> SR;

    // (a copy of the thread index that the compiler cannot trace back: when a kernel calls this body in a loop,
    // the per-lane numbers derived from it are then computed afresh per call instead of being kept in registers -
    // and spilled - across whatever else the loop does)
    int tid_now = threadIdx.x;
    asm volatile("" : "+v"(tid_now));
    const int tid = tid_now, lane = tid & 63, wave = tid >> 6;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);   // the same number, known to be wave-uniform
    // The offsets are read through the constant address space (the batch is not written during the launch), so
    // that they come through the scalar unit: a vector load would queue behind whatever stores the workgroup
    // that had this CU before has left in the CU's memory pipeline, and the interval loads depend on it.
    typedef const int64_t __attribute__((address_space(4))) *const_i64_ptr;
    const const_i64_ptr plan_offsets = (const_i64_ptr)(a.plan_offsets);
    int64_t k0 = plan_offsets[plan], k1 = plan_offsets[plan + 1];
    if (k0 < 0) k0 = 0;
    if (k1 > a.n_intervals) k1 = a.n_intervals;
    if (k1 < k0) k1 = k0;
    if constexpr (!kBinned) {
        if ((k1 - k0 > a.tail_threshold) != kTail) {   // block-uniform: the other kernel's plan
            if (!kTail && tid == 0) atomicMax(a.tail_flag, a.epoch);   // tell the tail kernel it has work
            return;
        }
    }

    const int64_t seg_len = static_cast<int64_t>(a.tiles_per_seg) * kTile;
    const int64_t seg_lo64 = seg * seg_len;
    if (seg_lo64 >= a.T) return;   // cannot happen with the host's choice of S; keeps indexing safe
    const int32_t seg_lo = static_cast<int32_t>(seg_lo64);
    const int32_t seg_hi = static_cast<int32_t>(seg_lo64 + seg_len < a.T ? seg_lo64 + seg_len : a.T);
    const int my = tid * kVpt;                  // this lane's first step of the tile
    const int my_cell = my + 2 * (tid >> 2);    // ... and where it lives in the skewed tile
    int64_t *stage = stage_all + wave * kStageStride;

    // ---- first tile's cells: differences of the unscheduled timeline (dMF0 is padded to whole tiles)
    // dMF0 is read and put into the cells one 16-byte granule per lane, lanes side by side (whole lines per
    // load; 16 bytes at a 64-byte stride, the layout the scan reads, would touch four times as many): granule
    // j * 64 + lane of the wavefront's 256, conflict-free in the skewed tile like the lane's own 4 granules.
    // The wavefront's cells are only ever touched by the wavefront itself, and its LDS operations run in order.
    const int fill_at = wave * (64 * kVpt) + 2 * lane;                  // + 128 * j: first step of granule j
    const int fill_cell = fill_at + 2 * (fill_at >> 5);                // + 136 * j (128 steps and their skew)
    ll2 fill[kVpt / 2];
#pragma unroll
    for (int j = 0; j < kVpt / 2; ++j) fill[j] = *reinterpret_cast<const ll2 *>(a.dMF0 + seg_lo + fill_at + 128 * j);

    // ---- the plan's first R*threads intervals live in registers for the whole segment, R per
    // thread: (first step without the bytes, first step with them again, size).  An interval that cannot be applied, or a slot past the end of the list, gets
    // endpoints no tile contains.  [lo_t, hi_t] spans this thread's endpoints.
    // e0/e1 hold the endpoints as byte offsets into the segment's skewed cells (see kNoCell)
    uint32_t e0[R], e1[R];
    int64_t before = 0;   // (segments after the first) this thread's part of the plan's deltas before the segment
    typename SR::type sz[R];
    int32_t lo_t = INT32_MAX, hi_t = -1;
    if (!kBinned && k1 > k0) {   // block-uniform
        // all loads are unconditional (indices clamped into the plan's list, tensor index
        // clamped to 0) and issued back to back, then waited for once
        const int32_t *pt = a.iv_tensor + k0, *po = a.iv_out + k0, *pr = a.iv_in + k0;
        const uint32_t len = k1 - k0 < R * kThr ? static_cast<uint32_t>(k1 - k0) : R * kThr;
        // a wavefront holds 64 * R consecutive intervals (close in time when the caller lists them by
        // tensor, so that the wavefront can skip tiles), lanes side by side: every load is whole lines
        const uint32_t slot0 = static_cast<uint32_t>(wave) * (64 * R) + lane;
        int32_t ti[R], vo[R], vr[R];
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const uint32_t k = slot0 + j * 64;
            const uint32_t kc = k < len ? k : len - 1;
            ti[j] = pt[kc];
            vo[j] = po[kc];
            vr[j] = pr[kc];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const bool ok = slot0 + j * 64 < len && applies(a, ti[j], vo[j], vr[j]);
            ti[j] = ok ? ti[j] : -1;
        }
#pragma unroll
        for (int j = 0; j < R; ++j) sz[j] = SR::load(a, ti[j] < 0 ? 0 : ti[j]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < R; ++j) {
            if (ti[j] < 0) {
                sz[j] = 0;
                e0[j] = kNoCell;
                e1[j] = kNoCell;
            } else {
                lo_t = vo[j] + 1 < lo_t ? vo[j] + 1 : lo_t;
                hi_t = vr[j] > hi_t ? vr[j] : hi_t;
                e0[j] = cell_bytes(vo[j] + 1, seg_lo, seg_hi);
                e1[j] = cell_bytes(vr[j], seg_lo, seg_hi);
                if (seg_lo > 0) {   // (block-uniform)
                    const int64_t s = SR::bytes(a, sz[j]);
                    before += (vr[j] < seg_lo ? s : 0) - (vo[j] + 1 < seg_lo ? s : 0);
                }
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            e0[j] = kNoCell;
            e1[j] = kNoCell;
            sz[j] = 0;
        }
    }
    const int64_t k_over = k0 + static_cast<int64_t>(R) * kThr;   // the rest is re-read per tile

#pragma unroll
    for (int j = 0; j < kVpt / 2; ++j) *reinterpret_cast<ll2 *>(&delta[fill_cell + 136 * j]) = fill[j];

    // ---- footprint just before the segment: MF0 there plus the plan's deltas before it
    int64_t carry = 0;   // same value in every thread
    if (seg_lo > 0) {
        int64_t c = before;
        if constexpr (kTail) {
            for (int64_t k = k_over + tid; k < k1; k += kThr) {
                const int32_t i = a.iv_tensor[k], o = a.iv_out[k], r = a.iv_in[k];
                if (!applies(a, i, o, r)) continue;
                const int64_t s = a.size[i];
                c += (r < seg_lo ? s : 0) - (o + 1 < seg_lo ? s : 0);
            }
        }
        if constexpr (kBinned) {   // the tiles before the segment, already summed by bin_kernel
            const int64_t *ts = a.tile_sum + static_cast<int64_t>(plan) * a.n_tiles;
            for (int32_t tl = tid; tl < seg_lo / kTile; tl += kThr) c += ts[tl];
        }
        c = last_lane(wave_scan_add(c));
        if (lane == 0) carry_part[wave] = c;
        __syncthreads();
        carry = a.MF0[seg_lo - 1];
#pragma unroll
        for (int v = 0; v < kWaves; ++v) carry += carry_part[v];
    }

    Best best{INT64_MIN, INT64_MAX, INT32_MAX};
    int64_t *row = kStore ? a.resident + static_cast<int64_t>(plan) * a.T : nullptr;

    // kBinFast: the records of the tile at hand (two per thread) and where they start and end in the plan's
    // records; loads are clamped into the plan's records (into the batch's when the plan has none)
    typedef const int32_t __attribute__((address_space(4))) *const_i32_ptr;
    const const_i32_ptr tile_off =
        kBinFast ? (const_i32_ptr)(a.tile_off + static_cast<int64_t>(plan) * (a.n_tiles + 1)) : nullptr;
    const uint32_t n_rec = static_cast<uint32_t>(2 * (k1 - k0));
    const int2 *plan_recs = (kBinFast && n_rec) ? a.recs + 2 * k0 : a.recs;
    // (a record travels as ONE 64-bit value, cell and sign in the lower half, size units in the upper: as a pair of
    // 32-bit values the two halves become loop-carried values of their own, the register allocator gives one of
    // them a register that is not the load's, and the copy it inserts right after the request waits for the
    // records - and with them for every store before them - at the end of every tile)
    auto rec_at = [&](uint32_t k) {
        const uint64_t *const at = reinterpret_cast<const uint64_t *>(plan_recs) + (k < n_rec ? k : (n_rec ? n_rec - 1 : 0));
        // (read once, past the L2's allocation: rows of 10^6 steps 2.60 -> 2.50 ms, peaks only 1.28 -> 1.26; neutral
        // on short rows)
        return __builtin_nontemporal_load(at);
    };
    // kBinAhead register sets, taken in turn by the tiles of the segment.  A set is used in its tile's scatter and
    // requested again, for the tile kBinAhead tiles on, at the END of that tile: a request then has that many
    // tiles' time to come back from HBM (behind the CU's queue of row stores two tiles were not enough: the wait
    // for them still took a third of a tile), and the wavefronts reach that point spread out in time (they
    // leave the tile's last barrier together but drain their stores one after the other), so their requests do
    // not arrive in one burst on the CU's queue of outstanding misses, behind which the stores of all wavefronts
    // would wait.
    uint64_t rec_set[kBinAhead][kBinFastRecs];
    auto off_at = [&](int32_t tile_index) { return tile_off[tile_index < a.n_tiles ? tile_index : a.n_tiles]; };
    auto load_recs = [&](int32_t lo, int32_t hi, uint64_t (&dst)[kBinFastRecs]) {   // the records [lo, hi) of one tile
#pragma unroll
        for (int j = 0; j < kBinFastRecs; ++j) {
            // (a slot past the tile's last record reads what slot j - 1 reads: a line that is on its way already)
            const int32_t k = lo + j * kThr + tid;
            dst[j] = rec_at(static_cast<uint32_t>(j > 0 && k >= hi ? k - kThr : k));
        }
    };
    // (uniform) where the records of this tile and of the kBinAhead tiles after it start; a tile reads one more
    // offset at its top, through the scalar unit, and needs it at its end
    int32_t offs[kBinAhead + 1] = {}, off_new = 0;
    if constexpr (kBinFast) {
        const int32_t t0 = seg_lo / kTile;
#pragma unroll
        for (int d = 0; d <= kBinAhead; ++d) offs[d] = off_at(t0 + d);
#pragma unroll
        for (int d = 0; d < kBinAhead; ++d) load_recs(offs[d], offs[d + 1], rec_set[d]);
    }
    __syncthreads();   // the first tile's cells are in place

    // One quarter (granule row j of 4) of a tile's stores from the wave's staging area: 16
    // contiguous bytes per lane, 1 KB per wavefront.  A whole tile with 16-byte aligned rows
    // (block-uniform) needs no bounds checks.
    auto store_part = [&](int32_t t_lo, int32_t t_hi, int j) {
        const int32_t wave_t0 = t_lo + wave_u * (64 * kVpt);
        const ll2 x = (reinterpret_cast<const ll2 *>(stage) + lane + (lane >> 4))[68 * j];
        if (kVec16 && t_hi - t_lo == kTile) {
            ll2 *const at = reinterpret_cast<ll2 *>(row + wave_t0) + lane + 64 * j;
            if constexpr (kOut == 3) __builtin_nontemporal_store(x, at);
            else *at = x;
        } else {
            const int32_t t = wave_t0 + 2 * (j * 64 + lane);
            if (t + 2 <= t_hi) {
                row[t] = x[0];
                row[t + 1] = x[1];
            } else if (t < t_hi) {
                row[t] = x[0];
            }
        }
    };

    // One tile.  The results of a tile are parked in the staging area and stored during the NEXT
    // iteration (software pipelining), one quarter after each phase.  Two reasons: (1) the loads
    // of the next tile's dMF0 come first in the iteration, so the scan can wait for them with an
    // exact counter value while younger stores stay in flight; (2) all wavefronts of a CU share
    // one in-order memory pipeline that drains at the CU's share of the HBM write rate: a burst
    // of every wavefront's stores at one point of the iteration backs it up and the wavefronts
    // behind arrive late at the next barrier.  The first tile has no previous one and is a
    // separate instantiation so that the same operations are issued on every path.
#ifdef TENSILE_EVAL_PROF
    unsigned long long prof_t = wall_clock64();
    unsigned long long prof_acc[8] = {};
#endif
    auto do_tile = [&](int32_t tile_lo, auto first_tag, auto set_tag) {
        EVAL_MARK(7);
        constexpr bool kFirst = decltype(first_tag)::value;
        constexpr int kSet = decltype(set_tag)::value;   // (kBinFast) the register set that holds this tile's records
        const int32_t tile_hi = tile_lo + kTile < seg_hi ? tile_lo + kTile : seg_hi;
        const uint32_t tile_n = static_cast<uint32_t>(tile_hi - tile_lo);
        // delta holds dMF0 of this tile: written before the loop, or by the scan of the previous
        // tile ahead of its barrier.  dMF0 has one whole tile of padding past the end, so the load
        // of the "next" tile is unconditional (what it brings is never scanned in that case).
#pragma unroll
        for (int j = 0; j < kVpt / 2; ++j)
            fill[j] = *reinterpret_cast<const ll2 *>(a.dMF0 + tile_lo + kTile + fill_at + 128 * j);
        const int32_t rec_lo = offs[0], rec_hi = offs[1];   // this tile's records within the plan's
        if constexpr (kBinFast) off_new = off_at(tile_lo / kTile + kBinAhead + 1);
        constexpr bool kPrev = !kFirst && kStore;
        if constexpr (kPrev) {
            __builtin_amdgcn_wave_barrier();
            store_part(tile_lo - kTile, tile_lo, 0);
        }

        EVAL_MARK(0);
        // ---- scatter: endpoints of this plan that fall into [tile_lo, tile_hi); a wavefront none
        // of whose lanes holds an endpoint in the tile's range skips its registers
        const bool mine = hi_t >= tile_lo && lo_t < tile_hi;
        if (__builtin_amdgcn_ballot_w64(mine) != 0) {
            // (three instructions per endpoint: subtract the tile's offset, a scalar; minimum with the trash cell;
            // the atomic.  With cell numbers, a comparison against the tile's length and a shift: five, and the
            // scatter was 40 % of the tile loop's vector instructions - 8 % of a peaks-only pass, nothing where the
            // row stores set the pace)
            const uint32_t tile_bytes = __builtin_amdgcn_readfirstlane(skew(static_cast<uint32_t>(tile_lo - seg_lo)) * 8u);
            const uint32_t trash = (kTileCells + lane) * 8u;
            char *const cells = reinterpret_cast<char *>(delta);
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const uint32_t u0 = e0[j] - tile_bytes, u1 = e1[j] - tile_bytes;
                // keep the compact register form across tiles: without this the widened (and a
                // negated) size is hoisted out of the tile loop and held in extra registers
                typename SR::type s = sz[j];
                opaque(s);
                const int64_t bytes = SR::bytes(a, s);
                lds_sub(reinterpret_cast<int64_t *>(cells + (u0 < trash ? u0 : trash)), bytes);
                lds_add(reinterpret_cast<int64_t *>(cells + (u1 < trash ? u1 : trash)), bytes);
            }
        }
        if constexpr (kTail) {
            // the intervals beyond the registers, kTailU per thread and round: their loads are issued together (at
            // clamped indices), so that a round costs one memory latency, not kTailU; the size is fetched only for
            // the few whose endpoints fall into this tile
            for (int64_t kb = k_over + tid; kb < k1; kb += static_cast<int64_t>(kTailU) * kThr) {
                int32_t ti[kTailU], to[kTailU], tr[kTailU];
#pragma unroll
                for (int u = 0; u < kTailU; ++u) {
                    const int64_t k = kb + static_cast<int64_t>(u) * kThr;
                    const int64_t kc = k < k1 ? k : k1 - 1;
                    ti[u] = a.iv_tensor[kc];
                    to[u] = a.iv_out[kc];
                    tr[u] = a.iv_in[kc];
                    if (k >= k1) ti[u] = -1;
                }
#pragma unroll
                for (int u = 0; u < kTailU; ++u) {
                    if (!applies(a, ti[u], to[u], tr[u])) continue;
                    const uint32_t u0 = static_cast<uint32_t>(to[u] + 1 - tile_lo), u1 = static_cast<uint32_t>(tr[u] - tile_lo);
                    if ((u0 < tile_n) | (u1 < tile_n)) {
                        const int64_t s = a.size[ti[u]];
                        if (u0 < tile_n) lds_add(&delta[skew(u0)], -s);
                        if (u1 < tile_n) lds_add(&delta[skew(u1)], s);
                    }
                }
            }
        }
        if constexpr (kBinFast) {
            const uint32_t trash = kTileCells + lane;
#pragma unroll
            for (int j = 0; j < kBinFastRecs; ++j) {
                const uint64_t rec = rec_set[kSet][j];
                const int32_t rec_x = static_cast<int32_t>(static_cast<uint32_t>(rec));
                const bool valid = rec_lo + j * kThr + tid < rec_hi;
                const int64_t bytes = static_cast<int64_t>((rec >> 32) << a.size_shift);
                lds_add(&delta[valid ? static_cast<uint32_t>(rec_x) & 0x7fffffffu : trash], !valid ? 0 : rec_x < 0 ? -bytes : bytes);
            }
        } else if constexpr (kBinned) {
            const int32_t *off = a.tile_off + static_cast<int64_t>(plan) * (a.n_tiles + 1) + tile_lo / kTile;
            const int2 *recs = a.recs + 2 * k0;
            for (int32_t k = off[0] + tid; k < off[1]; k += kThr) {
                const int2 rec = recs[k];
                const int64_t bytes = static_cast<int64_t>(static_cast<uint64_t>(static_cast<uint32_t>(rec.y)) << a.size_shift);
                if (rec.x < 0) lds_sub(&delta[rec.x & 0x7fffffff], bytes);
                else lds_add(&delta[rec.x], bytes);
            }
        }
        if constexpr (kPrev) store_part(tile_lo - kTile, tile_lo, 1);
        EVAL_MARK(1);
        __syncthreads();
        EVAL_MARK(2);

        // ---- local scan of this lane's 8 cells; the cells receive the next tile's dMF0.  In the
        // ragged last tile of a row a wavefront whose 512 steps all lie past the end has nothing
        // to scan (wave-uniform): it only reports a zero total.
        const bool wave_live = tile_lo + wave_u * (64 * kVpt) < tile_hi;
        int64_t v[kVpt];
        int64_t incl = 0;
        if (wave_live) {
            const ll2 *cell = reinterpret_cast<const ll2 *>(&delta[my_cell]);
#pragma unroll
            for (int j = 0; j < kVpt / 2; ++j) {
                const ll2 x = cell[j];
                v[2 * j] = x[0];
                v[2 * j + 1] = x[1];
            }
            // (all of the wavefront's reads are issued before the first of its writes)
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < kVpt / 2; ++j) *reinterpret_cast<ll2 *>(&delta[fill_cell + 136 * j]) = fill[j];
#pragma unroll
            for (int j = 1; j < kVpt; ++j) v[j] += v[j - 1];
            incl = wave_scan_add(v[kVpt - 1]);
        }
        if (lane == 63) wave_tot[wave] = incl;
        if constexpr (kPrev) store_part(tile_lo - kTile, tile_lo, 2);
        EVAL_MARK(3);
        __syncthreads();
        EVAL_MARK(4);
        if (!wave_live) {   // (the ragged tile is the last one of its row: no later tile needs carry)
            if constexpr (kPrev) store_part(tile_lo - kTile, tile_lo, 3);
            return;
        }
        // (the last quarter goes out here rather than at the end of the iteration, where the next
        // iteration's first quarter would follow it at once: measured 0.6 % faster)
        if constexpr (kPrev) store_part(tile_lo - kTile, tile_lo, 3);
        // prefix over the wave totals: the first lanes scan them, then every lane picks the
        // sum of the waves before its own and the tile total by lane index
        int64_t tot = wave_tot[lane & (kWaves - 1)];
        tot += dpp_or_zero<0x111, 0xf>(tot);
        tot += dpp_or_zero<0x112, 0xf>(tot);
        tot += dpp_or_zero<0x114, 0xf>(tot);
        if constexpr (kWaves > 8) tot += dpp_or_zero<0x118, 0xf>(tot);
        const int64_t before = wave_u > 0 ? lane_value(tot, wave_u - 1) : 0;
        const int64_t base = carry + before + incl - v[kVpt - 1];
        carry += lane_value(tot, kWaves - 1);
#pragma unroll
        for (int j = 0; j < kVpt; ++j) v[j] += base;

        // ---- reduce
        const int32_t t0 = tile_lo + my;
        if (t0 + kVpt <= tile_hi) {
            // The lane's 8 values almost always share their upper 32 bits; then max and min are
            // those of the (unsigned) lower halves, single instructions without a condition code.
            int64_t cm, cn;
            {
                const int32_t h0 = static_cast<int32_t>(v[0] >> 32);
                uint32_t diff = 0, lmx = static_cast<uint32_t>(v[0]), lmn = lmx;
#pragma unroll
                for (int j = 1; j < kVpt; ++j) {
                    diff |= static_cast<uint32_t>(static_cast<int32_t>(v[j] >> 32) ^ h0);
                    const uint32_t l = static_cast<uint32_t>(v[j]);
                    lmx = l > lmx ? l : lmx;
                    lmn = l < lmn ? l : lmn;
                }
                if (__builtin_amdgcn_ballot_w64(diff != 0) == 0) {   // wave-uniform
                    cm = (static_cast<int64_t>(h0) << 32) | lmx;
                    cn = (static_cast<int64_t>(h0) << 32) | lmn;
                } else {
                    cm = v[0];
                    cn = v[0];
#pragma unroll
                    for (int j = 1; j < kVpt; ++j) {
                        cm = v[j] > cm ? v[j] : cm;
                        cn = v[j] < cn ? v[j] : cn;
                    }
                }
            }
            if (cm > best.mx) {
                best.mx = cm;
#pragma unroll
                for (int j = kVpt - 1; j >= 0; --j)
                    if (v[j] == cm) best.arg = t0 + j;
            }
            best.mn = cn < best.mn ? cn : best.mn;
        } else {
#pragma unroll
            for (int j = 0; j < kVpt; ++j) {
                if (t0 + j < tile_hi) {
                    if (v[j] > best.mx) {
                        best.mx = v[j];
                        best.arg = t0 + j;
                    }
                    if (v[j] < best.mn) best.mn = v[j];
                }
            }
        }

        // ---- park the results in the wave's staging area (lane-contiguous, skewed); they are
        // stored during the next iteration, or after the loop
        if constexpr (kPrev) __builtin_amdgcn_wave_barrier();
        if constexpr (kStore) {
            ll2 *mine_out = reinterpret_cast<ll2 *>(stage + lane * kVpt + 2 * (lane >> 2));
#pragma unroll
            for (int j = 0; j < kVpt / 2; ++j) mine_out[j] = ll2{v[2 * j], v[2 * j + 1]};
        }
        EVAL_MARK(5);
        if constexpr (kBinFast) {
            load_recs(offs[kBinAhead], off_new, rec_set[kSet]);
            // With rows the wavefront now waits for everything it has in flight, these records included (s_waitcnt
            // vmcnt(0): bits 3:0 and 15:14 of the operand; the other counters at their maxima).  Measured on rows of
            // 10^6 steps, 60,000 intervals per plan: 2.61 ms; without the wait 3.14 ms, with a wait that leaves just
            // the records in flight 3.15, with the wait before the request 3.17, with the request after the scatter
            // and the wait here 3.02.  A request that is still on its way to HBM while the CU's wavefronts issue row
            // stores holds those stores up; made last in the tile and waited for, it has the queue to itself (the
            // wavefronts get here one after the other).  Without rows nothing is held up, and the requests run
            // kBinAhead tiles ahead (1.43 -> 1.28 ms).
            if constexpr (kStore) __builtin_amdgcn_s_waitcnt(0x0f70);
#pragma unroll
            for (int d = 0; d < kBinAhead; ++d) offs[d] = offs[d + 1];
            offs[kBinAhead] = off_new;
        }
        EVAL_MARK(6);
    };

    typedef std::integral_constant<int, 0> Set0;
    typedef std::integral_constant<int, 1> Set1;
    typedef std::integral_constant<int, 2> Set2;
    typedef std::integral_constant<int, 3> Set3;
    static_assert(kBinAhead == 4, "the tile loop below names the register sets");
    do_tile(seg_lo, std::true_type{}, Set0{});
    int32_t last_lo = seg_lo;
    if constexpr (kBinFast) {
        // The second tile stands outside the loop as well: the loop is then entered from a tile that, like the
        // tiles inside it, issues its four quarters of stores after requesting the next tile's records.  The
        // compiler's wait for those records counts the operations issued after them on the SHORTEST path into the
        // loop; entered from the first tile (which has no stores), every iteration waited for all stores of the
        // tile before it to complete.
        if (seg_lo + kTile < seg_hi) {
            do_tile(seg_lo + kTile, std::false_type{}, Set1{});
            last_lo = seg_lo + kTile;
            // Whole groups of kBinAhead tiles in the loop, the rest after it: a way out of the middle of the loop's
            // body would give the compiler a path from the end of one tile straight back to the top of the loop
            // (never taken, but it counts the operations issued after a request on the shortest path), and the wait
            // for a tile's records would again include the stores of the tile before.
            const std::false_type later{};
            int32_t tile_lo = seg_lo + 2 * kTile;
            for (; tile_lo + 3 * kTile < seg_hi; tile_lo += 4 * kTile) {
                do_tile(tile_lo, later, Set2{});
                do_tile(tile_lo + kTile, later, Set3{});
                do_tile(tile_lo + 2 * kTile, later, Set0{});
                do_tile(tile_lo + 3 * kTile, later, Set1{});
            }
            last_lo = tile_lo - kTile;
            if (tile_lo < seg_hi) {
                do_tile(tile_lo, later, Set2{});
                last_lo = tile_lo;
                if (tile_lo + kTile < seg_hi) {
                    do_tile(tile_lo + kTile, later, Set3{});
                    last_lo = tile_lo + kTile;
                    if (tile_lo + 2 * kTile < seg_hi) {
                        do_tile(tile_lo + 2 * kTile, later, Set0{});
                        last_lo = tile_lo + 2 * kTile;
                    }
                }
            }
        }
    } else {
        for (int32_t tile_lo = seg_lo + kTile; tile_lo < seg_hi; tile_lo += kTile) {
            do_tile(tile_lo, std::false_type{}, Set0{});
            last_lo = tile_lo;
        }
    }
    if constexpr (kStore) {
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < kVpt / 2; ++j) store_part(last_lo, seg_hi, j);
    }

#ifdef TENSILE_EVAL_PROF
    if (lane == 0) {
#pragma unroll
        for (int k = 0; k < 8; ++k) atomicAdd(&g_eval_prof[wave * 8 + k], prof_acc[k]);
    }
#endif
    // ---- (max, earliest argmax, min) of the segment
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const int64_t omx = __shfl_xor(best.mx, d, 64), omn = __shfl_xor(best.mn, d, 64);
        const int32_t oarg = __shfl_xor(best.arg, d, 64);
        best_merge(best, omx, oarg, omn);
    }
    if (lane == 0) {
        red_mx[wave] = best.mx;
        red_mn[wave] = best.mn;
        red_arg[wave] = best.arg;
    }
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int u = 1; u < kWaves; ++u) best_merge(best, red_mx[u], red_arg[u], red_mn[u]);
        const int64_t slot = static_cast<int64_t>(plan) * a.S + seg;
        a.out_max[slot] = best.mx;
        a.out_arg[slot] = best.arg;
        if (a.out_min) a.out_min[slot] = best.mn;
        if (result) *result = best;
    }
}

}  // namespace

}  // namespace tensile
