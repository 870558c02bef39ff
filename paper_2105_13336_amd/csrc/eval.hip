// Memory peak analysis of a batch of plans (Eq. 1, Eq. 2 and Alg. 1 of the paper)
// as one fused kernel: difference-array scatter of the interval endpoints into an
// LDS tile, prefix scan over the steps, store the footprint row, and reduce
// (max, earliest argmax, min) on the way.
//
// Work decomposition.  A workgroup owns one (plan, segment): `tiles_per_seg`
// consecutive tiles of 8 steps per thread.  Three geometries are compiled: 1024 threads
// with 8192-step tiles (one workgroup per CU: long rows), 512 threads with 4096-step
// tiles (two workgroups per CU, so that one can load while the other scans: short rows, and
// batches of more plans than CUs when they write no rows) and 256 threads with 2048-step tiles
// (four per CU: large batches of short rows and short plans; see launch_eval).  The running sum that
// enters a segment is MF0 just before it plus the plan's deltas before it, which
// the workgroup takes straight from the plan's intervals (an interval
// contributes -size if its out+1 lies before the segment and +size if its in
// step does), so segments of one plan need no communication and no look-back.
//
// The kernel is bound by instruction issue as much as by HBM (the chip issues
// about 39 lane-instructions per 8-byte element at full HBM speed and 64-bit
// integer adds take two), so the per-element work is kept small:
//  * The LDS tile is initialised with the DIFFERENCES of the unscheduled
//    timeline, dMF0[t] = MF0[t] - MF0[t-1], not with zeros: the scan then yields
//    the footprint itself and no separate "+ MF0" pass is needed.  The next
//    tile's dMF0 is loaded while the current tile is processed and written into
//    the cells as the scan reads them.
//  * The memory counter of a wavefront retires loads and stores in order, so a
//    load issued after a tile's stores can only be waited for together with
//    them.  The stores of a tile are therefore issued one iteration late, right
//    after the loads of that iteration, from the staging area.
//  * The plan's intervals are read once into registers (endpoints and size; R
//    per thread, chosen on the host from the average plan length; a longer plan
//    re-reads its tail from memory per tile).  Threads take CONSECUTIVE
//    intervals, so when a plan lists its intervals roughly in time order (plans
//    are usually built tensor by tensor) a wavefront's endpoints cluster in time
//    and the wavefront skips the scatter of tiles its endpoints cannot touch.
//    The result does not depend on the order.
//  * Each lane owns 8 consecutive steps of the tile: 7 local adds, one DPP wave
//    scan per 8 steps, one exchange of wave totals through LDS (two barriers per
//    tile), one add of the offset.
//  * Stores want 16 contiguous bytes per lane per instruction (a wavefront then
//    writes 1 KB of whole lines; 64 bytes per lane at a 64-byte stride reaches
//    only about 60 % of the streaming-store rate), so each wavefront transposes
//    its 512 results through a private LDS staging area.  Both the tile and the
//    staging area skew every group of four lanes by one 16-byte granule, which
//    makes the lane-contiguous and the striped access patterns conflict-free.
//  * max/min are reduced over the lane's 8 values first; the argmax is located
//    only when the lane's maximum improves.
//
// Workgroup ids are decoded so that all segments of a plan run on the same XCD
// (ids are dealt round-robin to the 8 XCDs, each with its own L2): the plan's
// interval list is then fetched from HBM once and re-read from that L2.
#include "eval_body.h"

namespace tensile {

namespace {

// Four waves per SIMD (one workgroup of 1024 threads or two of 512 per CU) need at most 128 VGPRs;
// up to 12 intervals per thread fit without spilling.  The tail kernel is left to the register allocator.
template <int kThr, int R, bool kNarrow, int kOut>
__global__ __launch_bounds__(kThr) __attribute__((amdgpu_waves_per_eu(4, 4))) void eval_kernel(const EvalArgs a) {
    __shared__ EvalLds<kThr> lds;
    int32_t plan, seg;
    if (!decode_block(a, blockIdx.x, plan, seg)) return;
    eval_body<kThr, R, false, kNarrow, kOut>(a, plan, seg, lds);
}

// ---- many plans per workgroup ------------------------------------------------------------
// A persistent grid: one workgroup per resident slot walks the plans slot, slot + grid, ... as ONE
// stream of tiles.  A workgroup that starts pays three dependent load latencies (offsets, intervals,
// sizes) before its first tile; here
//  * the next plan's intervals are requested during the current plan's first tile and their sizes during
//    its last, into registers of their own (a row of one tile: after its scatter and after its scan);
//  * the last tile's scan refills the cells with the next plan's first tile;
//  * a tile's results are stored during the next tile, whichever plan that belongs to;
//  * the wavefronts' (max, argmax, min) of a plan are combined after the next tile's first barrier.
// Measured on rows of 50,000 steps with 5,400 intervals per plan, 16,384 plans, 1024 threads: 11 % faster than
// one workgroup per plan when no rows are written (1.19 -> 1.05 ms; two workgroups of 512 threads per CU, one per
// plan, take 0.86 there and are what the host picks) and 6 % when they are (1.66 -> 1.55 ms), where the lists'
// way from HBM is the part a starting workgroup cannot hide; with the lists requested only one tile ahead it was no
// faster than one workgroup per plan.
// Plans with more intervals than the registers hold are left to the tail kernel as before.
template <int kThr, int R, bool kNarrow, int kOut>
__global__ __launch_bounds__(kThr) __attribute__((amdgpu_waves_per_eu(4, 4))) void eval_stream_kernel(const EvalArgs a) {
    constexpr bool kStore = kOut != 0, kVec16 = kOut == 2;
    constexpr int kWaves = Geom<kThr>::kWaves, kTile = Geom<kThr>::kTile, kTileCells = Geom<kThr>::kTileCells;
    __shared__ __attribute__((aligned(16))) int64_t delta[kTileCells + 64];   // the tile, then 64 "trash" cells
    __shared__ __attribute__((aligned(16))) int64_t stage_all[kWaves * kStageStride];
    __shared__ int64_t wave_tot[kWaves];
    __shared__ int64_t red_mx[kWaves], red_mn[kWaves];
    __shared__ int32_t red_arg[kWaves];
    __shared__ int64_t ahead_off[2][2];   // where the list of the plan after the next starts and ends (see the plan loop)
    typedef SizeReg<kNarrow> SR;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t stride = gridDim.x;
    // The same per-lane numbers (and the wavefront's staging area), derived afresh from a copy of the thread id that the compiler cannot
    // trace back: every tile takes its own, so that none of them (nor the addresses built on them)
    // stays in a register from one end of the kernel to the other.  Spilled registers are the thing
    // to avoid here: their reloads are vector memory loads, waited for together with every store.
    struct Ids {
        int tid, lane, wave, wave_u, my, my_cell;
        int fill_at, fill_cell;   // the lane's granule of dMF0 (see eval_body): first step within the tile, cell; + 128 / 136 per j
        int64_t *stage;
    };
    auto fresh_ids = [&]() {
        int t = threadIdx.x;
        asm volatile("" : "+v"(t));
        Ids L;
        L.tid = t;
        L.lane = t & 63;
        L.wave = t >> 6;
        L.wave_u = __builtin_amdgcn_readfirstlane(L.wave);
        L.my = t * kVpt;
        L.my_cell = L.my + 2 * (t >> 2);
        L.fill_at = L.wave * (64 * kVpt) + 2 * L.lane;
        L.fill_cell = L.fill_at + 2 * (L.fill_at >> 5);
        L.stage = stage_all + L.wave * kStageStride;
        return L;
    };

    // The offsets are read through the constant address space: the batch is not written during the
    // launch, and only then may a uniform load inside a loop that also stores go through the scalar
    // unit (a vector load would have to be waited for together with every store before it).
    typedef const int64_t __attribute__((address_space(4))) *const_i64_ptr;
    const const_i64_ptr plan_offsets = (const_i64_ptr)(a.plan_offsets);
    auto uniform = [](int64_t x) {   // (the value is the same in every lane; this tells the compiler)
        const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(x));
        const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(static_cast<uint64_t>(x) >> 32));
        return static_cast<int64_t>((static_cast<uint64_t>(hi) << 32) | lo);
    };
    auto list_of = [&](int64_t p, int64_t &k0, int64_t &k1) {
        k0 = plan_offsets[p];
        k1 = plan_offsets[p + 1];
        if (k0 < 0) k0 = 0;
        if (k1 > a.n_intervals) k1 = a.n_intervals;
        if (k1 < k0) k1 = k0;
    };
    // the first plan at or after p, in steps of the grid, whose intervals fit the registers
    auto next_mine = [&](int64_t p) {
        bool left_one = false;
        for (p = uniform(p); p < a.B; p = uniform(p + stride)) {
            int64_t k0, k1;
            list_of(p, k0, k1);
            if (k1 - k0 <= a.tail_threshold) break;
            left_one = true;
        }
        if (left_one && tid == 0) atomicMax(a.tail_flag, a.epoch);   // tell the tail kernel it has work
        return p;
    };

    // A plan's intervals on their way into the registers: (tensor, out, in), then (size, out, in)
    // with in = -1 for an interval that is not applied or a slot past the end of the list.  All
    // loads are unconditional, at clamped addresses (an empty list reads the offsets array).
    int32_t nti[R], nvo[R], nvr[R];
    typename SR::type nsz[R];
    auto load_list = [&](const Ids &L, int64_t k0, int64_t k1) {
        const bool some = k1 > k0;
        const uint32_t len = some ? static_cast<uint32_t>(k1 - k0) : 1u;   // (at most R * kThr)
        const int32_t *none = reinterpret_cast<const int32_t *>(a.plan_offsets);
        const int32_t *pt = some ? a.iv_tensor + k0 : none, *po = some ? a.iv_out + k0 : none, *pr = some ? a.iv_in + k0 : none;
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const uint32_t k = static_cast<uint32_t>(L.wave) * (64 * R) + j * 64 + L.lane;   // (as in eval_body)
            const uint32_t kc = k < len ? k : len - 1;
            // (when rows are written the lists are read past the L2's allocation: they are used once, and the lines
            // they would take are the unscheduled timeline's, which every workgroup of the XCD reads - c3 1.575 ->
            // 1.547 ms; without row stores it is 1 % slower, and in the kernel with one workgroup per plan, which
            // waits for the lists at once, 3 % on 24,000-step rows and 40 % on 6,000-step ones)
            if constexpr (kStore) {
                nti[j] = __builtin_nontemporal_load(pt + kc);
                nvo[j] = __builtin_nontemporal_load(po + kc);
                nvr[j] = __builtin_nontemporal_load(pr + kc);
            } else {
                nti[j] = pt[kc];
                nvo[j] = po[kc];
                nvr[j] = pr[kc];
            }
        }
    };
    auto load_sizes = [&](const Ids &L, int64_t k0, int64_t k1) {
        const uint32_t len = static_cast<uint32_t>(k1 - k0);
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const bool ok = static_cast<uint32_t>(L.wave) * (64 * R) + j * 64 + L.lane < len && applies(a, nti[j], nvo[j], nvr[j]);
            nvr[j] = ok ? nvr[j] : -1;
            nti[j] = ok ? nti[j] : 0;
        }
#pragma unroll
        for (int j = 0; j < R; ++j) nsz[j] = SR::load(a, nti[j]);
    };
    // the current plan's intervals, as in eval_body
    uint32_t e0[R], e1[R];
    typename SR::type sz[R];
    int32_t lo_t = INT32_MAX, hi_t = -1;
    auto take_list = [&]() {
        lo_t = INT32_MAX;
        hi_t = -1;
#pragma unroll
        for (int j = 0; j < R; ++j) {
            if (nvr[j] < 0) {
                sz[j] = 0;
                e0[j] = kNoCell;
                e1[j] = kNoCell;
            } else {
                sz[j] = nsz[j];
                lo_t = nvo[j] + 1 < lo_t ? nvo[j] + 1 : lo_t;
                hi_t = nvr[j] > hi_t ? nvr[j] : hi_t;
                e0[j] = cell_bytes(nvo[j] + 1, 0, a.T);
                e1[j] = cell_bytes(nvr[j], 0, a.T);
            }
        }
    };

    int64_t plan = next_mine(blockIdx.x);
    if (plan >= a.B) return;   // (block-uniform)
    ll2 fill[kVpt / 2];
    {
        const Ids L0 = fresh_ids();
#pragma unroll
        for (int j = 0; j < kVpt / 2; ++j) fill[j] = *reinterpret_cast<const ll2 *>(a.dMF0 + L0.fill_at + 128 * j);
    }
    {
        int64_t k0, k1;
        list_of(plan, k0, k1);
        const Ids L = fresh_ids();
        load_list(L, k0, k1);
        __builtin_amdgcn_sched_barrier(0);
        load_sizes(L, k0, k1);
        __builtin_amdgcn_sched_barrier(0);
        take_list();
    }
    {
        const Ids L0 = fresh_ids();
#pragma unroll
        for (int j = 0; j < kVpt / 2; ++j) *reinterpret_cast<ll2 *>(&delta[L0.fill_cell + 136 * j]) = fill[j];
    }

    int64_t carry = 0;
    Best best{INT64_MIN, INT64_MAX, INT32_MAX};
    int64_t *row = nullptr;
    // the tile whose results wait in the staging areas (none yet: an empty range stores nothing)
    int64_t *prev_row = a.resident;
    int32_t prev_lo = 0, prev_hi = 0;
    int64_t done_plan = -1;      // the plan whose per-wavefront results wait in red_*
    int64_t nk0 = 0, nk1 = 0;    // the next plan's list
    int64_t ahead = a.B;         // the plan after the next (a.B: none), whose offsets the first wavefront fetches
    int ahead_slot = 0;          // ... into ahead_off[ahead_slot]
    __syncthreads();

    // Every path through a tile issues the same memory instructions, so that the waits for its loads
    // can name an exact count of younger operations.  A quarter of the previous tile's results:
    //  * kFull (the tile before is a whole tile of the same row): one 16-byte store per lane, or two
    //    8-byte ones when rows are not 16-byte aligned, no bounds;
    //  * otherwise (it is the last tile of the previous plan's row, ragged or not, or there is none):
    //    two 8-byte buffer stores over the valid part of that row; the hardware drops what lies
    //    beyond the range, so nothing is conditional here either.
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    auto store_part = [&](const Ids &L, int j, auto full_tag) {
        constexpr bool kFull = decltype(full_tag)::value;
        if constexpr (kStore) {
            const int32_t wave_t0 = prev_lo + L.wave_u * (64 * kVpt);
            const ll2 x = (reinterpret_cast<const ll2 *>(L.stage) + L.lane + (L.lane >> 4))[68 * j];
            if constexpr (kFull) {
                if constexpr (kVec16) {
                    (reinterpret_cast<ll2 *>(prev_row + wave_t0) + L.lane)[64 * j] = x;
                } else {
                    int64_t *dst = prev_row + wave_t0 + 2 * (j * 64 + L.lane);
                    dst[0] = x[0];
                    dst[1] = x[1];
                }
            } else {
                // (byte offsets fit 32 bits: the host sends rows of more than 2^28 steps elsewhere)
                const __amdgpu_buffer_rsrc_t rows =
                    __builtin_amdgcn_make_buffer_rsrc(prev_row, 0, static_cast<int32_t>(static_cast<uint32_t>(prev_hi) * 8u), 0x00020000);
                const uint32_t off = static_cast<uint32_t>(wave_t0 + 2 * (j * 64 + L.lane)) * 8u;
                u32x2 w0, w1;
                w0[0] = static_cast<uint32_t>(x[0]);
                w0[1] = static_cast<uint32_t>(static_cast<uint64_t>(x[0]) >> 32);
                w1[0] = static_cast<uint32_t>(x[1]);
                w1[1] = static_cast<uint32_t>(static_cast<uint64_t>(x[1]) >> 32);
                __builtin_amdgcn_raw_buffer_store_b64(w0, rows, static_cast<int32_t>(off), 0, 0);
                __builtin_amdgcn_raw_buffer_store_b64(w1, rows, static_cast<int32_t>(off + 8u), 0, 0);
            }
        }
    };
    // The finished plan's result: every wavefront combines the per-wavefront values (cheaper than a
    // branch), and every lane issues the three stores, through buffers of one element that only lane 0
    // of the last wavefront addresses in range (of no element when no plan is finished, or no minimum is wanted).
    auto write_result = [&](const Ids &L) {
        Best b{INT64_MIN, INT64_MAX, INT32_MAX};
        if (L.lane < kWaves) {
            b.mx = red_mx[L.lane];
            b.mn = red_mn[L.lane];
            b.arg = red_arg[L.lane];
        }
#pragma unroll
        for (int d = kWaves / 2; d >= 1; d >>= 1) {
            const int64_t omx = __shfl_xor(b.mx, d, 64), omn = __shfl_xor(b.mn, d, 64);
            const int32_t oarg = __shfl_xor(b.arg, d, 64);
            best_merge(b, omx, oarg, omn);
        }
        const bool some = done_plan >= 0;
        const int64_t slot = some ? done_plan : 0;
        const __amdgpu_buffer_rsrc_t r_mx = __builtin_amdgcn_make_buffer_rsrc(a.out_max + slot, 0, some ? 8 : 0, 0x00020000);
        const __amdgpu_buffer_rsrc_t r_arg = __builtin_amdgcn_make_buffer_rsrc(a.out_arg + slot, 0, some ? 4 : 0, 0x00020000);
        const __amdgpu_buffer_rsrc_t r_mn =
            __builtin_amdgcn_make_buffer_rsrc(a.out_min ? a.out_min + slot : a.out_max, 0, some && a.out_min ? 8 : 0, 0x00020000);
        const int32_t off = L.tid == kThr - 64 ? 0 : 64;   // (the last wavefront's L.lane 0; anything else is out of range)
        u32x2 w;
        w[0] = static_cast<uint32_t>(b.mx);
        w[1] = static_cast<uint32_t>(static_cast<uint64_t>(b.mx) >> 32);
        __builtin_amdgcn_raw_buffer_store_b64(w, r_mx, off, 0, 0);
        __builtin_amdgcn_raw_buffer_store_b32(static_cast<uint32_t>(b.arg), r_arg, off, 0, 0);
        w[0] = static_cast<uint32_t>(b.mn);
        w[1] = static_cast<uint32_t>(static_cast<uint64_t>(b.mn) >> 32);
        __builtin_amdgcn_raw_buffer_store_b64(w, r_mn, off, 0, 0);
    };

    // kFirst / kLast: the plan's first / last tile (both for a row of one tile)
    auto do_tile = [&](int32_t tile_lo, auto first_tag, auto last_tag) {
        const Ids L = fresh_ids();
        constexpr bool kFirst = decltype(first_tag)::value, kLast = decltype(last_tag)::value;
        const std::integral_constant<bool, !kFirst> prev_full{};
        const int32_t tile_hi = tile_lo + kTile < a.T ? tile_lo + kTile : a.T;
        // loads first: the cells of the tile that follows (the next plan's first one after a last
        // tile; dMF0 is padded to whole tiles), then the next plan's intervals
        {   // (uniform base plus a 32-bit byte offset: no 64-bit address is kept per L.lane)
            const uint32_t at = static_cast<uint32_t>((kLast ? 0 : tile_lo + kTile) + L.fill_at) * 8u;
            const char *cells = reinterpret_cast<const char *>(a.dMF0) + at;
#pragma unroll
            for (int j = 0; j < kVpt / 2; ++j) fill[j] = *reinterpret_cast<const ll2 *>(cells + 1024 * j);
        }
        // The next plan's intervals are requested in this plan's first tile and their sizes (which come from the
        // L2) in its last, into registers of their own: every vector memory instruction of the CU queues behind
        // the stores that have not left it yet (most of a tile's worth when the rows are written) and the lists
        // then come from HBM while it is busy with those stores.  Requested where this plan's registers become
        // free (after the last scatter) they were waited for during most of a tile; one tile ahead changed little
        // (c3 with rows 1.745 ms either way), a whole row ahead does (1.57).
        if constexpr (kFirst && !kLast) load_list(L, nk0, nk1);
        if constexpr (kLast && !kFirst) load_sizes(L, nk0, nk1);
        __builtin_amdgcn_wave_barrier();
        store_part(L, 0, prev_full);

        // ---- scatter
        const bool mine = hi_t >= tile_lo && lo_t < tile_hi;
        if (__builtin_amdgcn_ballot_w64(mine) != 0) {
            const uint32_t tile_bytes = __builtin_amdgcn_readfirstlane(skew(static_cast<uint32_t>(tile_lo)) * 8u);
            const uint32_t trash = (kTileCells + L.lane) * 8u;
            char *const cells = reinterpret_cast<char *>(delta);
#pragma unroll
            for (int j = 0; j < R; ++j) {   // (as in eval_body)
                const uint32_t u0 = e0[j] - tile_bytes, u1 = e1[j] - tile_bytes;
                typename SR::type s = sz[j];
                opaque(s);
                const int64_t bytes = SR::bytes(a, s);
                lds_sub(reinterpret_cast<int64_t *>(cells + (u0 < trash ? u0 : trash)), bytes);
                lds_add(reinterpret_cast<int64_t *>(cells + (u1 < trash ? u1 : trash)), bytes);
            }
        }
        // (a row of one tile: the next plan's intervals as soon as this plan's have been scattered)
        if constexpr (kLast && kFirst) load_list(L, nk0, nk1);
        // The offsets of the plan after the next come through the scalar unit, whose loads every wait for an LDS
        // operation waits for as well: the first wavefront, which is the one with time to spare before this barrier,
        // fetches them for all.
        if constexpr (kFirst) {
            if (L.wave_u == 0 && ahead < a.B) {
                const int64_t c0 = plan_offsets[ahead], c1 = plan_offsets[ahead + 1];
                if (L.lane == 0) {
                    ahead_off[ahead_slot][0] = c0;
                    ahead_off[ahead_slot][1] = c1;
                }
            }
        }
        store_part(L, 1, prev_full);
        __syncthreads();
        if constexpr (kFirst) {
            write_result(L);
            done_plan = -1;
        }

        // ---- local scan; the cells receive the following tile
        const bool wave_live = tile_lo + L.wave_u * (64 * kVpt) < tile_hi;
        int64_t v[kVpt];
        int64_t incl = 0;
        {
            const ll2 *cell = reinterpret_cast<const ll2 *>(&delta[L.my_cell]);
            if (wave_live) {
#pragma unroll
                for (int j = 0; j < kVpt / 2; ++j) {
                    const ll2 x = cell[j];
                    v[2 * j] = x[0];
                    v[2 * j + 1] = x[1];
                }
                __builtin_amdgcn_sched_barrier(0);   // (the wavefront's reads before its writes, as in eval_body)
#pragma unroll
                for (int j = 0; j < kVpt / 2; ++j) *reinterpret_cast<ll2 *>(&delta[L.fill_cell + 136 * j]) = fill[j];
#pragma unroll
                for (int j = 1; j < kVpt; ++j) v[j] += v[j - 1];
                incl = wave_scan_add(v[kVpt - 1]);
            } else {   // (only in a row's ragged last tile: nothing to scan, but the next plan needs its cells)
#pragma unroll
                for (int j = 0; j < kVpt / 2; ++j) *reinterpret_cast<ll2 *>(&delta[L.fill_cell + 136 * j]) = fill[j];
#pragma unroll
                for (int j = 0; j < kVpt; ++j) v[j] = 0;
            }
        }
        if (L.lane == 63) wave_tot[L.wave] = incl;
        if constexpr (kLast && kFirst) load_sizes(L, nk0, nk1);
        store_part(L, 2, prev_full);
        __syncthreads();
        if (wave_live) {
            int64_t tot = wave_tot[L.lane & (kWaves - 1)];
            tot += dpp_or_zero<0x111, 0xf>(tot);
            tot += dpp_or_zero<0x112, 0xf>(tot);
            tot += dpp_or_zero<0x114, 0xf>(tot);
            if constexpr (kWaves > 8) tot += dpp_or_zero<0x118, 0xf>(tot);
            const int64_t before = L.wave_u > 0 ? lane_value(tot, L.wave_u - 1) : 0;
            const int64_t base = carry + before + incl - v[kVpt - 1];
            carry += lane_value(tot, kWaves - 1);
#pragma unroll
            for (int j = 0; j < kVpt; ++j) v[j] += base;

            // ---- reduce (as in eval_body)
            const int32_t t0 = tile_lo + L.my;
            if (t0 + kVpt <= tile_hi) {
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
                    if (__builtin_amdgcn_ballot_w64(diff != 0) == 0) {   // L.wave-uniform
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
        }
        // ---- the previous tile's last quarter leaves the staging area, this tile's results enter it
        store_part(L, 3, prev_full);
        __builtin_amdgcn_wave_barrier();
        if constexpr (kStore) {
            ll2 *mine_out = reinterpret_cast<ll2 *>(L.stage + L.lane * kVpt + 2 * (L.lane >> 2));
#pragma unroll
            for (int j = 0; j < kVpt / 2; ++j) mine_out[j] = ll2{v[2 * j], v[2 * j + 1]};
        }
        prev_row = row;
        prev_lo = tile_lo;
        prev_hi = tile_hi;
    };

    int64_t next = next_mine(plan + stride);
    if (next < a.B) list_of(next, nk0, nk1);
    for (;;) {
        ahead = next < a.B && next + stride < a.B ? next + stride : a.B;
        row = kStore ? a.resident + plan * a.T : nullptr;
        carry = 0;
        best = Best{INT64_MIN, INT64_MAX, INT32_MAX};
        if (a.T <= kTile) {
            do_tile(0, std::true_type{}, std::true_type{});
        } else {
            do_tile(0, std::true_type{}, std::false_type{});
            int32_t tile_lo = kTile;
            for (; tile_lo + kTile < a.T; tile_lo += kTile) do_tile(tile_lo, std::false_type{}, std::false_type{});
            do_tile(tile_lo, std::false_type{}, std::true_type{});
        }
        // this wavefront's share of the plan's result
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
        done_plan = plan;
        if (next >= a.B) break;
        take_list();
        plan = next;
        // the plan after it: the one whose offsets were fetched during the first tile (the last barrier lies
        // between that write and this read, and the slots alternate, so the first wavefront's write for the plan
        // after cannot overtake a wavefront that still reads here), unless it is left to the tail kernel
        next = a.B;
        nk0 = 0;
        nk1 = 0;
        if (ahead < a.B) {
            int64_t c0 = uniform(ahead_off[ahead_slot][0]), c1 = uniform(ahead_off[ahead_slot][1]);
            if (c0 < 0) c0 = 0;
            if (c1 > a.n_intervals) c1 = a.n_intervals;
            if (c1 < c0) c1 = c0;
            if (c1 - c0 <= a.tail_threshold) {
                next = ahead;
                nk0 = c0;
                nk1 = c1;
            } else {
                next = next_mine(ahead);
                if (next < a.B) list_of(next, nk0, nk1);
            }
        }
        ahead_slot ^= 1;
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int j = 0; j < kVpt / 2; ++j) store_part(fresh_ids(), j, std::false_type{});
    __syncthreads();
    write_result(fresh_ids());
}

// The tail kernel runs after the common one on the same stream with a small persistent grid.  It does nothing
// unless the common kernel met a plan it had to leave (flag == this launch's epoch).  Then every workgroup
// walks the batch's offsets, kThr plans at a time, numbers the long plans as it meets them (ballots: the count
// is the same in every workgroup), and takes the (long plan, segment) pairs whose running number is its own
// modulo the grid: the long plans are spread evenly over the workgroups wherever they sit in the batch.
template <int kThr, bool kNarrow, int kOut>
__global__ __launch_bounds__(kThr) void eval_tail_kernel(const EvalArgs a) {
    if (*a.tail_flag != a.epoch) return;
    constexpr int kWaves = kThr / 64;
    __shared__ EvalLds<kThr> lds;
    __shared__ unsigned long long long_mask[kWaves];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int32_t grid = static_cast<int32_t>(gridDim.x), me = static_cast<int32_t>(blockIdx.x);
    const int32_t s_step = a.S % grid;
    int32_t item_mod = 0;     // (number of the long plan at hand) * S modulo the grid: block-uniform, kept without divisions
    for (int64_t base = 0; base < a.B; base += kThr) {
        const int64_t p = base + tid;
        bool is_long = false;
        if (p < a.B) {
            int64_t k0 = a.plan_offsets[p], k1 = a.plan_offsets[p + 1];
            if (k0 < 0) k0 = 0;
            if (k1 > a.n_intervals) k1 = a.n_intervals;
            is_long = k1 - k0 > a.tail_threshold;
        }
        const unsigned long long mine = __builtin_amdgcn_ballot_w64(is_long);
        if (lane == 0) long_mask[wave] = mine;
        __syncthreads();
        for (int w = 0; w < kWaves; ++w) {
            const unsigned long long m_any = long_mask[w];
            unsigned long long m = (static_cast<unsigned long long>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(m_any >> 32))) << 32) |
                                   __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(m_any));
            while (m) {       // (block-uniform)
                const int32_t plan = static_cast<int32_t>(base + w * 64 + __builtin_ctzll(m));
                m &= m - 1;
                // this workgroup's segments of the plan: those whose item number, long plan * S + seg, is its own modulo the grid
                for (int32_t seg = me >= item_mod ? me - item_mod : me - item_mod + grid; seg < a.S; seg += grid) {
                    eval_body<kThr, kCapTail / kThr, true, kNarrow, kOut>(a, plan, seg, lds);
                    __syncthreads();   // LDS is reused by the next pair
                }
                item_mod += s_step;
                if (item_mod >= grid) item_mod -= grid;
            }
        }
        __syncthreads();   // everybody has read the masks
    }
}

// ---- batches of long plans -------------------------------------------------------------
// When the average plan is longer than the registers hold, the whole batch is binned first:
// one workgroup per plan sorts the plan's endpoints by tile (counting sort with LDS counters;
// two passes over the plan) into records {cell | sign, size units} and sums each tile's deltas.
// The evaluation kernel then reads, per tile, only that tile's records, and takes the running
// sum entering a segment from the tile sums.  Records of a tile are in no particular order
// (integer additions commute).
constexpr int kMaxBinTiles = 4096;
constexpr int kBinU = 4;   // intervals per thread and round of bin_kernel's passes

// kSums: the tiles' delta sums are wanted (rows cut into several segments take their entering sums from them).
// Without them the first pass needs no sizes: it reads the steps only, and an interval whose tensor index is
// out of range is counted there like any other and gets records of size zero in the second pass.
template <int kThr, bool kSums>
__global__ __launch_bounds__(1024) void bin_kernel(const EvalArgs a, int2 *recs_all, int32_t *tile_off, int64_t *tile_sum) {
    constexpr int kTile = Geom<kThr>::kTile;
    __shared__ int32_t cnt[kMaxBinTiles + 1];
    __shared__ int64_t sum[kMaxBinTiles];
    __shared__ int32_t wave_cnt[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int32_t plan = blockIdx.x, nt = a.n_tiles;
    int64_t k0 = a.plan_offsets[plan], k1 = a.plan_offsets[plan + 1];
    if (k0 < 0) k0 = 0;
    if (k1 > a.n_intervals) k1 = a.n_intervals;
    if (k1 < k0) k1 = k0;
    for (int32_t t = tid; t <= nt; t += 1024) cnt[t] = 0;
    for (int32_t t = tid; t < nt; t += 1024) sum[t] = 0;
    __syncthreads();
    // Both passes take kBinU intervals per thread and round: their loads are issued together (at clamped
    // indices, so unconditionally), then the size gathers together.  The rounds are counted per wavefront, so
    // that all 64 lanes stay in the loop to its end (the wavefront-wide operations below need them).
    const int64_t n_iv = k1 - k0;
    auto load_round = [&](int64_t kb, int32_t (&i)[kBinU], int32_t (&o)[kBinU], int32_t (&r)[kBinU], uint32_t (&units)[kBinU]) {
#pragma unroll
        for (int u = 0; u < kBinU; ++u) {
            const int64_t k = kb + u * 1024;
            const int64_t kc = k < k1 ? k : k1 - 1;      // (only called on a list that is not empty)
            // (nontemporal: the second pass, which these loads serve - and the first when tile sums are wanted - is the
            // last to read the lists: 2.50 -> 2.48 ms for the call on c4; on the counting pass's own loads and on the
            // record stores the same hint changes nothing or costs)
            i[u] = __builtin_nontemporal_load(a.iv_tensor + kc);
            o[u] = __builtin_nontemporal_load(a.iv_out + kc);
            r[u] = __builtin_nontemporal_load(a.iv_in + kc);
        }
#pragma unroll
        for (int u = 0; u < kBinU; ++u) {
            if (kb + u * 1024 >= k1 || !applies(a, i[u], o[u], r[u])) i[u] = -1;
            units[u] = a.size_units[i[u] < 0 ? 0 : i[u]];
        }
    };
    // A caller's list keeps the intervals of one tensor, and of tensors generated one after the other, together,
    // so the 64 endpoints a wavefront holds at a time mostly fall into one or two tiles - and LDS atomics of 64
    // lanes on one address take 64 turns.  The wavefront therefore handles its endpoints tile by tile: f(tile,
    // lanes holding it, the lowest of them) once per distinct tile among the lanes with `active` set.
    auto for_each_tile = [&](bool active, int32_t tl, auto f) {
        uint64_t todo = __ballot(active);
        while (todo) {   // (wave-uniform)
            const int leader = __builtin_ctzll(todo);
            const int32_t t = __builtin_amdgcn_readlane(tl, leader);
            const uint64_t group = __ballot(active && tl == t);
            f(t, group, leader);
            todo &= ~group;
        }
    };
    // which intervals the passes take when the sizes are not looked at: those whose steps can be applied
    auto steps_apply = [&](int32_t o, int32_t r) { return o >= a.o_min && r <= a.T && r > o; };
    for (int64_t base = wave * 64; base < n_iv; base += kBinU * 1024) {
        int32_t i[kBinU], o[kBinU], r[kBinU];
        uint32_t units[kBinU];
        if constexpr (kSums) {
            load_round(k0 + base + lane, i, o, r, units);
        } else {
#pragma unroll
            for (int u = 0; u < kBinU; ++u) {
                const int64_t k = k0 + base + lane + u * 1024;
                const int64_t kc = k < k1 ? k : k1 - 1;
                o[u] = a.iv_out[kc];
                r[u] = a.iv_in[kc];
                i[u] = (k < k1 && steps_apply(o[u], r[u])) ? 0 : -1;
                units[u] = 0;
            }
        }
#pragma unroll
        for (int u = 0; u < kBinU; ++u) {
            const int64_t bytes = static_cast<int64_t>(static_cast<uint64_t>(units[u]) << a.size_shift);
            const bool has_out = i[u] >= 0 && o[u] + 1 < a.T, has_in = i[u] >= 0 && r[u] < a.T;
            const int32_t tl_out = (o[u] + 1) / kTile, tl_in = r[u] / kTile;
            for_each_tile(has_out, tl_out, [&](int32_t t, uint64_t group, int leader) {
                if constexpr (kSums) {
                    const int64_t tot = last_lane(wave_scan_add(has_out && tl_out == t ? bytes : 0));
                    if (lane == leader) lds_sub(&sum[t], tot);
                }
                if (lane == leader) atomicAdd(&cnt[t], __popcll(group));
            });
            for_each_tile(has_in, tl_in, [&](int32_t t, uint64_t group, int leader) {
                if constexpr (kSums) {
                    const int64_t tot = last_lane(wave_scan_add(has_in && tl_in == t ? bytes : 0));
                    if (lane == leader) lds_add(&sum[t], tot);
                }
                if (lane == leader) atomicAdd(&cnt[t], __popcll(group));
            });
        }
    }
    __syncthreads();
    // exclusive prefix of the counts, 4 consecutive tiles per thread (nt <= 4096)
    {
        int32_t c[4], run = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            c[j] = 4 * tid + j < nt ? cnt[4 * tid + j] : 0;
            run += c[j];
        }
        const int32_t incl = static_cast<int32_t>(wave_scan_add(run));
        if (lane == 63) wave_cnt[wave] = incl;
        __syncthreads();
        int32_t before = incl - run;
        for (int v = 0; v < wave; ++v) before += wave_cnt[v];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (4 * tid + j <= nt) cnt[4 * tid + j] = before;      // (entry nt receives the total)
            before += c[j];
        }
    }
    __syncthreads();
    int32_t *off_out = tile_off + static_cast<int64_t>(plan) * (nt + 1);
    int64_t *sum_out = tile_sum + static_cast<int64_t>(plan) * nt;
    for (int32_t t = tid; t <= nt; t += 1024) off_out[t] = cnt[t];
    for (int32_t t = tid; t < nt; t += 1024) sum_out[t] = sum[t];
    __syncthreads();
    // second pass: cnt[] now serves as the tiles' write cursors
    int2 *recs = recs_all + 2 * k0;
    const uint64_t lanes_below = (1ull << lane) - 1;
    for (int64_t base = wave * 64; base < n_iv; base += kBinU * 1024) {
        int32_t i[kBinU], o[kBinU], r[kBinU];
        uint32_t units[kBinU];
        load_round(k0 + base + lane, i, o, r, units);
        if constexpr (!kSums) {   // (the first pass counted by the steps alone)
#pragma unroll
            for (int u = 0; u < kBinU; ++u) {
                if (i[u] < 0 && base + lane + u * 1024 < n_iv && steps_apply(o[u], r[u])) {
                    i[u] = 0;
                    units[u] = 0;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kBinU; ++u) {
            const bool has_out = i[u] >= 0 && o[u] + 1 < a.T, has_in = i[u] >= 0 && r[u] < a.T;
            const int32_t tl_out = (o[u] + 1) / kTile, tl_in = r[u] / kTile;
            // the group's records go to consecutive places: one atomic per group reserves them
            for_each_tile(has_out, tl_out, [&](int32_t t, uint64_t group, int leader) {
                int32_t at = 0;
                if (lane == leader) at = atomicAdd(&cnt[t], __popcll(group));
                at = __builtin_amdgcn_readlane(at, leader) + __popcll(group & lanes_below);
                if (has_out && tl_out == t)
                    recs[at] = make_int2(static_cast<int32_t>(skew(o[u] + 1 - t * kTile) | 0x80000000u), static_cast<int32_t>(units[u]));
            });
            for_each_tile(has_in, tl_in, [&](int32_t t, uint64_t group, int leader) {
                int32_t at = 0;
                if (lane == leader) at = atomicAdd(&cnt[t], __popcll(group));
                at = __builtin_amdgcn_readlane(at, leader) + __popcll(group & lanes_below);
                if (has_in && tl_in == t) recs[at] = make_int2(static_cast<int32_t>(skew(r[u] - t * kTile)), static_cast<int32_t>(units[u]));
            });
        }
    }
}

// Two launches per binned batch: kFast takes the plans none of whose tiles holds more records than the
// fast form's two per thread, the other launch the rest; a workgroup whose plan belongs to the other
// launch exits at once.  (Checked over the whole plan, not only the workgroup's segment, so that all
// segments of a plan agree.)
template <int kThr, int kOut, bool kFast>
__global__ __launch_bounds__(kThr) __attribute__((amdgpu_waves_per_eu(4, 4))) void eval_binned_kernel(const EvalArgs a) {
    int32_t plan, seg;
    if (!decode_block(a, blockIdx.x, plan, seg)) return;
    bool over = false;
    const int32_t *off = a.tile_off + static_cast<int64_t>(plan) * (a.n_tiles + 1);
    for (int32_t t = threadIdx.x; t < a.n_tiles; t += kThr) over = over || off[t + 1] - off[t] > kBinFastRecs * kThr;
    if ((__syncthreads_or(over) != 0) == kFast) return;
    __shared__ EvalLds<kThr> lds;
    eval_body<kThr, 1, false, true, kOut, true, kFast>(a, plan, seg, lds);
}

// Combine the per-segment partials of each plan; segments are in time order, so
// a strict '>' keeps the earliest step.
__global__ void eval_finalize_kernel(int32_t B, int32_t S, const int64_t *part_max, const int32_t *part_arg,
                                     const int64_t *part_min, int64_t *peak, int32_t *argmax, int64_t *min_resident) {
    const int32_t b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int64_t base = static_cast<int64_t>(b) * S;
    int64_t mx = part_max[base], mn = part_min[base];
    int32_t arg = part_arg[base];
    for (int32_t s = 1; s < S; ++s) {
        const int64_t v = part_max[base + s];
        if (v > mx) {
            mx = v;
            arg = part_arg[base + s];
        }
        const int64_t m = part_min[base + s];
        if (m < mn) mn = m;
    }
    peak[b] = mx;
    argmax[b] = arg;
    if (min_resident) min_resident[b] = mn;
}

// Rows whose unscheduled timeline (8 bytes per step, read by every workgroup tile by tile) is larger than this
// are written with nontemporal stores.  Ordinary stores allocate their lines in the L2 of the XCD, and the
// stream of rows then pushes dMF0 out between two workgroups' reads of the same tile; every tile of every
// workgroup ends up waiting for a miss.  Measured with a plain probe (1024 workgroups copying a shared buffer
// into their own 8 MB rows through LDS, one tile ahead): shared buffer of 0.4 MB 5.9 TB/s with ordinary and 5.65
// with nontemporal stores; 2 MB 4.1 and 5.6; 8 MB 3.7 and 5.85.
constexpr int64_t kStreamRowsBytes = 1 << 20;

constexpr int kSmallGeometryMaxT = 16384;   // rows up to this length use the 512-thread geometry

// Whether a batch whose average plan holds `avg` intervals, on rows of n_tiles tiles, is sorted by tile first.
// Sorting costs a pass of its own (two reads of the lists, 16 bytes of records per interval written and read
// back) that is spread over the row's tiles; without it a plan's intervals beyond the 8192 a workgroup keeps
// in registers are read again for every tile.  Per tile, in microseconds, measured on rows of 10^6 and of
// 50,000 steps with 9,000 to 60,000 intervals per plan: re-reading 0.35 per 1024 intervals beyond the registers,
// sorting 1.5 + 3 per 1024 intervals of the plan divided by the number of tiles.  (Long rows: sorted from about
// 12,000 intervals per plan; rows of a few tiles: never - 16,000 intervals on 7 tiles take 1.18 ms for 4,096
// plans re-read and 1.72 ms sorted.)
bool binning_pays(double avg, int64_t n_tiles) {
    if (avg <= kCapTail) return false;
    return 0.35 * (avg - kCapTail) / 1024.0 > 1.5 + 3.0 * avg / 1024.0 / static_cast<double>(n_tiles);
}

// The launches of one geometry: common kernel (three register capacities), tail kernel.
template <int kThr>
int launch_geometry(const tensile_tas *tas, Workspace &ws, const EvalArgs &a, int64_t blocks, int cap, int out, bool narrow,
                    bool binned, bool persistent) {
    const hipStream_t stream = ws.stream;
    dim3 grid(static_cast<uint32_t>(blocks)), block(kThr);
    if (binned) {
        if (a.S > 1) hipLaunchKernelGGL((bin_kernel<kThr, true>), dim3(a.B), dim3(1024), 0, stream, a, ws.bin_recs.p, ws.bin_off.p, ws.bin_sum.p);
        else hipLaunchKernelGGL((bin_kernel<kThr, false>), dim3(a.B), dim3(1024), 0, stream, a, ws.bin_recs.p, ws.bin_off.p, ws.bin_sum.p);
        TS_HIP(hipGetLastError());
        if (out == 3) {
            hipLaunchKernelGGL((eval_binned_kernel<kThr, 3, true>), grid, block, 0, stream, a);
            hipLaunchKernelGGL((eval_binned_kernel<kThr, 3, false>), grid, block, 0, stream, a);
        } else if (out >= 2) {
            hipLaunchKernelGGL((eval_binned_kernel<kThr, 2, true>), grid, block, 0, stream, a);
            hipLaunchKernelGGL((eval_binned_kernel<kThr, 2, false>), grid, block, 0, stream, a);
        } else if (out == 1) {
            hipLaunchKernelGGL((eval_binned_kernel<kThr, 1, true>), grid, block, 0, stream, a);
            hipLaunchKernelGGL((eval_binned_kernel<kThr, 1, false>), grid, block, 0, stream, a);
        } else {
            hipLaunchKernelGGL((eval_binned_kernel<kThr, 0, true>), grid, block, 0, stream, a);
            hipLaunchKernelGGL((eval_binned_kernel<kThr, 0, false>), grid, block, 0, stream, a);
        }
        TS_HIP(hipGetLastError());
        return TENSILE_OK;
    }
#define TS_LAUNCH_OUT(KERNEL, ...)                                                                   \
    do {                                                                                             \
        if (out >= 2) hipLaunchKernelGGL((KERNEL<__VA_ARGS__, 2>), grid, block, 0, stream, a);       \
        else if (out == 1) hipLaunchKernelGGL((KERNEL<__VA_ARGS__, 1>), grid, block, 0, stream, a);  \
        else hipLaunchKernelGGL((KERNEL<__VA_ARGS__, 0>), grid, block, 0, stream, a);                \
    } while (0)
#define TS_LAUNCH_EVAL(R)                                                    \
    do {                                                                     \
        if (persistent) {                                                    \
            if (narrow) TS_LAUNCH_OUT(eval_stream_kernel, kThr, R, true);    \
            else TS_LAUNCH_OUT(eval_stream_kernel, kThr, R, false);          \
        } else {                                                             \
            if (narrow) TS_LAUNCH_OUT(eval_kernel, kThr, R, true);           \
            else TS_LAUNCH_OUT(eval_kernel, kThr, R, false);                 \
        }                                                                    \
    } while (0)
    // (with 512 threads only the smallest register capacity leaves room for the next plan's intervals)
    if (kThr == 512 && cap != kCapSmall) persistent = false;
    if (persistent) {   // one workgroup per resident slot, the plans dealt evenly among them
        int64_t slots = static_cast<int64_t>(tas->num_cus) * (1024 / kThr);
        if (g_tuning.eval_slots > 0) slots = g_tuning.eval_slots;
        const int64_t rounds = (blocks + slots - 1) / slots;
        grid = dim3(static_cast<uint32_t>((blocks + rounds - 1) / rounds));
    }
    if (out == 3 && kThr == 1024 && !persistent) {   // nontemporal rows: compiled for the large geometry only (long rows use no other)
#define TS_LAUNCH_NT(R)                                                                                  \
    do {                                                                                                 \
        if (narrow) hipLaunchKernelGGL((eval_kernel<1024, R, true, 3>), grid, block, 0, stream, a);      \
        else hipLaunchKernelGGL((eval_kernel<1024, R, false, 3>), grid, block, 0, stream, a);            \
    } while (0)
        if (cap == kCapSmall) TS_LAUNCH_NT(kCapSmall / 1024);
        else if (cap == kCapMid) TS_LAUNCH_NT(kCapMid / 1024);
        else if (cap == kCapTail) TS_LAUNCH_NT(kCapTail / 1024);
        else TS_LAUNCH_NT(kCapBig / 1024);
#undef TS_LAUNCH_NT
    } else if (cap == kCapSmall) TS_LAUNCH_EVAL(kCapSmall / kThr);
    else if (cap == kCapMid) TS_LAUNCH_EVAL(kCapMid / kThr);
    else if (cap == kCapTail && kThr == 1024) {   // (one workgroup per plan only: the host does not ask for the persistent grid here)
        if (narrow) TS_LAUNCH_OUT(eval_kernel, 1024, kCapTail / 1024, true);
        else TS_LAUNCH_OUT(eval_kernel, 1024, kCapTail / 1024, false);
    } else TS_LAUNCH_EVAL(kCapBig / kThr);
    TS_HIP(hipGetLastError());
#undef TS_LAUNCH_EVAL
#undef TS_LAUNCH_OUT
    if (a.n_intervals > a.tail_threshold) {   // (otherwise no plan can be longer than the registers hold)
        const int64_t resident = static_cast<int64_t>(tas->num_cus) * (1024 / kThr);
        const dim3 tgrid(static_cast<uint32_t>(blocks < resident ? blocks : resident));
#define TS_LAUNCH_TAIL(NARROW)                                                                                            \
    do {                                                                                                                  \
        if (out == 3 && kThr == 1024) hipLaunchKernelGGL((eval_tail_kernel<1024, NARROW, 3>), tgrid, block, 0, stream, a); \
        else if (out >= 2) hipLaunchKernelGGL((eval_tail_kernel<kThr, NARROW, 2>), tgrid, block, 0, stream, a);   \
        else if (out == 1) hipLaunchKernelGGL((eval_tail_kernel<kThr, NARROW, 1>), tgrid, block, 0, stream, a);   \
        else hipLaunchKernelGGL((eval_tail_kernel<kThr, NARROW, 0>), tgrid, block, 0, stream, a);                 \
    } while (0)
        if (narrow) TS_LAUNCH_TAIL(true);
        else TS_LAUNCH_TAIL(false);
#undef TS_LAUNCH_TAIL
    }
    TS_HIP(hipGetLastError());
    return TENSILE_OK;
}

// The smallest geometry: 256 threads, 2048-step tiles, 36 KB of LDS, four workgroups per CU.  Only the common
// kernel with 8 intervals per thread (plans of up to 2048 intervals; longer ones go to the tail kernel).
int launch_tiny_geometry(const tensile_tas *tas, Workspace &ws, const EvalArgs &a, int64_t blocks, int out, bool narrow) {
    constexpr int kThr = 256;
    const hipStream_t stream = ws.stream;
    const dim3 grid(static_cast<uint32_t>(blocks)), block(kThr);
    const int64_t resident = static_cast<int64_t>(tas->num_cus) * (1024 / kThr);
    const dim3 tgrid(static_cast<uint32_t>(blocks < resident ? blocks : resident));
#define TS_LAUNCH_TINY(NARROW, OUT)                                                                                  \
    do {                                                                                                             \
        hipLaunchKernelGGL((eval_kernel<kThr, kCapSmall / kThr, NARROW, OUT>), grid, block, 0, stream, a);           \
        if (a.n_intervals > a.tail_threshold) /* else no plan can be longer than the registers hold */              \
            hipLaunchKernelGGL((eval_tail_kernel<kThr, NARROW, OUT>), tgrid, block, 0, stream, a);                   \
    } while (0)
    if (narrow) {
        if (out >= 2) TS_LAUNCH_TINY(true, 2);
        else if (out == 1) TS_LAUNCH_TINY(true, 1);
        else TS_LAUNCH_TINY(true, 0);
    } else {
        if (out >= 2) TS_LAUNCH_TINY(false, 2);
        else if (out == 1) TS_LAUNCH_TINY(false, 1);
        else TS_LAUNCH_TINY(false, 0);
    }
#undef TS_LAUNCH_TINY
    TS_HIP(hipGetLastError());
    return TENSILE_OK;
}

// ---- one more interval per plan: windowed update -----------------------------------------
// The rows exist already; plan b gains the interval (tensor[b], out[b], in[b]).  A workgroup takes a
// run of 8192-step chunks of one row: 16 contiguous bytes per lane and load, one chunk ahead; the
// window's steps lose the tensor's size and are the only ones written back; the run's (max, earliest
// argmax, min) go to the per-segment partials that eval_finalize_kernel combines, or straight to the
// outputs when a row is one run.  Reads 8 bytes per step, writes 8 per step of the window.
constexpr int kApplyThr = 1024, kApplyChunk = kApplyThr * 8;

struct ApplyArgs {
    int32_t T, N, S, chunks_per_group;
    const int64_t *size;
    const int32_t *tensor, *out, *in;      // [B] the new intervals
    int64_t *resident;
    int64_t *part_max, *part_min;          // [B*S] per-run partials when S > 1
    int32_t *part_arg;
    unsigned int *tickets;                 // [B] zero between launches: runs of a row that have finished (S > 1)
    int64_t *peak, *min_resident;          // [B] results (min may be null)
    int32_t *argmax;
};

template <bool kVec16>
__global__ __launch_bounds__(kApplyThr) void apply_interval_kernel(const ApplyArgs a) {
    constexpr int kWaves = kApplyThr / 64;
    __shared__ int64_t red_mx[kWaves], red_mn[kWaves];
    __shared__ int32_t red_arg[kWaves];
    const int32_t T = a.T, S = a.S;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t plan = blockIdx.x / S;
    const int32_t group = static_cast<int32_t>(blockIdx.x % S);     // this workgroup's run of chunks of the row
    const int32_t g_lo = group * a.chunks_per_group * kApplyChunk;  // (fits: the host keeps S * chunks_per_group * chunk near T)
    const int32_t g_hi = T - g_lo < a.chunks_per_group * kApplyChunk ? T : g_lo + a.chunks_per_group * kApplyChunk;
    const int32_t i = a.tensor[plan], o = a.out[plan], r = a.in[plan];
    const bool ok = static_cast<uint32_t>(i) < static_cast<uint32_t>(a.N) && o >= 0 && r <= T && r > o;
    const int64_t sz = ok ? a.size[i] : 0;
    const int32_t win_lo = ok ? o + 1 : 0, win_hi = ok ? r : 0;   // steps win_lo .. win_hi - 1 change
    int64_t *row = a.resident + plan * T;
    Best best{INT64_MIN, INT64_MAX, INT32_MAX};
    auto take = [&](int32_t t, int64_t v) {   // (a thread meets its steps in ascending order)
        if (v > best.mx) {
            best.mx = v;
            best.arg = t;
        }
        if (v < best.mn) best.mn = v;
    };
    // the loads of a chunk are issued one chunk ahead (at clamped addresses past the end of the run)
    ll2 nxt[4];
    auto load_chunk = [&](int32_t lo) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int32_t t = lo + 2 * (j * kApplyThr + tid);
            if (kVec16) nxt[j] = *reinterpret_cast<const ll2 *>(row + (t + 2 <= T ? t : T - 2));
            else nxt[j] = ll2{row[t < T ? t : T - 1], row[t + 1 < T ? t + 1 : T - 1]};
        }
    };
    load_chunk(g_lo);
    for (int32_t lo = g_lo; lo < g_hi; lo += kApplyChunk) {
        ll2 cur[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) cur[j] = nxt[j];
        if (lo + kApplyChunk < g_hi) load_chunk(lo + kApplyChunk);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int32_t t = lo + 2 * (j * kApplyThr + tid);
            const bool in0 = t >= win_lo && t < win_hi, in1 = t + 1 >= win_lo && t + 1 < win_hi;
            ll2 x = cur[j];
            x[0] -= in0 ? sz : 0;
            x[1] -= in1 ? sz : 0;
            if (kVec16 && in0 && in1) {
                *reinterpret_cast<ll2 *>(row + t) = x;     // (t + 1 < win_hi <= T: both steps exist)
            } else {
                if (in0) row[t] = x[0];
                if (in1) row[t + 1] = x[1];
            }
            if (t < g_hi) take(t, x[0]);
            if (t + 1 < g_hi) take(t + 1, x[1]);
        }
    }
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
    if (tid != 0) return;
#pragma unroll
    for (int u = 1; u < kWaves; ++u) best_merge(best, red_mx[u], red_arg[u], red_mn[u]);
    if (S > 1) {
        // the run that finishes last combines the row's partials (they are in time order: a strict '>' keeps
        // the earliest step) and leaves the ticket counter at zero for the next launch
        const int64_t slot = plan * S + group;
        a.part_max[slot] = best.mx;
        a.part_arg[slot] = best.arg;
        a.part_min[slot] = best.mn;
        __threadfence();
        if (atomicAdd(&a.tickets[plan], 1u) != static_cast<unsigned int>(S - 1)) return;
        __threadfence();
        best = Best{INT64_MIN, INT64_MAX, INT32_MAX};
        for (int32_t s = 0; s < S; ++s) {
            const int64_t mx = __hip_atomic_load(&a.part_max[plan * S + s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int64_t mn = __hip_atomic_load(&a.part_min[plan * S + s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int32_t arg = __hip_atomic_load(&a.part_arg[plan * S + s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (mx > best.mx) {
                best.mx = mx;
                best.arg = arg;
            }
            if (mn < best.mn) best.mn = mn;
        }
        __hip_atomic_store(&a.tickets[plan], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    a.peak[plan] = best.mx;
    a.argmax[plan] = best.arg;
    if (a.min_resident) a.min_resident[plan] = best.mn;
}

}  // namespace

int launch_apply(const tensile_tas *tas, Workspace &ws, int32_t B, const int32_t *tensor, const int32_t *out,
                 const int32_t *in, int64_t *resident, int64_t *peak, int32_t *argmax, int64_t *min_resident) {
    if (B == 0) return TENSILE_OK;
    const hipStream_t stream = ws.stream;
    const int32_t T = tas->T;
    // a row is cut into runs of chunks, one workgroup each: one run per row when the batch fills the chip by
    // itself (no partials), otherwise enough runs for about four workgroups per CU
    const int64_t n_chunks = (static_cast<int64_t>(T) + kApplyChunk - 1) / kApplyChunk;
    const int64_t want = (4 * static_cast<int64_t>(tas->num_cus) + B - 1) / B;
    int64_t S = want < 1 ? 1 : want > n_chunks ? n_chunks : want;
    const int64_t per_group = (n_chunks + S - 1) / S;
    S = (n_chunks + per_group - 1) / per_group;
    const int64_t blocks = static_cast<int64_t>(B) * S;
    if (blocks > 0x7fffffffLL) {
        set_error("apply_intervals: B*runs = %lld workgroups exceeds the grid limit", static_cast<long long>(blocks));
        return TENSILE_E_INVAL;
    }
    ApplyArgs a{};
    a.T = T; a.N = tas->N; a.S = static_cast<int32_t>(S); a.chunks_per_group = static_cast<int32_t>(per_group);
    a.size = tas->d_size.p; a.tensor = tensor; a.out = out; a.in = in; a.resident = resident;
    a.peak = peak; a.argmax = argmax; a.min_resident = min_resident;
    if (S > 1) {
        const size_t n = static_cast<size_t>(blocks);
        int rc = ws.provide(ws.part_max, n, "apply_intervals: partial maxima");
        if (rc == TENSILE_OK) rc = ws.provide(ws.part_arg, n, "apply_intervals: partial peak steps");
        if (rc == TENSILE_OK) rc = ws.provide(ws.part_min, n, "apply_intervals: partial minima");
        bool fresh = false;
        if (rc == TENSILE_OK) rc = ws.provide(ws.apply_tickets, static_cast<size_t>(B), "apply_intervals: tickets", &fresh);
        if (rc == TENSILE_OK && fresh) rc = fill_words(stream, ws.apply_tickets.p, ws.apply_tickets.n, 0u);   // (kernels leave them at zero)
        if (rc != TENSILE_OK) return rc;
        a.part_max = ws.part_max.p; a.part_arg = ws.part_arg.p; a.part_min = ws.part_min.p;
        a.tickets = ws.apply_tickets.p;
    }
    const bool vec16 = (T % 2 == 0) && (reinterpret_cast<uintptr_t>(resident) % 16 == 0);
    const dim3 grid(static_cast<uint32_t>(blocks)), block(kApplyThr);
    if (vec16) hipLaunchKernelGGL(apply_interval_kernel<true>, grid, block, 0, stream, a);
    else hipLaunchKernelGGL(apply_interval_kernel<false>, grid, block, 0, stream, a);
    TS_HIP(hipGetLastError());
    return TENSILE_OK;
}

int launch_eval(const tensile_tas *tas, Workspace &ws, const EvalArgs &proto, int64_t *peak, int32_t *argmax,
                int64_t *min_resident) {
    EvalArgs a = proto;
    if (a.B == 0) return TENSILE_OK;
    const hipStream_t stream = ws.stream;
    // geometry: short rows get the small workgroups (see the top of the file).  So do batches of more than one
    // plan per CU when they write no rows or their rows have at most 32,768 steps: two workgroups per CU cover
    // each other's start.  Measured: 24,000-step rows, 8,192 plans 0.49 -> 0.43 ms, 384 plans 30.9 -> 26.5 us;
    // 50,000-step rows without row output, 16,384 plans 1.06 -> 0.91 ms per pass, 384 plans 39.0 -> 35.9 us.
    // With row output the two geometries are within 3 % of each other on 50,000-step rows whatever the batch,
    // and with at most one plan per CU the large geometry and its segments are ahead (256 plans: 29 vs 34 us).
    // intervals kept in registers by the common kernel: sized for the average plan with some
    // slack; longer plans are left to the tail kernel
    const int64_t avg_k = (a.n_intervals + a.B - 1) / a.B;
    int64_t need = avg_k + avg_k / 8;
    const int r_forced = g_tuning.eval_r;   // tuning knob: intervals per thread in registers at 1024 threads
    if (r_forced > 0) need = static_cast<int64_t>(r_forced) * 1024;
    int cap = need <= kCapSmall ? kCapSmall : need <= kCapMid ? kCapMid : need <= kCapBig ? kCapBig : kCapTail;
    const int bin_forced = g_tuning.eval_binned;   // tuning knob: 0 = never, 1 = whenever possible
    int threads = a.T <= kSmallGeometryMaxT ? 512 : 1024;
    if (a.B > tas->num_cus && (!a.resident || a.T <= 2 * kSmallGeometryMaxT)) threads = 512;
    const int threads_forced = g_tuning.eval_threads;   // tuning knob
    if (threads_forced == 512 || threads_forced == 1024) threads = threads_forced;
    // Rows up to 16,384 steps in batches of at least four plans per CU, plans short enough for 8 intervals per
    // thread: 256 threads, four workgroups per CU (it has neither a binned nor a persistent form).  Four
    // workgroups cover each other's starts better than two, and short rows waste less of their last tile:
    // 4,096 plans of 6,000 steps 70.8 -> 51.9 us, of 1,000 steps 46.9 -> 29.5, of 16,384 steps 157 -> 146;
    // on 300 plans the 512-thread geometry is level or ahead.
    const bool tiny_ok = cap == kCapSmall && bin_forced != 1;
    if (tiny_ok && threads_forced == 0 && a.T <= kSmallGeometryMaxT && a.B >= 4 * static_cast<int64_t>(tas->num_cus)) threads = 256;
    if (threads_forced == 256 && tiny_ok) threads = 256;
    if (cap == kCapTail && threads != 1024) cap = kCapBig;   // (8 intervals per thread only exist for 1024 threads)
    const bool small_for_batch = threads == 512 && a.T > kSmallGeometryMaxT;
    const int tile = threads * kVpt;
    const int64_t n_tiles = (static_cast<int64_t>(a.T) + tile - 1) / tile;
    // Segments per plan.  Every segment's workgroup starts with the plan's whole interval list (loads,
    // size gathers, the sum entering the segment), which costs about as much as p tiles of work, and more
    // than one segment needs the combining kernel afterwards (about one tile's time).  With the workgroups
    // running in rounds of one per CU, S is the count that minimises rounds x (p + tiles per segment):
    // several segments pay only while the batch leaves CUs idle, or for rows of very many tiles.
    int64_t S = 1;
    {
        const double avg = a.B > 0 ? static_cast<double>(a.n_intervals) / a.B : 0.0;
        const bool likely_binned = a.size_units != nullptr && n_tiles < kMaxBinTiles && binning_pays(avg, n_tiles);
        const double p = likely_binned ? 0.25 : 0.3 + (avg < kCapBig ? avg : kCapBig) / 3500.0;
        double best = 0.0;
        const int64_t s_max = n_tiles < 1024 ? n_tiles : 1024;
        for (int64_t s = 1; s <= s_max; ++s) {
            // (the small geometry chosen for the size of the batch: two workgroups per CU run side by side)
            const int64_t slots = small_for_batch ? 2 * static_cast<int64_t>(tas->num_cus) : tas->num_cus;
            const int64_t rounds = (static_cast<int64_t>(a.B) * s + slots - 1) / slots;
            const double cost = rounds * (p + static_cast<double>((n_tiles + s - 1) / s)) + (s > 1 ? 1.0 : 0.0);
            if (s == 1 || cost < best) {
                best = cost;
                S = s;
            }
        }
    }
    const int forced = g_tuning.eval_segments;   // tuning knob
    if (forced > 0) S = forced;
    if (S < 1) S = 1;
    // (the kernels keep an interval's endpoints as 32-bit byte offsets into the segment's cells: at most 2^28 steps
    // and a tile per segment)
    {
        const int64_t most = g_tuning.eval_seg_steps > 0 && g_tuning.eval_seg_steps < (1 << 28) ? g_tuning.eval_seg_steps : (1 << 28);
        const int64_t s_min = (static_cast<int64_t>(a.T) + most - 1) / most;
        if (S < s_min) S = s_min;
    }
    if (S > n_tiles) S = n_tiles;
    const int64_t tps = (n_tiles + S - 1) / S;
    S = (n_tiles + tps - 1) / tps;
    a.S = static_cast<int32_t>(S);
    a.tiles_per_seg = static_cast<int32_t>(tps);

    const int64_t groups = (static_cast<int64_t>(a.B) + 7) / 8;
    const int64_t blocks = groups * 8 * S;
    if (blocks > 0x7fffffffLL) {
        set_error("eval: B*segments = %lld workgroups exceeds the grid limit", static_cast<long long>(blocks));
        return TENSILE_E_INVAL;
    }
    if (S == 1) {
        a.out_max = peak;
        a.out_arg = argmax;
        a.out_min = min_resident;
    } else {
        const size_t n = static_cast<size_t>(a.B) * static_cast<size_t>(S);
        int rc = ws.provide(ws.part_max, n, "eval: partial maxima");
        if (rc == TENSILE_OK) rc = ws.provide(ws.part_arg, n, "eval: partial peak steps");
        if (rc == TENSILE_OK) rc = ws.provide(ws.part_min, n, "eval: partial minima");
        if (rc != TENSILE_OK) return rc;
        a.out_max = ws.part_max.p;
        a.out_arg = ws.part_arg.p;
        a.out_min = ws.part_min.p;
    }
    int out = !a.resident ? 0
              : ((a.T % 2 == 0) && (reinterpret_cast<uintptr_t>(a.resident) % 16 == 0)) ? 2 : 1;
    // long rows: nontemporal stores (see kStreamRowsBytes; tuning knob eval_nt: 0 never, 1 always).  Compiled for the
    // large geometry and for the binned kernels; which it is is known further down
    const bool nt_wanted = out == 2 && (g_tuning.eval_nt >= 0 ? g_tuning.eval_nt == 1
                                                              : static_cast<int64_t>(a.T) * 8 > kStreamRowsBytes);
    const bool narrow = a.size_units != nullptr;
    a.tail_threshold = cap;
    if (!ws.fixed_base) {   // (a fixed workspace brings its flag: zero when the code object is loaded, then monotone)
        bool fresh = false;
        const int rc = ws.provide(ws.tail_flag, 1, "eval: launch flag", &fresh);
        if (rc == TENSILE_OK && fresh) {
            const int rc_fill = fill_words(stream, ws.tail_flag.p, 2, 0u);
            if (rc_fill != TENSILE_OK) return rc_fill;
        }
        if (rc != TENSILE_OK) return rc;
    }
    a.tail_flag = ws.tail_flag.p;
    a.epoch = ++ws.epoch;
    // a batch whose average plan does not fit the registers is binned by tile first
    bool binned = narrow && n_tiles < kMaxBinTiles && a.n_intervals <= (INT32_MAX / 2) &&
                  binning_pays(static_cast<double>(a.n_intervals) / a.B, n_tiles);
    if (bin_forced == 0) binned = false;
    if (bin_forced == 1) binned = narrow && n_tiles < kMaxBinTiles && a.n_intervals <= (INT32_MAX / 2);
    if (a.n_intervals == 0) binned = false;   // nothing to bin (and no record for the binned kernel's clamped loads)
    if (binned) {
        const size_t n_recs = 2 * static_cast<size_t>(a.n_intervals), n_off = static_cast<size_t>(a.B) * (n_tiles + 1),
                     n_sum = static_cast<size_t>(a.B) * n_tiles;
        if (ws.fixed_base) {
            // a preallocated workspace that cannot hold the sorted records: the plans are evaluated from their
            // lists as they are (the tail kernel re-reads them per tile), slower but in no need of scratch
            const size_t need = (n_recs * sizeof(int2) + 255) / 256 * 256 + (n_off * sizeof(int32_t) + 255) / 256 * 256 +
                                (n_sum * sizeof(int64_t) + 255) / 256 * 256;
            if (need > ws.fixed_bytes - ws.fixed_used) binned = false;
        }
    }
    if (nt_wanted && (threads == 1024 || (binned && threads == 512))) out = 3;
    if (binned) {
        const size_t n_recs = 2 * static_cast<size_t>(a.n_intervals), n_off = static_cast<size_t>(a.B) * (n_tiles + 1),
                     n_sum = static_cast<size_t>(a.B) * n_tiles;
        int rc = ws.provide(ws.bin_recs, n_recs, "eval: sorted endpoint records");
        if (rc == TENSILE_OK) rc = ws.provide(ws.bin_off, n_off, "eval: tile offsets");
        if (rc == TENSILE_OK) rc = ws.provide(ws.bin_sum, n_sum, "eval: tile sums");
        if (rc != TENSILE_OK) return rc;
        a.recs = ws.bin_recs.p;
        a.tile_off = ws.bin_off.p;
        a.tile_sum = ws.bin_sum.p;
        a.n_tiles = static_cast<int32_t>(n_tiles);
    }
    // several plans per resident workgroup: the persistent kernel (it addresses a row's bytes with 32 bits)
    const bool pers_ok = S == 1 && !binned && a.N > 0 && a.T <= (1 << 28) && cap != kCapTail;
    // Without rows: batches of at least four plans per CU (where the host has not chosen two small workgroups per
    // CU, which are ahead there).  With rows, in the large geometry: the same batches when a row has at least three
    // tiles, from three plans per CU - the next plan's lists are then requested most of a row ahead (50,000-step
    // rows, 5,400 intervals per plan: 16,384 plans 1.66 -> 1.52 ms, 4,096 plans 0.423 -> 0.391, 768 plans 87 -> 78 us,
    // 512 plans 53 -> 55 us).
    const int64_t per_cu = a.B / tas->num_cus;
    bool persistent = pers_ok && ((out == 0 && per_cu >= 4) || (out != 0 && out != 3 && threads == 1024 && n_tiles >= 3 && per_cu >= 3));
    const int pers_forced = g_tuning.eval_persistent;   // tuning knob: 0 = never, 1 = whenever possible
    if (pers_forced == 0) persistent = false;
    if (pers_forced == 1) persistent = pers_ok;
    const int rc = threads == 256   ? launch_tiny_geometry(tas, ws, a, blocks, out, narrow)
                   : threads == 512 ? launch_geometry<512>(tas, ws, a, blocks, cap, out, narrow, binned, persistent)
                                    : launch_geometry<1024>(tas, ws, a, blocks, cap, out, narrow, binned, persistent);
    if (rc != TENSILE_OK) return rc;
    if (S > 1) {
        const int fthreads = 256;
        hipLaunchKernelGGL(eval_finalize_kernel, dim3((a.B + fthreads - 1) / fthreads), dim3(fthreads), 0, stream, a.B,
                           a.S, a.out_max, a.out_arg, a.out_min, peak, argmax, min_resident);
        TS_HIP(hipGetLastError());
    }
    return TENSILE_OK;
}

}  // namespace tensile

// ---- evaluation without any allocation ---------------------------------------------------
// For callers that cannot allocate (HIP graph capture, serving loops, harnesses that forbid it): the same
// kernels with their scratch in a preallocated device array instead of the handle's workspaces.  Every GPU
// the library runs on holds its own copy of the array for the life of the process.  Layout: the first 256
// bytes hold the launch flag of the evaluation kernels (zero when the code object is loaded, then only ever
// raised to the number of the latest launch, so it never needs clearing); the rest is carved up anew by every
// call (per-segment partials, the records of binned batches), all of it written before it is read.
constexpr size_t kStaticScratchBytes = size_t{16} << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
struct StaticWorkspace {
    std::once_flag once;
    hipError_t status = hipSuccess;
    tensile::Workspace ws;
};
StaticWorkspace g_static_ws[kMaxDevices];
}  // namespace

extern "C" int tensile_eval_plans_static(const tensile_tas *tas, const tensile_plans *plans, int64_t *resident, int64_t *peak,
                                         int32_t *argmax, int64_t *min_resident, void *hip_stream) {
    using namespace tensile;
    int rc = check_plans(tas, plans, "eval_plans_static");
    if (rc != TENSILE_OK) return rc;
    if (plans->B == 0) return TENSILE_OK;
    if (!peak || !argmax) { set_error("eval_plans_static: peak and argmax are required"); return TENSILE_E_INVAL; }
    int dev = -1;
    TS_HIP(hipGetDevice(&dev));
    if (dev != tas->device) {
        set_error("eval_plans_static: the handle lives on device %d, the current device is %d", tas->device, dev);
        return TENSILE_E_INVAL;
    }
    if (dev < 0 || dev >= kMaxDevices) { set_error("eval_plans_static: device %d is beyond the %d supported", dev, kMaxDevices); return TENSILE_E_RANGE; }
    StaticWorkspace &sw = g_static_ws[dev];
    // once per device, with that device current: where this device keeps its copy of the array
    std::call_once(sw.once, [&sw]() {
        void *ptr = nullptr;
        sw.status = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (sw.status != hipSuccess) return;
        sw.ws.fixed_base = static_cast<char *>(ptr);
        sw.ws.fixed_bytes = kStaticScratchBytes;
        sw.ws.tail_flag.owned = false;
        sw.ws.tail_flag.p = static_cast<unsigned long long *>(ptr);
        sw.ws.tail_flag.n = 1;
    });
    if (sw.status != hipSuccess) return hip_fail(sw.status, "hipGetSymbolAddress(scratch)");
    std::lock_guard<std::mutex> g(sw.ws.mu);   // (serialises the enqueueing only; see the header about overlapping calls)
    sw.ws.stream = static_cast<hipStream_t>(hip_stream);
    sw.ws.begin_call();
    EvalArgs a{};
    a.T = tas->T; a.N = tas->N; a.B = plans->B; a.o_min = 0; a.n_intervals = plans->n_intervals;
    a.plan_offsets = plans->plan_offsets;
    a.iv_tensor = plans->iv_tensor; a.iv_out = plans->iv_out; a.iv_in = plans->iv_in;
    a.size = tas->d_size.p; a.size_units = tas->d_size_units.p; a.size_shift = tas->size_shift;
    a.MF0 = tas->d_MF0.p; a.dMF0 = tas->d_dMF0.p; a.resident = resident;
    return launch_eval(tas, sw.ws, a, peak, argmax, min_resident);
}

#ifdef TENSILE_EVAL_PROF
extern "C" int tensile_debug_eval_prof(unsigned long long *out, int reset) {
    if (out) (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(tensile::g_eval_prof), sizeof(tensile::g_eval_prof));
    if (reset) {
        unsigned long long z[16 * 8] = {};
        (void)hipMemcpyToSymbol(HIP_SYMBOL(tensile::g_eval_prof), z, sizeof(z));
    }
    return 0;
}
#endif
