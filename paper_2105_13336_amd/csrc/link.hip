// Occupancy of the host link by the transfers of each plan (section IV-C of the paper, "Swap Event
// Scheduling": data transfers use the PCIe channel exclusively, so only one tensor can be on its way
// at a time; a plan respects that iff no step of its occupancy timeline exceeds one).
//
// A plan stores, for a swap of tensor i, the last resident step o and the step r at which the bytes
// are back.  The transfers are taken in their shortest form: the swap-out ends with step o and
// occupies s..o for the latest s with C[o+1] - C[s] >= x_i, the swap-in ends right before step r and
// occupies s'..r-1 for the latest s' with C[r] - C[s'] >= x_i (C = cumulative operator latency, x_i =
// transfer time; step 0 if the past is too short).  Recomputation intervals use no link.  With host
// copy reuse (section III-C: the copy in host memory stays until the tensor's last access) only the
// earliest swap-out of a tensor within a plan transfers anything.
//
// One persistent workgroup of 1024 threads per CU walks the plans slot, slot + grid, ...:
//  * the start step of a transfer is a search in C: first in a table of every stride-th value kept in
//    LDS for the whole launch (up to 7167 entries), then, when every operator latency is below 2^21 ns,
//    one 16-byte load of the block of seven values the table entry starts (see link_kernel), else
//    log2(stride) probes of C itself (L2 resident); a thread's twelve searches run in lockstep, one
//    probe each per round, so that their latencies overlap;
//  * the four endpoints of an interval (+1 at s, -1 at o+1, +1 at s', -1 at r) stay in registers, six
//    intervals per thread; a longer plan takes several passes of 6144 intervals, each over all tiles,
//    and the passes add up in the output row (or in a scratch row per workgroup when no rows are
//    wanted): occupancy is additive over the intervals;
//  * per tile of 32768 steps: scatter into a difference tile in LDS that packs two steps into one 32-bit
//    word (16-bit counters: a pass holds at most 12288 endpoints, so every count and every prefix of
//    counts fits; the adds are done on the whole word, +-1 or +-65536, and the two halves are taken apart
//    after the scatter, which is exact because sums are linear modulo 2^32), barrier; each wavefront owns
//    2048 consecutive steps of the tile as four blocks of 512: per block each lane takes one 16-byte
//    granule (8 steps), clears it for the next tile, scans locally and across the wave (DPP), blocks
//    chained through the wavefront's running total; wave totals through LDS, barrier; then per block
//    reduce (max, earliest argmax, steps occupied twice) and the row leaves through a per-wavefront
//    staging area as 16 contiguous bytes per lane.  Large tiles matter because every tile tests every
//    endpoint held in registers: the scatter of a 50,000-step row costs two rounds instead of seven;
//  * reuse: a table of the earliest swap-out step per tensor is filled before a plan's first pass and cleaned
//    after its last: in LDS (over the tile and the staging areas, idle at that point) for plans of one pass on
//    sequences of up to 25,088 tensors, else one row of N entries per workgroup in global memory, L2 atomics.
#include "common.h"
#include "wave_ops.h"

namespace tensile {

namespace {

constexpr int kThr = 1024, kWaves = kThr / 64;
constexpr int kVpt = 8;                              // steps per lane per block (one 16-byte granule of packed counters)
constexpr int kSub = 4;                              // blocks per wavefront and tile
constexpr int kBlock = 64 * kVpt;                    // 512 steps
constexpr int kWaveSteps = kSub * kBlock;            // 2048 steps per wavefront and tile
constexpr int kTile = kWaves * kWaveSteps;           // 32768
constexpr int kTileWords = kTile / 2;                // two 16-bit counters per word: 64 KB
constexpr int kR = 6;                                // intervals per thread and pass
constexpr int kPass = kR * kThr;                     // 6144 (at most 2 * kPass endpoints per step: far below 2^15)
// Coarse table of C in LDS: the descent runs over kTabBits bits, indices are clamped to the last entry,
// which always holds +inf (the host keeps the number of real entries below kTabMax).
constexpr int kTabBits = 13, kTabMax = 7168;
static_assert(kTabMax <= (1 << kTabBits) && 2 * kPass < (1 << 15), "table descent / 16-bit counters");
// The staging area is skewed by one 16-byte granule per 16 granules (cell u lives at u + 4 * (u >> 6)): both
// the lane-contiguous pattern (8 cells per lane) and the striped one (one granule per lane) are then
// free of bank conflicts.  A lane's two granules never straddle a multiple of 16.  The difference tile
// needs no skew: it is read one granule per lane, lanes side by side.
constexpr int kStageCells = kBlock + 4 * (kBlock >> 6);   // 544 per wavefront

typedef int i32x4 __attribute__((ext_vector_type(4)));

struct LinkArgs {
    int32_t T, N, B;
    int32_t reuse;
    int64_t n_intervals;
    const int64_t *plan_offsets;
    const int32_t *iv_tensor, *iv_out, *iv_in;
    const uint8_t *iv_kind;        // may be null: every interval is a swap
    const int64_t *C;              // [T+1]
    const int64_t *x;              // [N]
    int32_t tab_stride, n_tab;     // coarse table: C[k * tab_stride], k < n_tab
    int32_t fine_bits;             // probe rounds after the table: ceil(log2(tab_stride)), packed: ceil(log2(blocks_per_entry))
    const uint4 *Cpack;            // packed mode: per block of kCBlock steps the differences of its C values (see tas.hip)
    int32_t blocks_per_entry;      // packed mode: tab_stride / kCBlock
    int32_t *first_out;            // [grid][N], INT32_MAX everywhere between plans (reuse only)
    int32_t *acc_rows;             // [grid][T] scratch rows for plans of several passes when link == null
    int32_t *link;                 // [B*T] or null
    int32_t *peak, *argmax, *overbooked;   // [B]; the last two may be null
};

// inclusive add-scan over the 64 lanes (32-bit)
__device__ __forceinline__ int32_t wave_scan_add32(int32_t x) {
    x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, true);
    x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, true);
    x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, true);
    x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, true);
    x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, true);
    x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, true);
    return x;
}

// Phase timing for tuning, compiled in with -DTENSILE_LINK_PROF only: thread 0 of every workgroup adds the
// 100 MHz ticks it spent in each phase to g_link_prof.
#ifdef TENSILE_LINK_PROF
__device__ unsigned long long g_link_prof[8];
#define LINK_MARK(k)                                              \
    do {                                                          \
        if (threadIdx.x == 0) {                                   \
            const unsigned long long now_ = wall_clock64();       \
            atomicAdd(&g_link_prof[k], now_ - prof_t);            \
            prof_t = now_;                                        \
        }                                                         \
    } while (0)
#else
#define LINK_MARK(k) do { } while (0)
#endif

// kPacked: every operator latency is below 2^21 ns and the host has packed C in blocks of kLinkCBlock = 7
// steps, 16 bytes each: the six 21-bit differences between the block's values.  A search then ends with
// ONE 16-byte load (the block's first value comes from the table or from the last probe) instead of three
// dependent 8-byte probes; with the table covering every block (rows up to 50,168 steps) it is the only
// load of the search.  The searches are bound by the number of scattered loads (the texture unit takes
// one lane's cache line per cycle), not by their latency.
template <bool kPacked>
__global__ __launch_bounds__(kThr) void link_kernel(const LinkArgs a) {
    // the difference tile and the staging areas, one array: between two plans it also serves as the table of
    // the earliest swap-out step per tensor (host copy reuse) when the sequence has few enough tensors
    __shared__ __attribute__((aligned(16))) uint32_t work[kTileWords + kWaves * kStageCells];
    uint32_t *const delta = work;
    int32_t *const stage_all = reinterpret_cast<int32_t *>(work + kTileWords);
    int32_t *const first_lds = reinterpret_cast<int32_t *>(work);
    constexpr int32_t kFirstLds = kTileWords + kWaves * kStageCells;   // tensors the LDS table has room for
    __shared__ int64_t tab[kTabMax];
    __shared__ int32_t wave_tot[kWaves];
    __shared__ int32_t red_mx[kWaves], red_arg[kWaves], red_over[kWaves];

    for (int k = threadIdx.x; k < kTabMax; k += kThr) tab[k] = k < a.n_tab ? a.C[static_cast<int64_t>(k) * a.tab_stride] : INT64_MAX;
    for (int u = threadIdx.x; u < kTileWords; u += kThr) delta[u] = 0;
    __syncthreads();

    // C[k] through the uniform base and a 32-bit byte offset (the host keeps T below 2^28): no 64-bit
    // address per probe
    auto c_at = [&](uint32_t k) { return *reinterpret_cast<const int64_t *>(reinterpret_cast<const char *>(a.C) + k * 8u); };
    int32_t *first_out = a.reuse ? a.first_out + static_cast<int64_t>(blockIdx.x) * a.N : nullptr;

#ifdef TENSILE_LINK_PROF
    unsigned long long prof_t = wall_clock64();
#endif
    for (int64_t plan = blockIdx.x; plan < a.B; plan += gridDim.x) {
        LINK_MARK(0);
        // the per-lane numbers, derived afresh for every plan from a copy of the thread id that the compiler
        // cannot trace back: otherwise dozens of values computed from it are kept (and spilled) across the kernel
        int tid_now = threadIdx.x;
        asm volatile("" : "+v"(tid_now));
        const int tid = tid_now, lane = tid & 63, wave = tid >> 6;
        // (the offsets through the constant address space, i.e. the scalar unit: as a vector load they would queue
        // behind the row stores of the plan before, and the interval loads depend on them)
        typedef const int64_t __attribute__((address_space(4))) *const_i64_ptr;
        int64_t k0 = ((const_i64_ptr)a.plan_offsets)[plan], k1 = ((const_i64_ptr)a.plan_offsets)[plan + 1];
        if (k0 < 0) k0 = 0;
        if (k1 > a.n_intervals) k1 = a.n_intervals;
        if (k1 < k0) k1 = k0;
        auto swap_at = [&](int64_t k, int32_t &i, int32_t &o, int32_t &r) {   // an applicable swap interval?
            i = a.iv_tensor[k];
            o = a.iv_out[k];
            r = a.iv_in[k];
            const bool kind0 = a.iv_kind ? a.iv_kind[k] == 0 : true;
            return kind0 && static_cast<uint32_t>(i) < static_cast<uint32_t>(a.N) && o >= 0 && r <= a.T && r > o;
        };
        // Host copy reuse needs the earliest swap-out step of every tensor of the plan.  A plan of one pass on a
        // sequence of at most kFirstLds tensors collects them in LDS (below, once its intervals are in registers);
        // any other plan in a table in global memory, with L2 atomics - six times the time of the whole rest.
        const bool reuse_lds = a.reuse && a.N <= kFirstLds && k1 - k0 <= kPass;   // (block-uniform)
        if (a.reuse && !reuse_lds) {
            for (int64_t k = k0 + tid; k < k1; k += kThr) {
                int32_t i, o, r;
                if (swap_at(k, i, o, r)) atomicMin(&first_out[i], o);
            }
            __threadfence();   // the minima are in L2 before anyone reads them
            __syncthreads();
        }
        const int64_t n_pass = k1 > k0 ? (k1 - k0 + kPass - 1) / kPass : 1;
        int32_t *row = a.link ? a.link + plan * a.T : nullptr;
        // where the passes add up: the output row, else this workgroup's scratch row
        int32_t *acc = row ? row : (n_pass > 1 ? a.acc_rows + static_cast<int64_t>(blockIdx.x) * a.T : nullptr);
        int32_t best_mx = -1, best_arg = 0, over = 0;

        for (int64_t pass = 0; pass < n_pass; ++pass) {
            const bool first = pass == 0, last = pass == n_pass - 1;
            // ---- this pass's intervals: their endpoints (steps), UINT32_MAX = none.
            // Every load is issued for all kR intervals before the first is used, at clamped indices, and the
            // 2 * kR searches (start of the swap-out, start of the swap-in) advance together, one probe
            // each per round: a search alone is a chain of dependent memory latencies.
            uint32_t e[kR][4];
            int32_t lo_t = INT32_MAX, hi_t = -1;
            const int64_t kb = k0 + pass * kPass;
            int32_t iv_i[kR], iv_o[kR], iv_r[kR];
            bool ok[kR], charged[kR];
            {
                const uint32_t len = k1 - kb < kPass ? static_cast<uint32_t>(k1 - kb) : kPass;   // (>= 1 unless the plan is empty)
                uint32_t kind[kR];
#pragma unroll
                for (int j = 0; j < kR; ++j) {
                    const uint32_t k = j * kThr + tid;   // (lanes side by side: every load is two whole lines per wavefront)
                    ok[j] = k < len;
                    const int64_t kc = kb + (ok[j] ? k : 0);
                    const bool any = len > 0;
                    iv_i[j] = any ? a.iv_tensor[kc] : 0;
                    iv_o[j] = any ? a.iv_out[kc] : 0;
                    iv_r[j] = any ? a.iv_in[kc] : 0;
                    kind[j] = (any && a.iv_kind) ? a.iv_kind[kc] : 0;
                }
#pragma unroll
                for (int j = 0; j < kR; ++j) {
                    ok[j] = ok[j] && kind[j] == 0 && static_cast<uint32_t>(iv_i[j]) < static_cast<uint32_t>(a.N) && iv_o[j] >= 0 &&
                            iv_r[j] <= a.T && iv_r[j] > iv_o[j];
                    if (!ok[j]) {   // harmless stand-ins for the loads below
                        iv_i[j] = 0;
                        iv_o[j] = 0;
                        iv_r[j] = 1;
                    }
                }
            }
            if (reuse_lds) {
                // only the entries this plan touches are set up, and put back to zero afterwards: the rest of the
                // tile is zero already (the scan clears what it reads) and the staging areas may hold anything
#pragma unroll
                for (int j = 0; j < kR; ++j)
                    if (ok[j]) first_lds[iv_i[j]] = INT32_MAX;
                __syncthreads();
#pragma unroll
                for (int j = 0; j < kR; ++j)
                    if (ok[j]) atomicMin(&first_lds[iv_i[j]], iv_o[j]);
                __syncthreads();
#pragma unroll
                for (int j = 0; j < kR; ++j) charged[j] = ok[j] && first_lds[iv_i[j]] == iv_o[j];
                __syncthreads();
#pragma unroll
                for (int j = 0; j < kR; ++j)
                    if (ok[j]) first_lds[iv_i[j]] = 0;
                __syncthreads();
            }
            LINK_MARK(1);
            int64_t v[kR][2];     // C at the transfer's end minus its duration: the transfer starts inside the last step that begins at or before v
#pragma unroll
            for (int j = 0; j < kR; ++j) {
                const int64_t x = a.x[iv_i[j]];
                if (!reuse_lds) {
                    charged[j] = true;
                    if (a.reuse) charged[j] = __hip_atomic_load(&first_out[iv_i[j]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == iv_o[j];
                }
                v[j][0] = c_at(static_cast<uint32_t>(iv_o[j] + 1)) - x;
                v[j][1] = c_at(static_cast<uint32_t>(iv_r[j])) - x;
                ok[j] = ok[j] && x > 0;
            }
            LINK_MARK(2);
            // coarse: the last table entry <= v (none when v < 0: position 0, and the fine rounds then stay at step 0)
            uint32_t pos[kR][2];
#pragma unroll
            for (int j = 0; j < kR; ++j) pos[j][0] = pos[j][1] = 0;
#pragma unroll
            for (int bit = kTabBits - 1; bit >= 0; --bit) {
#pragma unroll
                for (int j = 0; j < kR; ++j) {
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        const uint32_t cand = pos[j][q] | (1u << bit);
                        pos[j][q] = tab[cand < kTabMax - 1 ? cand : kTabMax - 1] <= v[j][q] ? cand : pos[j][q];
                    }
                }
            }
            LINK_MARK(3);
            if constexpr (!kPacked) {
                // fine: from the block's first step, forward by decreasing powers of two while C stays <= v.  C increases,
                // so a probe beyond the block (or beyond the transfer's end) fails by itself; only the array's end needs a guard.
#pragma unroll
                for (int j = 0; j < kR; ++j) {
                    pos[j][0] *= a.tab_stride;
                    pos[j][1] *= a.tab_stride;
                }
                for (int bit = a.fine_bits - 1; bit >= 0; --bit) {   // (uniform)
                    int64_t c[kR][2];
#pragma unroll
                    for (int j = 0; j < kR; ++j) {
#pragma unroll
                        for (int q = 0; q < 2; ++q) {
                            const uint32_t at = pos[j][q] + (1u << bit);
                            c[j][q] = c_at(at <= static_cast<uint32_t>(a.T) ? at : static_cast<uint32_t>(a.T));
                        }
                    }
#pragma unroll
                    for (int j = 0; j < kR; ++j) {
#pragma unroll
                        for (int q = 0; q < 2; ++q) {
                            const uint32_t at = pos[j][q] + (1u << bit);
                            pos[j][q] = (at <= static_cast<uint32_t>(a.T) && c[j][q] <= v[j][q]) ? at : pos[j][q];
                        }
                    }
                }
            } else {
                // from table entries to blocks; probes of the blocks' first values when the table skips blocks
#pragma unroll
                for (int j = 0; j < kR; ++j) {
                    pos[j][0] *= a.blocks_per_entry;
                    pos[j][1] *= a.blocks_per_entry;
                }
                const uint32_t last_block = static_cast<uint32_t>(a.T) / kLinkCBlock;
                for (int bit = a.fine_bits - 1; bit >= 0; --bit) {   // (uniform; no round when the table has every block)
                    int64_t c[kR][2];
#pragma unroll
                    for (int j = 0; j < kR; ++j) {
#pragma unroll
                        for (int q = 0; q < 2; ++q) {
                            const uint32_t at = pos[j][q] + (1u << bit);
                            c[j][q] = c_at((at <= last_block ? at : last_block) * kLinkCBlock);
                        }
                    }
#pragma unroll
                    for (int j = 0; j < kR; ++j) {
#pragma unroll
                        for (int q = 0; q < 2; ++q) {
                            const uint32_t at = pos[j][q] + (1u << bit);
                            pos[j][q] = (at <= last_block && c[j][q] <= v[j][q]) ? at : pos[j][q];
                        }
                    }
                }
                // v relative to the block's first value
                if (a.blocks_per_entry == 1) {
#pragma unroll
                    for (int j = 0; j < kR; ++j) {
                        v[j][0] -= tab[pos[j][0]];
                        v[j][1] -= tab[pos[j][1]];
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < kR; ++j) {
                        v[j][0] -= c_at(pos[j][0] * kLinkCBlock);
                        v[j][1] -= c_at(pos[j][1] * kLinkCBlock);
                    }
                }
                // the block's record: how many of its further values are <= v
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    uint4 rec[kR];
#pragma unroll
                    for (int j = 0; j < kR; ++j)
                        rec[j] = *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(a.Cpack) + pos[j][q] * 16u);
#pragma unroll
                    for (int j = 0; j < kR; ++j) {
                        constexpr uint32_t kM = (1u << 21) - 1;
                        const uint4 w = rec[j];
                        const int64_t rest = v[j][q];
                        const int32_t lim = rest < 0 ? -1 : rest > INT32_MAX ? INT32_MAX : static_cast<int32_t>(rest);
                        int32_t sum = static_cast<int32_t>(w.x & kM), n = sum <= lim;
                        sum += static_cast<int32_t>(((w.x >> 21) | (w.y << 11)) & kM); n += sum <= lim;
                        sum += static_cast<int32_t>((w.y >> 10) & kM); n += sum <= lim;
                        sum += static_cast<int32_t>(((w.y >> 31) | (w.z << 1)) & kM); n += sum <= lim;
                        sum += static_cast<int32_t>(((w.z >> 20) | (w.w << 12)) & kM); n += sum <= lim;
                        sum += static_cast<int32_t>((w.w >> 9) & kM); n += sum <= lim;
                        const uint32_t at = pos[j][q] * kLinkCBlock + static_cast<uint32_t>(n);
                        pos[j][q] = at <= static_cast<uint32_t>(a.T) ? at : static_cast<uint32_t>(a.T);
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < kR; ++j) {
                e[j][0] = e[j][1] = e[j][2] = e[j][3] = UINT32_MAX;
                if (ok[j]) {
                    const int32_t s = static_cast<int32_t>(pos[j][0]), s2 = static_cast<int32_t>(pos[j][1]);
                    if (charged[j]) {
                        e[j][0] = static_cast<uint32_t>(s);
                        e[j][1] = static_cast<uint32_t>(iv_o[j] + 1);
                        lo_t = s < lo_t ? s : lo_t;
                    }
                    e[j][2] = static_cast<uint32_t>(s2);
                    e[j][3] = static_cast<uint32_t>(iv_r[j]);
                    lo_t = s2 < lo_t ? s2 : lo_t;
                    hi_t = iv_r[j] > hi_t ? iv_r[j] : hi_t;
                }
            }

            LINK_MARK(4);
            int32_t carry = 0;
            for (int32_t tile_lo = 0; tile_lo < a.T; tile_lo += kTile) {
                const int32_t tile_hi = a.T - tile_lo < kTile ? a.T : tile_lo + kTile;
                const uint32_t tile_n = static_cast<uint32_t>(tile_hi - tile_lo);
                // (per-lane addresses are derived afresh in every tile, see above: otherwise one 64-bit address per
                // block and output array is computed per plan and spilled)
                int tid_tile = tid;
                asm volatile("" : "+v"(tid_tile));
                const int lane = tid_tile & 63, wave = __builtin_amdgcn_readfirstlane(tid_tile >> 6);
                int32_t *stage = stage_all + wave * kStageCells;
                // ---- scatter (a wavefront none of whose lanes has an endpoint in range skips it)
                const bool mine = hi_t >= tile_lo && lo_t < tile_hi;
                if (__builtin_amdgcn_ballot_w64(mine) != 0) {
#pragma unroll
                    for (int j = 0; j < kR; ++j) {
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const uint32_t u = e[j][q] - static_cast<uint32_t>(tile_lo);
                            const uint32_t one = (q & 1) ? 0xffffffffu : 1u;          // -1 or +1 ...
                            if (u < tile_n) atomicAdd(&delta[u >> 1], one << (16 * (u & 1)));   // ... on the step's half
                        }
                    }
                }
                __syncthreads();
                LINK_MARK(5);
                // ---- the wavefront's four blocks: read, clear for the next tile, take the halves apart, local
                // scan, wave scan; v = sums from the wavefront's first step on
                int32_t v[kSub][kVpt];
                int32_t run = 0;   // (wave-uniform)
#pragma unroll
                for (int g = 0; g < kSub; ++g) {
                    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
                    u32x4 *cell = reinterpret_cast<u32x4 *>(&delta[wave * (kWaveSteps / 2) + g * (kBlock / 2) + 4 * lane]);
                    const u32x4 c = *cell;
                    *cell = u32x4{0, 0, 0, 0};
#pragma unroll
                    for (int h = 0; h < 4; ++h) {
                        const int32_t lo = static_cast<int16_t>(c[h] & 0xffffu);
                        v[g][2 * h] = lo;
                        v[g][2 * h + 1] = static_cast<int32_t>(c[h] - static_cast<uint32_t>(lo)) >> 16;
                    }
#pragma unroll
                    for (int j = 1; j < kVpt; ++j) v[g][j] += v[g][j - 1];
                    const int32_t incl = wave_scan_add32(v[g][kVpt - 1]);
                    const int32_t before_me = run + incl - v[g][kVpt - 1];
#pragma unroll
                    for (int j = 0; j < kVpt; ++j) v[g][j] += before_me;
                    run += __builtin_amdgcn_readlane(incl, 63);
                }
                if (lane == 0) wave_tot[wave] = run;
                __syncthreads();
                int32_t before = 0, total = 0;
#pragma unroll
                for (int w = 0; w < kWaves; ++w) {
                    const int32_t t = wave_tot[w];
                    before += w < wave ? t : 0;
                    total += t;
                }
                const int32_t base = carry + before;
                carry += total;
#pragma unroll
                for (int g = 0; g < kSub; ++g) {
                    const int32_t block_t0 = tile_lo + wave * kWaveSteps + g * kBlock;   // (wave-uniform)
                    if (block_t0 >= tile_hi) break;
                    const int32_t t0 = block_t0 + kVpt * lane;
#pragma unroll
                    for (int j = 0; j < kVpt; ++j) v[g][j] += base;
                    // ---- earlier passes of a long plan
                    if (!first) {
#pragma unroll
                        for (int j = 0; j < kVpt; ++j)
                            if (t0 + j < tile_hi) v[g][j] += __hip_atomic_load(&acc[t0 + j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                    if (!last) {
#pragma unroll
                        for (int j = 0; j < kVpt; ++j)
                            if (t0 + j < tile_hi) __hip_atomic_store(&acc[t0 + j], v[g][j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        continue;   // (block-uniform; the next pass reads these sums back in the same lanes)
                    }
                    // ---- reduce
#pragma unroll
                    for (int j = 0; j < kVpt; ++j) {
                        if (t0 + j < tile_hi) {
                            if (v[g][j] > best_mx) {
                                best_mx = v[g][j];
                                best_arg = t0 + j;
                            }
                            over += v[g][j] >= 2 ? 1 : 0;
                        }
                    }
                    // ---- the row: through the wavefront's staging area, 16 contiguous bytes per lane
                    if (row) {
                        __builtin_amdgcn_wave_barrier();
                        i32x4 *mine_out = reinterpret_cast<i32x4 *>(stage + 8 * lane + 4 * (lane >> 3));
                        mine_out[0] = i32x4{v[g][0], v[g][1], v[g][2], v[g][3]};
                        mine_out[1] = i32x4{v[g][4], v[g][5], v[g][6], v[g][7]};
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                        const bool wide = (reinterpret_cast<uintptr_t>(row + block_t0) & 15) == 0 && block_t0 + kBlock <= tile_hi;
#pragma unroll
                        for (int j = 0; j < 2; ++j) {
                            const i32x4 xv = (reinterpret_cast<const i32x4 *>(stage) + lane + (lane >> 4))[68 * j];
                            const int32_t t = block_t0 + 4 * (j * 64 + lane);
                            if (wide) {
                                *reinterpret_cast<i32x4 *>(row + t) = xv;
                            } else {
#pragma unroll
                                for (int q = 0; q < 4; ++q)
                                    if (t + q < tile_hi) row[t + q] = xv[q];
                            }
                        }
                        __builtin_amdgcn_wave_barrier();
                    }
                }
                LINK_MARK(6);
            }
        }

        LINK_MARK(6);
        // ---- the plan's result
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            const int32_t omx = __shfl_xor(best_mx, d, 64), oarg = __shfl_xor(best_arg, d, 64);
            over += __shfl_xor(over, d, 64);
            if (omx > best_mx || (omx == best_mx && oarg < best_arg)) {
                best_mx = omx;
                best_arg = oarg;
            }
        }
        if (lane == 0) {
            red_mx[wave] = best_mx;
            red_arg[wave] = best_arg;
            red_over[wave] = over;
        }
        __syncthreads();
        if (tid == 0) {
            int32_t mx = red_mx[0], arg = red_arg[0], ov = red_over[0];
            for (int w = 1; w < kWaves; ++w) {
                if (red_mx[w] > mx || (red_mx[w] == mx && red_arg[w] < arg)) {
                    mx = red_mx[w];
                    arg = red_arg[w];
                }
                ov += red_over[w];
            }
            a.peak[plan] = mx;
            if (a.argmax) a.argmax[plan] = arg;
            if (a.overbooked) a.overbooked[plan] = ov;
        }
        if (a.reuse && !reuse_lds) {   // leave the table as it was found
            for (int64_t k = k0 + tid; k < k1; k += kThr) {
                int32_t i, o, r;
                if (swap_at(k, i, o, r)) __hip_atomic_store(&first_out[i], INT32_MAX, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            __threadfence();   // ... before the next plan's minima arrive
        }
        __syncthreads();   // red_* and the table are reused by the next plan
    }
}

// Without latencies nothing is transferred in measurable time: every output is zero.
__global__ void link_zero_kernel(int64_t n_rows, int32_t *link, int32_t B, int32_t *peak, int32_t *argmax, int32_t *overbooked) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t k = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; k < n_rows; k += stride) link[k] = 0;
    for (int64_t k = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; k < B; k += stride) {
        peak[k] = 0;
        if (argmax) argmax[k] = 0;
        if (overbooked) overbooked[k] = 0;
    }
}

__global__ void link_fill_kernel(int32_t *p, int64_t n, int32_t v) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t k = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; k < n; k += stride) p[k] = v;
}

}  // namespace

int launch_link(const tensile_tas *tas, Workspace &ws, const tensile_plans *plans, bool reuse, int32_t *link, int32_t *peak,
                int32_t *argmax, int32_t *overbooked) {
    const hipStream_t stream = ws.stream;
    const int32_t B = plans->B, T = tas->T;
    if (B == 0) return TENSILE_OK;
    if (T > (1 << 28)) { set_error("eval_link: T = %d exceeds 2^28 steps", T); return TENSILE_E_RANGE; }
    if (!tas->timed || tas->N == 0) {
        const int64_t n_rows = link ? static_cast<int64_t>(B) * T : 0;
        hipLaunchKernelGGL(link_zero_kernel, dim3(tas->num_cus * 4), dim3(256), 0, stream, n_rows, link, B, peak, argmax, overbooked);
        TS_HIP(hipGetLastError());
        return TENSILE_OK;
    }
    LinkArgs a{};
    a.T = T; a.N = tas->N; a.B = B; a.reuse = reuse ? 1 : 0;
    a.n_intervals = plans->n_intervals;
    a.plan_offsets = plans->plan_offsets;
    a.iv_tensor = plans->iv_tensor; a.iv_out = plans->iv_out; a.iv_in = plans->iv_in; a.iv_kind = plans->iv_kind;
    a.C = tas->d_C.p; a.x = tas->d_x.p;
    constexpr int kTabReal = kTabMax - 1;   // the last entry stays +inf
    const bool packed = tas->c_packed && g_tuning.link_packed != 0;   // (0: testing aid, the probe search)
    a.fine_bits = 0;
    if (packed) {
        const int64_t n_blocks = static_cast<int64_t>(T) / kLinkCBlock + 1;
        a.blocks_per_entry = static_cast<int32_t>((n_blocks + kTabReal - 1) / kTabReal);
        a.tab_stride = a.blocks_per_entry * kLinkCBlock;
        a.Cpack = tas->d_Cpack.p;
        while ((1 << a.fine_bits) < a.blocks_per_entry) ++a.fine_bits;
    } else {
        a.tab_stride = static_cast<int32_t>((static_cast<int64_t>(T) + kTabReal) / kTabReal);   // ceil((T + 1) / kTabReal)
        while ((1 << a.fine_bits) < a.tab_stride) ++a.fine_bits;
    }
    a.n_tab = static_cast<int32_t>(static_cast<int64_t>(T) / a.tab_stride + 1);   // entries k with k * stride <= T: at most kTabReal
    const int32_t grid = B < tas->num_cus ? B : tas->num_cus;
    // (the table in global memory is only for plans the kernel cannot serve from LDS: see reuse_lds there)
    if (reuse && (tas->N > kTileWords + kWaves * kStageCells || plans->n_intervals > kPass)) {
        const size_t need = static_cast<size_t>(grid) * static_cast<size_t>(tas->N);
        bool fresh = false;
        const int rc = ws.provide(ws.link_first, need, "eval_link: earliest swap-out table", &fresh);
        if (rc != TENSILE_OK) return rc;
        if (fresh) {   // (the kernel leaves the table as it found it)
            hipLaunchKernelGGL(link_fill_kernel, dim3(tas->num_cus * 4), dim3(256), 0, stream, ws.link_first.p,
                               static_cast<int64_t>(ws.link_first.n), INT32_MAX);
            TS_HIP(hipGetLastError());
        }
        a.first_out = ws.link_first.p;
    }
    if (!link && plans->n_intervals > kPass) {   // some plan may need several passes
        const size_t need = static_cast<size_t>(grid) * static_cast<size_t>(T);
        const int rc = ws.provide(ws.link_acc, need, "eval_link: accumulation rows");
        if (rc != TENSILE_OK) return rc;
        a.acc_rows = ws.link_acc.p;
    }
    a.link = link; a.peak = peak; a.argmax = argmax; a.overbooked = overbooked;
    if (packed) hipLaunchKernelGGL(link_kernel<true>, dim3(grid), dim3(kThr), 0, stream, a);
    else hipLaunchKernelGGL(link_kernel<false>, dim3(grid), dim3(kThr), 0, stream, a);
    TS_HIP(hipGetLastError());
    return TENSILE_OK;
}

#ifdef TENSILE_LINK_PROF
extern "C" int tensile_debug_link_prof(unsigned long long *out, int reset) {
    if (out) (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_link_prof), sizeof(g_link_prof));
    if (reset) {
        unsigned long long z[8] = {};
        (void)hipMemcpyToSymbol(HIP_SYMBOL(g_link_prof), z, sizeof(z));
    }
    return 0;
}
#endif

}  // namespace tensile
