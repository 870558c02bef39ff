// Memory peak analysis of a batch of plans (Eq. 1, Eq. 2 and Alg. 1 of the paper)
// as one fused kernel: difference-array scatter of the interval endpoints into an
// LDS tile, prefix scan over the steps, add the unscheduled timeline, store the
// footprint row, and reduce (max, earliest argmax, min) on the way.
//
// Work decomposition.  A workgroup owns one (plan, segment): `tiles_per_seg`
// consecutive tiles of kEvalTile steps.  The running sum that enters a segment
// is the sum of the deltas before it, which the workgroup takes straight from
// the plan's intervals while it scans them for the first tile (an interval
// contributes -size if its out+1 lies before the segment and +size if its in
// step does), so segments of one plan need no communication and no look-back.
// Per tile every thread walks the plan's interval list (coalesced int32 loads,
// served by L2 after the first touch) and adds the endpoints that fall into the
// tile with 64-bit LDS atomics.  Each of the four wavefronts then owns a
// contiguous quarter of the tile: one pass sums the quarters (to get each
// wave's starting carry), one pass scans 256 steps at a time (4 per lane + a
// wave scan), adds MF0 and writes 32 contiguous bytes per lane.
//
// Workgroup ids are decoded so that all segments of a plan run on the same XCD
// (ids are dealt round-robin to the 8 XCDs, each with its own L2): the plan's
// interval list is then fetched from HBM once and re-read from that L2.
#include "common.h"

#include <cstdlib>

namespace tensile {

namespace {

constexpr int kWaves = kEvalThreads / 64;
constexpr int kQuarter = kEvalTile / kWaves;   // steps per wave per tile
constexpr int kVpt = 4;                        // steps per lane per chunk
constexpr int kChunk = 64 * kVpt;              // steps per wave per scan step
static_assert(kQuarter % kChunk == 0, "tile must split into whole chunks");

__device__ __forceinline__ int64_t wave_sum(int64_t v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// inclusive scan over the 64 lanes
__device__ __forceinline__ int64_t wave_scan_add(int64_t v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int64_t y = __shfl_up(v, d, 64);
        if (lane >= d) v += y;
    }
    return v;
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

template <bool kVec16, bool kNonTemporal>
__device__ __forceinline__ void store4(int64_t *dst, const int64_t (&v)[kVpt], int32_t n_valid) {
    if (n_valid >= kVpt) {
        if constexpr (kVec16) {
            typedef long long ll2 __attribute__((ext_vector_type(2)));
            ll2 a = {v[0], v[1]}, b = {v[2], v[3]};
            if constexpr (kNonTemporal) {
                __builtin_nontemporal_store(a, reinterpret_cast<ll2 *>(dst));
                __builtin_nontemporal_store(b, reinterpret_cast<ll2 *>(dst) + 1);
            } else {
                reinterpret_cast<ll2 *>(dst)[0] = a;
                reinterpret_cast<ll2 *>(dst)[1] = b;
            }
        } else {
#pragma unroll
            for (int j = 0; j < kVpt; ++j) {
                if constexpr (kNonTemporal) __builtin_nontemporal_store(v[j], dst + j);
                else dst[j] = v[j];
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < kVpt; ++j)
            if (j < n_valid) dst[j] = v[j];
    }
}

template <bool kVec16, bool kNonTemporal>
__global__ __launch_bounds__(kEvalThreads) void eval_kernel(const EvalArgs a) {
    __shared__ int64_t delta[kEvalTile];
    __shared__ int64_t wave_tot[kWaves];
    __shared__ int64_t carry_part[kWaves];
    __shared__ int64_t red_mx[kWaves], red_mn[kWaves];
    __shared__ int32_t red_arg[kWaves];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // XCD-aware decode: block w runs on XCD w % 8; give XCD x the plans = x (mod 8)
    const int64_t w = blockIdx.x;
    const int32_t xcd = static_cast<int32_t>(w & 7);
    const int64_t q = w >> 3;
    const int64_t plan64 = (q / a.S) * 8 + xcd;
    const int32_t seg = static_cast<int32_t>(q % a.S);
    if (plan64 >= a.B) return;
    const int32_t plan = static_cast<int32_t>(plan64);

    int64_t k0 = a.plan_offsets[plan], k1 = a.plan_offsets[plan + 1];
    if (k0 < 0) k0 = 0;
    if (k1 > a.n_intervals) k1 = a.n_intervals;
    if (k1 < k0) k1 = k0;

    const int64_t seg_len = static_cast<int64_t>(a.tiles_per_seg) * kEvalTile;
    const int64_t seg_lo64 = seg * seg_len;
    if (seg_lo64 >= a.T) return;   // cannot happen with the host's choice of S; keeps indexing safe
    const int32_t seg_lo = static_cast<int32_t>(seg_lo64);
    const int32_t seg_hi = static_cast<int32_t>(seg_lo64 + seg_len < a.T ? seg_lo64 + seg_len : a.T);

    for (int j = tid; j < kEvalTile; j += kEvalThreads) delta[j] = 0;

    int64_t carry = 0;   // running sum of the deltas before the current tile (same in every thread)
    Best best{INT64_MIN, INT64_MAX, INT32_MAX};
    int64_t *row = a.resident ? a.resident + static_cast<int64_t>(plan) * a.T : nullptr;

    for (int32_t tile_lo = seg_lo; tile_lo < seg_hi; tile_lo += kEvalTile) {
        const int32_t tile_hi = tile_lo + kEvalTile < seg_hi ? tile_lo + kEvalTile : seg_hi;
        const bool first = tile_lo == seg_lo;
        __syncthreads();   // delta is all zero here (initial fill, or re-zeroed by the scan below)

        // ---- scatter: endpoints of this plan that fall into [tile_lo, tile_hi)
        int64_t carry_local = 0;
        for (int64_t k = k0 + tid; k < k1; k += kEvalThreads) {
            const int32_t i = a.iv_tensor[k], o = a.iv_out[k], r = a.iv_in[k];
            if (static_cast<uint32_t>(i) >= static_cast<uint32_t>(a.N) || o < a.o_min || r > a.T || r <= o) continue;
            const int32_t e0 = o + 1;   // -size from here on
            const int32_t e1 = r;       // +size from here on
            const bool in0 = e0 >= tile_lo && e0 < tile_hi;
            const bool in1 = e1 >= tile_lo && e1 < tile_hi;
            const bool before0 = first && e0 < seg_lo;
            const bool before1 = first && e1 < seg_lo;
            if (in0 | in1 | before0 | before1) {
                const int64_t s = a.size[i];
                if (in0) atomicAdd(reinterpret_cast<unsigned long long *>(&delta[e0 - tile_lo]),
                                   static_cast<unsigned long long>(-s));
                if (in1) atomicAdd(reinterpret_cast<unsigned long long *>(&delta[e1 - tile_lo]),
                                   static_cast<unsigned long long>(s));
                carry_local += (before1 ? s : 0) - (before0 ? s : 0);
            }
        }
        if (first) {
            carry_local = wave_sum(carry_local);
            if (lane == 0) carry_part[wave] = carry_local;
        }
        __syncthreads();
        if (first) {
#pragma unroll
            for (int v = 0; v < kWaves; ++v) carry += carry_part[v];
        }

        // ---- each wave sums its quarter of the tile (lane-strided reads: no bank conflicts)
        const int qbase = wave * kQuarter;
        int64_t qs = 0;
#pragma unroll
        for (int j = 0; j < kQuarter / 64; ++j) qs += delta[qbase + j * 64 + lane];
        qs = wave_sum(qs);
        if (lane == 0) wave_tot[wave] = qs;
        __syncthreads();
        int64_t wave_carry = carry;
#pragma unroll
        for (int v = 0; v < kWaves; ++v) {
            const int64_t tv = wave_tot[v];
            if (v < wave) wave_carry += tv;
            carry += tv;
        }

        // ---- scan the quarter, 256 steps at a time; re-zero what was read
#pragma unroll 1
        for (int c = 0; c < kQuarter / kChunk; ++c) {
            const int base = qbase + c * kChunk + lane * kVpt;
            const int32_t t0 = tile_lo + base;
            if (tile_lo + qbase + c * kChunk >= tile_hi) break;   // wave-uniform: nothing left in this tile
            int64_t v[kVpt];
#pragma unroll
            for (int j = 0; j < kVpt; ++j) {
                v[j] = delta[base + j];
                delta[base + j] = 0;
            }
#pragma unroll
            for (int j = 1; j < kVpt; ++j) v[j] += v[j - 1];
            const int64_t incl = wave_scan_add(v[kVpt - 1], lane);
            const int64_t excl = incl - v[kVpt - 1] + wave_carry;
            wave_carry += __shfl(incl, 63, 64);
            const int32_t n_valid = t0 >= tile_hi ? 0 : (tile_hi - t0 < kVpt ? tile_hi - t0 : kVpt);
            if (n_valid > 0) {
#pragma unroll
                for (int j = 0; j < kVpt; ++j) {
                    if (j < n_valid) {
                        v[j] += excl + a.MF0[t0 + j];
                        if (v[j] > best.mx) {
                            best.mx = v[j];
                            best.arg = t0 + j;
                        }
                        if (v[j] < best.mn) best.mn = v[j];
                    }
                }
                if (row) store4<kVec16, kNonTemporal>(row + t0, v, n_valid);
            }
        }
    }

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
        for (int v = 1; v < kWaves; ++v) best_merge(best, red_mx[v], red_arg[v], red_mn[v]);
        const int64_t slot = static_cast<int64_t>(plan) * a.S + seg;
        a.out_max[slot] = best.mx;
        a.out_arg[slot] = best.arg;
        if (a.out_min) a.out_min[slot] = best.mn;
    }
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

int env_int(const char *name, int fallback) {
    const char *s = std::getenv(name);
    if (!s || !*s) return fallback;
    return std::atoi(s);
}

}  // namespace

int launch_eval(const tensile_tas *tas, const EvalArgs &proto, int64_t *peak, int32_t *argmax, int64_t *min_resident,
                hipStream_t stream) {
    EvalArgs a = proto;
    if (a.B == 0) return TENSILE_OK;
    const int64_t n_tiles = (static_cast<int64_t>(a.T) + kEvalTile - 1) / kEvalTile;
    // enough workgroups to fill the chip several times over; otherwise one segment per plan
    const int64_t want_blocks = static_cast<int64_t>(tas->num_cus) * 16;
    int64_t S = (want_blocks + a.B - 1) / a.B;
    const int forced = env_int("TENSILE_EVAL_SEGMENTS", 0);   // tuning knob
    if (forced > 0) S = forced;
    if (S < 1) S = 1;
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
        Scratch &sc = tas->scratch;
        const size_t n = static_cast<size_t>(a.B) * static_cast<size_t>(S);
        if (sc.part_max.n < n || sc.part_arg.n < n || sc.part_min.n < n) {
            TS_HIP(hipDeviceSynchronize());   // an earlier launch may still read the old buffers
            TS_HIP(sc.part_max.reserve(n));
            TS_HIP(sc.part_arg.reserve(n));
            TS_HIP(sc.part_min.reserve(n));
        }
        a.out_max = sc.part_max.p;
        a.out_arg = sc.part_arg.p;
        a.out_min = sc.part_min.p;
    }
    const bool vec16 = a.resident && (a.T % 2 == 0) && (reinterpret_cast<uintptr_t>(a.resident) % 16 == 0);
    const bool nt = env_int("TENSILE_EVAL_NT", 1) != 0;
    const dim3 grid(static_cast<uint32_t>(blocks)), block(kEvalThreads);
    if (vec16 && nt) hipLaunchKernelGGL((eval_kernel<true, true>), grid, block, 0, stream, a);
    else if (vec16) hipLaunchKernelGGL((eval_kernel<true, false>), grid, block, 0, stream, a);
    else if (nt) hipLaunchKernelGGL((eval_kernel<false, true>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((eval_kernel<false, false>), grid, block, 0, stream, a);
    TS_HIP(hipGetLastError());
    if (S > 1) {
        const int threads = 256;
        hipLaunchKernelGGL(eval_finalize_kernel, dim3((a.B + threads - 1) / threads), dim3(threads), 0, stream, a.B,
                           a.S, a.out_max, a.out_arg, a.out_min, peak, argmax, min_resident);
        TS_HIP(hipGetLastError());
    }
    return TENSILE_OK;
}

}  // namespace tensile
