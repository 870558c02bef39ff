/* Random candidate plans for a tensor access sequence.
 *
 * For every plan b and every tensor i that has at least one gap of two or more
 * steps between consecutive touch points (allocation, accesses), the tensor is
 * swapped with probability p; the gap is uniform among the tensor's eligible
 * gaps (p_g, p_{g+1}), the last resident step o is uniform in [p_g, p_{g+1}-2]
 * and the step r at which the bytes are back is uniform in [o+2, p_{g+1}].
 *
 * Every draw is a pure function of (seed, stream, b*N+i): the mixer below is
 * the same one as in prng.py (SplitMix64's finaliser).  This file only lays
 * out inputs; it holds none of the method's arithmetic.
 */
#include <stdint.h>
#include <stddef.h>

static inline uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}
#define GOLDEN 0x9E3779B97F4A7C15ULL
static inline uint64_t make_key(uint64_t seed, uint64_t stream) {
    uint64_t k = mix64(seed + GOLDEN) ^ (stream * 0xD1B54A32D192ED03ULL);
    return mix64(k + GOLDEN);
}
static inline uint64_t draw(uint64_t key, uint64_t index) { return mix64(key + (index + 1) * GOLDEN); }

/* exported for the cross-check against prng.py */
uint64_t plangen_u64(uint64_t seed, uint64_t stream, uint64_t index) { return draw(make_key(seed, stream), index); }

/* counts[b] = number of intervals of plan b0+b; thr53 = floor(p * 2^53) */
void plangen_count(uint64_t seed, int64_t b0, int64_t nb, int64_t N, const int64_t *elig_offsets,
                   uint64_t thr53, int64_t *counts) {
    const uint64_t k_sel = make_key(seed, 1);
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < nb; ++b) {
        int64_t c = 0;
        const uint64_t base = (uint64_t)(b0 + b) * (uint64_t)N;
        for (int64_t i = 0; i < N; ++i) {
            if (elig_offsets[i + 1] == elig_offsets[i]) continue;
            if ((draw(k_sel, base + (uint64_t)i) >> 11) < thr53) ++c;
        }
        counts[b] = c;
    }
}

/* plan_offsets[nb+1] are offsets relative to the output arrays of this chunk */
void plangen_fill(uint64_t seed, int64_t b0, int64_t nb, int64_t N, const int64_t *elig_offsets,
                  const int32_t *elig_p, const int32_t *elig_q, uint64_t thr53, const int64_t *plan_offsets,
                  int32_t *iv_tensor, int32_t *iv_out, int32_t *iv_in, uint8_t *iv_kind) {
    const uint64_t k_sel = make_key(seed, 1), k_gap = make_key(seed, 2), k_out = make_key(seed, 3),
                   k_in = make_key(seed, 4);
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < nb; ++b) {
        int64_t w = plan_offsets[b];
        const uint64_t base = (uint64_t)(b0 + b) * (uint64_t)N;
        for (int64_t i = 0; i < N; ++i) {
            const int64_t e0 = elig_offsets[i], ne = elig_offsets[i + 1] - e0;
            if (ne == 0) continue;
            const uint64_t idx = base + (uint64_t)i;
            if ((draw(k_sel, idx) >> 11) >= thr53) continue;
            const int64_t g = e0 + (int64_t)(draw(k_gap, idx) % (uint64_t)ne);
            const int64_t p = elig_p[g], q = elig_q[g];
            const int64_t o = p + (int64_t)(draw(k_out, idx) % (uint64_t)(q - 2 - p + 1));
            const int64_t r = o + 2 + (int64_t)(draw(k_in, idx) % (uint64_t)(q - (o + 2) + 1));
            iv_tensor[w] = (int32_t)i;
            iv_out[w] = (int32_t)o;
            iv_in[w] = (int32_t)r;
            iv_kind[w] = 0;
            ++w;
        }
    }
}
