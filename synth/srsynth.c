/*
 * Seeded synthetic inputs for the selective-rollout decode path.
 *
 * This file holds only input generation (random token ids, random weight
 * tensors, random action tables).  It contains none of the method's
 * arithmetic: no edit distance, no gate rule, no decoder maths.  Both the CPU
 * checker and the GPU library consume the arrays it writes.
 *
 * Generator: SplitMix64 (Steele, Lea & Flood 2014) used as a counter-based
 * generator.  Stream `key` yields r_i = finalize(key + (i+1)*GOLDEN), which is
 * the i-th output of SplitMix64 seeded with `key`; any element can be drawn
 * independently of the others.  A stream key is derived from (seed, stream id)
 * by two further finalizer rounds.
 *
 * Normal variates are drawn by table lookup: the top 16 bits of r_i index a
 * 65536-entry table of N(0, sigma) quantiles already rounded to bf16 (the
 * table is built by the Python side in fp64).  This keeps every
 * implementation of the generator (this file, and the device fill kernel
 * that mirrors it) bit-identical, with no transcendental function in the
 * loop.
 */
#include <stdint.h>
#include <stddef.h>

#define SRS_GOLDEN 0x9E3779B97F4A7C15ULL

static inline uint64_t srs_finalize(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

uint64_t srs_stream_key(uint64_t seed, uint64_t stream) {
    return srs_finalize(srs_finalize(seed + SRS_GOLDEN) ^ (stream * 0xD1342543DE82EF95ULL + 1ULL));
}

uint64_t srs_draw(uint64_t key, uint64_t i) {
    return srs_finalize(key + (i + 1ULL) * SRS_GOLDEN);
}

/* dst[i] = table[top 16 bits of draw(key, first + i)],  i in [0, n) */
void srs_fill_table16(uint16_t *dst, size_t n, uint64_t seed, uint64_t stream,
                      uint64_t first, const uint16_t *table) {
    const uint64_t key = srs_stream_key(seed, stream);
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i)
        dst[i] = table[srs_draw(key, first + i) >> 48];
}

/* dst[i] = uniform id in [0, modulus) by multiply-shift of the top 32 bits */
void srs_fill_ids(int32_t *dst, size_t n, uint64_t seed, uint64_t stream,
                  uint32_t modulus) {
    const uint64_t key = srs_stream_key(seed, stream);
    for (size_t i = 0; i < n; ++i)
        dst[i] = (int32_t)(((srs_draw(key, i) >> 32) * (uint64_t)modulus) >> 32);
}

/*
 * Action tables for the gate-only workload: n_groups x G x len int32 over
 * `alphabet` symbols.  Per group a latent leader sequence is uniform; every
 * member copies the leader's symbol with probability p, else draws a uniform
 * symbol; p is picked per group, uniformly, from p_q16[0..n_p) (probabilities
 * in units of 1/65536; 65536 means "always copy").  p_index[g] receives the
 * index picked.
 */
void srs_gate_actions(int32_t *dst, int n_groups, int G, int len, int alphabet,
                      const uint32_t *p_q16, int n_p, uint64_t seed,
                      int32_t *p_index) {
#pragma omp parallel for schedule(static)
    for (int g = 0; g < n_groups; ++g) {
        const uint64_t key = srs_stream_key(seed, 0x6A7E000000000000ULL + (uint64_t)g);
        const int pi = (int)(((srs_draw(key, 0) >> 32) * (uint64_t)n_p) >> 32);
        const uint32_t p = p_q16[pi];
        if (p_index) p_index[g] = pi;
        for (int t = 0; t < len; ++t) {
            const int32_t lead =
                (int32_t)(((srs_draw(key, 1 + (uint64_t)t) >> 32) * (uint64_t)alphabet) >> 32);
            for (int m = 0; m < G; ++m) {
                const uint64_t r = srs_draw(key, 1 + (uint64_t)len + ((uint64_t)m * len + t));
                const uint32_t u = (uint32_t)(r >> 48);               /* 16-bit uniform */
                const int32_t own = (int32_t)((((r >> 8) & 0xFFFFFFFFULL) * (uint64_t)alphabet) >> 32);
                dst[((size_t)g * G + m) * len + t] = (u < p) ? lead : own;
            }
        }
    }
}
