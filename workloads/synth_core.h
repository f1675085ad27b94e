/*
 * Counter-based synthetic gradient rows -- INPUT GENERATOR ONLY (no balancing,
 * no reordering, no gradient formula lives here).
 *
 * One header, compiled twice: by gcc into the host library and by hipcc into the
 * gfx950 kernel.  Every element is a pure function of (seed, row, element), and
 * the arithmetic uses only integer operations and correctly rounded fp32
 * add / multiply / divide / sqrt with contraction disabled, so the host and the
 * GPU produce the same bits.
 *
 * Row model (the streaming workloads of this build):
 *     g[row][e] = block_scale[e / block_len] * (mu[e] + row_scale[row] * T)
 * with T ~ Student-t(3), optionally forced to exactly 0 with probability
 * zero_threshold / 65536 (a per-row, per-element Bernoulli mask).  mu, row_scale
 * and block_scale are small seeded tables drawn on the host with numpy and
 * handed in as plain arrays.
 *
 * Student-t(3) is drawn with the polar method for t variates (Bailey 1994):
 * (u, v) uniform on the unit disc, w = u^2 + v^2, T = u * sqrt(nu (w^(-2/nu) - 1) / w).
 * w^(-1/3) comes from an integer first guess refined by three Newton steps
 * y <- y (4 - w y^3) / 3, which needs multiplications only.
 */
#ifndef CDGRAB_SYNTH_CORE_H
#define CDGRAB_SYNTH_CORE_H

#include <stdint.h>
#include <string.h>

#ifdef __HIPCC__
#define SYN_FN __host__ __device__ __forceinline__
#else
#define SYN_FN static inline
#endif

typedef struct synth_params {
    uint64_t seed;
    int64_t m, n, d;           /* workers, rows per worker, elements per row           */
    const float *mu;           /* [d] shared mean                                      */
    const float *row_scale;    /* [m*n] per-row noise scale, row id = worker*n + j     */
    const float *block_scale;  /* [n_block_scales] or NULL                             */
    int64_t block_len;         /* elements per scale block (ceil(d / n_block_scales))  */
    int32_t n_block_scales;    /* 0: no block scaling                                  */
    uint32_t zero_threshold;   /* element is 0 when a 16-bit draw < this (0: never)    */
} synth_params;

/* 64-bit mixing function of this generator: xor-shift / odd-multiply rounds with
 * constants drawn for it. */
SYN_FN uint64_t syn_mix(uint64_t x) {
    x ^= x >> 31;
    x *= 0xa6dd34c6341e636bULL;
    x ^= x >> 29;
    x *= 0xcfa72ea4d22ea969ULL;
    x ^= x >> 32;
    x *= 0xae2de0081eb3edf1ULL;
    x ^= x >> 30;
    return x;
}

/* One 64-bit word for (seed, row, element, draw): the counter packs row (24 bits),
 * element (32 bits) and draw (8 bits) without collisions. */
SYN_FN uint64_t syn_word(uint64_t seed_mixed, uint64_t row, uint64_t elem, uint32_t draw) {
    uint64_t ctr = (row << 40) | (elem << 8) | (uint64_t)draw;
    return syn_mix(ctr ^ seed_mixed);
}

SYN_FN float syn_bits_to_float(uint32_t b) {
    float f;
    memcpy(&f, &b, sizeof f);
    return f;
}
SYN_FN uint32_t syn_float_to_bits(float f) {
    uint32_t b;
    memcpy(&b, &f, sizeof b);
    return b;
}

/* 24 bits -> odd multiple of 2^-24 in (-1, 1): symmetric about 0 and never 0. */
SYN_FN float syn_uniform_pm1(uint32_t bits24) {
    int32_t k = (int32_t)bits24 - (1 << 23);
    return (float)(2 * k + 1) * 5.9604644775390625e-08f; /* 2^-24, exact */
}

/* w^(-1/3) for w in (0, 1]. */
SYN_FN float syn_inv_cbrt(float w) {
    uint32_t i = 0x54a2fa8cu - syn_float_to_bits(w) / 3u;
    float y = syn_bits_to_float(i);
    for (int it = 0; it < 3; ++it) {
        float y2 = y * y;
        float y3 = y2 * y;
        float wy3 = w * y3;
        float corr = 1.3333334f - 0.33333334f * wy3;
        y = y * corr;
    }
    return y;
}

/* Student-t(3) variate for (row, element); also returns the 16 mask bits. */
SYN_FN float syn_student_t3(uint64_t seed_mixed, uint64_t row, uint64_t elem, uint32_t *mask_bits) {
    /* rejection loop: only the draw and the disc test, so that lanes of a wavefront
     * that accept at different draws do not repeat the transform below */
    float u = 0.0f, w = 2.0f;
    *mask_bits = 0;
    for (uint32_t draw = 0; draw < 64; ++draw) {
        uint64_t x = syn_word(seed_mixed, row, elem, draw);
        if (draw == 0) *mask_bits = (uint32_t)(x & 0xffffu);
        float uc = syn_uniform_pm1((uint32_t)(x >> 40));
        float vc = syn_uniform_pm1((uint32_t)(x >> 16) & 0xffffffu);
        float uu = uc * uc;
        float vv = vc * vc;
        float wc = uu + vv;
        if (wc <= 1.0f) {
            u = uc;
            w = wc;
            break;
        }
    }
    if (w > 1.0f) return 0.0f;  /* 64 rejections in a row: probability 1e-43 */
    float y = syn_inv_cbrt(w);
    float c = y * y;            /* w^(-2/3) */
    float num = 3.0f * (c - 1.0f);
    if (num < 0.0f) num = 0.0f; /* rounding when w is 1 */
    float q = num / w;
    return u * __builtin_sqrtf(q);
}

/* Element e of a row; `block` = e / block_len (ignored without block scales). */
SYN_FN float syn_element_in_block(const synth_params *p, uint64_t seed_mixed, int64_t row, int64_t e,
                                  int64_t block) {
    uint32_t mask_bits;
    float t = syn_student_t3(seed_mixed, (uint64_t)row, (uint64_t)e, &mask_bits);
    if (mask_bits < p->zero_threshold) return 0.0f;
    float noise = p->row_scale[row] * t;
    float v = p->mu[e] + noise;
    if (p->n_block_scales > 0) v = v * p->block_scale[block];
    return v;
}

SYN_FN float syn_element(const synth_params *p, uint64_t seed_mixed, int64_t row, int64_t e) {
    return syn_element_in_block(p, seed_mixed, row, e, p->n_block_scales > 0 ? e / p->block_len : 0);
}

SYN_FN uint64_t syn_seed_mixed(uint64_t seed) { return syn_mix(seed ^ 0x5bd1e9955bd1e995ULL) | 1ULL; }

/* Row id of (flattened pair p, which) : worker p % m, visiting position 2 (p / m) + which. */
SYN_FN int64_t syn_row_of_pair(const synth_params *p, int64_t pair, int which) {
    int64_t k = pair / p->m;
    int64_t i = pair - k * p->m;
    return i * p->n + 2 * k + which;
}

#endif /* CDGRAB_SYNTH_CORE_H */
