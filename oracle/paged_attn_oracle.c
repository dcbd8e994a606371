/*
 * CPU oracle for paged-KV decode attention.  TEST INFRASTRUCTURE ONLY: nothing on
 * the product path may link or call this file.  It shares no code with the HIP
 * kernels.
 *
 * What it computes is the plain definition of what the paper's attention decode
 * kernel produces (Section 3.1, "Prefetch KV Blocks"; Algorithm 1 only reorders
 * memory traffic and changes no value):
 *
 *   for every sequence b and query head h, with kv head g = h / (Hq / Hkv):
 *     K_b[t,:] = k_cache[ block_tables[b][t / bs] ][g][t % bs][:]   t = 0..n_b-1
 *     V_b[t,:]   likewise from v_cache                (block-table lookup, Sec. 3.1)
 *     s[t]   = scale * sum_c q[b][h][c] * K_b[t][c]   (Q.K^T, Sec. 3.1 stage 2)
 *     p[t]   = exp(s[t] - max_t s) / sum_t exp(s[t] - max_t s)
 *     out[b][h][:] = sum_t p[t] * V_b[t][:]           (logits.V, Sec. 3.1)
 *
 * Every product and sum is taken in fp64 on the exact fp16 / bf16 input values.
 * Nothing is blocked, fused or reordered: one pass for the logits, one for the
 * maximum, one for the weights, one for the weighted sum.
 *
 * Readings where the paper is silent:
 *   - context_lens[b] counts every token attended to (the caller has already
 *     appended the new token's K/V); there is no causal mask.
 *   - query head h uses kv head h / (Hq/Hkv) (contiguous groups).
 *   - cache slots at t >= n_b and block-table entries at index >= ceil(n_b/bs)
 *     are never read.
 *   - n_b <= 0 gives an all-zero output row.
 *
 * Layouts (all dense, row-major, 16-bit elements passed as raw bits):
 *   q            [B][Hq][d]
 *   k_cache      [NBLK][Hkv][bs][d]      v_cache the same
 *   block_tables [B][MB] int32           context_lens [B] int32
 *   out          [npairs][d] fp64 (or [B][Hq][d] when pairs == NULL)
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1 };

/* IEEE binary16 bits -> double, every case spelled out (checked in the tests
 * against numpy on all 65536 bit patterns). */
double oracle_f16_to_f64(uint16_t h) {
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);             /* zero and subnormals */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp(1.0 + (double)frac / 1024.0, expo - 15);
    }
    return sign ? -v : v;
}

/* bfloat16 is the upper half of an IEEE binary32. */
double oracle_bf16_to_f64(uint16_t h) {
    uint32_t w = (uint32_t)h << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

static double widen(uint16_t bits, int dtype) {
    return dtype == ORACLE_F16 ? oracle_f16_to_f64(bits) : oracle_bf16_to_f64(bits);
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* One (b, h) pair.  probs (optional, length n_b) receives the softmax row. */
static int attend_one(const uint16_t* q, const uint16_t* k_cache, const uint16_t* v_cache,
                      const int32_t* block_tables, const int32_t* context_lens,
                      int b, int h, int Hq, int Hkv, int d, int bs, int MB, int64_t NBLK,
                      int dtype, double scale, double* out_row, double* probs) {
    int n = context_lens[b];
    for (int c = 0; c < d; ++c) out_row[c] = 0.0;
    if (n <= 0) return 0;
    int group = Hq / Hkv;
    int g = h / group;
    double* s = (double*)malloc((size_t)n * sizeof(double));
    if (!s) return -1;
    const uint16_t* qrow = q + ((size_t)b * Hq + h) * d;

    /* logits */
    for (int t = 0; t < n; ++t) {
        int64_t blk = block_tables[(size_t)b * MB + t / bs];
        if (blk < 0 || blk >= NBLK) { free(s); return -2; }
        const uint16_t* krow = k_cache + (((size_t)blk * Hkv + g) * bs + (t % bs)) * d;
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += widen(qrow[c], dtype) * widen(krow[c], dtype);
        s[t] = scale * dot;
    }
    /* softmax over the n tokens */
    double mx = s[0];
    for (int t = 1; t < n; ++t) if (s[t] > mx) mx = s[t];
    double denom = 0.0;
    for (int t = 0; t < n; ++t) { s[t] = exp(s[t] - mx); denom += s[t]; }
    for (int t = 0; t < n; ++t) s[t] /= denom;
    if (probs) memcpy(probs, s, (size_t)n * sizeof(double));
    /* weighted sum of V rows */
    for (int t = 0; t < n; ++t) {
        int64_t blk = block_tables[(size_t)b * MB + t / bs];
        const uint16_t* vrow = v_cache + (((size_t)blk * Hkv + g) * bs + (t % bs)) * d;
        for (int c = 0; c < d; ++c) out_row[c] += s[t] * widen(vrow[c], dtype);
    }
    free(s);
    return 0;
}

/*
 * pairs == NULL: all (b, h), out is [B][Hq][d].
 * pairs != NULL: npairs rows of (b, h), out is [npairs][d].
 * Returns 0, -1 (out of memory) or -2 (a needed block id outside [0, NBLK)).
 */
int oracle_paged_attention(const uint16_t* q, const uint16_t* k_cache, const uint16_t* v_cache,
                           const int32_t* block_tables, const int32_t* context_lens,
                           double* out, int B, int Hq, int Hkv, int d, int bs, int MB,
                           int64_t NBLK, int dtype, double scale,
                           const int32_t* pairs, int npairs) {
    int total = pairs ? npairs : B * Hq;
    int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < total; ++i) {
        int b = pairs ? pairs[2 * i] : i / Hq;
        int h = pairs ? pairs[2 * i + 1] : i % Hq;
        int rc = attend_one(q, k_cache, v_cache, block_tables, context_lens, b, h, Hq, Hkv, d, bs,
                            MB, NBLK, dtype, scale, out + (size_t)i * d, NULL);
        if (rc != 0) {
#pragma omp critical
            status = rc;
        }
    }
    return status;
}

/* Softmax row of one (b, h): probs has room for context_lens[b] doubles. */
int oracle_paged_attention_probs(const uint16_t* q, const uint16_t* k_cache,
                                 const uint16_t* v_cache, const int32_t* block_tables,
                                 const int32_t* context_lens, double* out_row, double* probs,
                                 int b, int h, int Hq, int Hkv, int d, int bs, int MB,
                                 int64_t NBLK, int dtype, double scale) {
    return attend_one(q, k_cache, v_cache, block_tables, context_lens, b, h, Hq, Hkv, d, bs, MB,
                      NBLK, dtype, scale, out_row, probs);
}

/* ------------------------------------------------------------------------------------------
 * 8-bit KV cache.  Not in the paper: the same operation (Section 3.1) on a cache whose K and
 * V elements are OCP FP8 E4M3 codes with one scale per tensor,
 *     K_b[t][c] = k_scale * e4m3(k_cache[...])      V_b[t][c] = v_scale * e4m3(v_cache[...]),
 * q and out staying 16-bit.  Halving the bytes per token is what changes; the definition does
 * not.  Layouts as above with one byte per cache element.
 * ------------------------------------------------------------------------------------------ */

/* OCP FP8 E4M3 ("fn": no infinities, one NaN code per sign): 1 sign, 4 exponent (bias 7),
 * 3 mantissa bits.  Checked in the tests on all 256 codes. */
double oracle_fp8e4m3_to_f64(uint8_t x) {
    int sign = (x >> 7) & 1;
    int expo = (x >> 3) & 0xf;
    int frac = x & 7;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -9);              /* zero and subnormals: frac/8 * 2^-6 */
    } else if (expo == 15 && frac == 7) {
        v = NAN;
    } else {
        v = ldexp(1.0 + (double)frac / 8.0, expo - 7);
    }
    return sign ? -v : v;
}

static int attend_one_kv8(const uint16_t* q, const uint8_t* k_cache, const uint8_t* v_cache,
                          const int32_t* block_tables, const int32_t* context_lens,
                          int b, int h, int Hq, int Hkv, int d, int bs, int MB, int64_t NBLK,
                          int qdtype, double scale, double k_scale, double v_scale, double* out_row) {
    int n = context_lens[b];
    for (int c = 0; c < d; ++c) out_row[c] = 0.0;
    if (n <= 0) return 0;
    int g = h / (Hq / Hkv);
    double* s = (double*)malloc((size_t)n * sizeof(double));
    if (!s) return -1;
    const uint16_t* qrow = q + ((size_t)b * Hq + h) * d;
    for (int t = 0; t < n; ++t) {
        int64_t blk = block_tables[(size_t)b * MB + t / bs];
        if (blk < 0 || blk >= NBLK) { free(s); return -2; }
        const uint8_t* krow = k_cache + (((size_t)blk * Hkv + g) * bs + (t % bs)) * d;
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += widen(qrow[c], qdtype) * (k_scale * oracle_fp8e4m3_to_f64(krow[c]));
        s[t] = scale * dot;
    }
    double mx = s[0];
    for (int t = 1; t < n; ++t) if (s[t] > mx) mx = s[t];
    double denom = 0.0;
    for (int t = 0; t < n; ++t) { s[t] = exp(s[t] - mx); denom += s[t]; }
    for (int t = 0; t < n; ++t) s[t] /= denom;
    for (int t = 0; t < n; ++t) {
        int64_t blk = block_tables[(size_t)b * MB + t / bs];
        const uint8_t* vrow = v_cache + (((size_t)blk * Hkv + g) * bs + (t % bs)) * d;
        for (int c = 0; c < d; ++c) out_row[c] += s[t] * (v_scale * oracle_fp8e4m3_to_f64(vrow[c]));
    }
    free(s);
    return 0;
}

/* As oracle_paged_attention, for an FP8 E4M3 cache; qdtype is the type of q. */
int oracle_paged_attention_kv8(const uint16_t* q, const uint8_t* k_cache, const uint8_t* v_cache,
                               const int32_t* block_tables, const int32_t* context_lens,
                               double* out, int B, int Hq, int Hkv, int d, int bs, int MB,
                               int64_t NBLK, int qdtype, double scale, double k_scale, double v_scale,
                               const int32_t* pairs, int npairs) {
    int total = pairs ? npairs : B * Hq;
    int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < total; ++i) {
        int b = pairs ? pairs[2 * i] : i / Hq;
        int h = pairs ? pairs[2 * i + 1] : i % Hq;
        int rc = attend_one_kv8(q, k_cache, v_cache, block_tables, context_lens, b, h, Hq, Hkv, d, bs,
                                MB, NBLK, qdtype, scale, k_scale, v_scale, out + (size_t)i * d);
        if (rc != 0) {
#pragma omp critical
            status = rc;
        }
    }
    return status;
}
