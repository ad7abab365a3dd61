/*
 * coopt_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, float64 CPU statement of what the paged FP8 grouped-query
 * decode-attention path computes.  Only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may call it.  It shares no source, header,
 * table or helper with the HIP library and is written to be checked against the
 * paper by eye: no blocking, no fusion, no online softmax.
 *
 * What follows what:
 *   - cache write with the negative-slot skip rule ........ Opt-KV, Eq. 5, Alg. 1 phase 1
 *   - dequantise-before-attention ......................... Opt-KV, Eq. 6, Alg. 1 phase 2
 *   - query head -> KV head map  g(h) = floor(h / (H_q/H_k)) Opt-GQA, Eq. 7, Alg. 2 phase 1
 *   - softmax(q K^T / sqrt(d)) V over the tokens j < t ..... Background Eq. 1; Alg. 2 phase 2
 *   - only blocks b < ceil(t/B) are touched ................ Opt-Pa, Eq. 9, Alg. 3 phase 1
 *   - max-subtracted softmax weights ....................... Opt-Pa, Eq. 10
 *   - partition-wise partial results and their merge ....... Conclusion ("partitioned parallel"),
 *                                                            formalised here as the exact
 *                                                            log-sum-exp merge
 *
 * The paper says only "FP8".  The format used here is OCP E4M3 (1-4-3, bias 7,
 * no infinities, S.1111.111 = NaN, max finite 448) with one binary32 scale per
 * (token, KV head): scale = amax/448, round to nearest even, saturate at +-448.
 * The two divisions of the write path are done in binary32 so that the cache
 * bytes and the scales are *defined* bit for bit; everything else is float64.
 *
 * The alternatives that reading stands against are here too, for comparison on
 * the same cache layout (orc_kv_cache_write_fp8_scaled): OCP E5M2 codes (1-5-2,
 * bias 15, max finite 57344, S.11111.00 = infinity, other S.11111.xx = NaN),
 * and a scale that is not the row's own: one per cache block (the largest absmax
 * among the call's rows that land in the block) or a static one per KV head.
 * kv_dtype: 0 = fp16 cache, 1 = E4M3 codes, 2 = E5M2 codes.
 *
 * Tensor layouts (the oracle owns one index function per tensor):
 *   k, v (new tokens) ... [T, H_k, d]        fp16 bit patterns
 *   k_cache ............. [NB*H_k tiles][d/E][B][E]            E = elements per 16 bytes
 *   v_cache ............. [NB*H_k tiles][d/(4E)][B/4][16][E/4][4]   (see idx_kcache / idx_vcache)
 *   k_scale, v_scale .... [NB, H_k, B]       binary32
 *   block_tables ........ [S, max_blocks]    int32, logical block -> physical block
 *   q, out .............. [S, H_q, d]
 *
 * Parity status: every function in this file is pinned by tests/test_oracle_*.py
 * (closed forms, brute force on tiny inputs, invariants, library cross-checks).
 * The paper prints no worked example for this path, so no pin is a paper value.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ formats */

/* IEEE binary16 bit pattern -> exact double. */
double orc_f16_to_f64(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);                 /* subnormal: m * 2^-10 * 2^-14 */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)m / 1024.0, e - 15);
    return sign ? -v : v;
}

/* OCP E4M3 code -> exact double.  exponent field 0: (m/8)*2^-6; else (1+m/8)*2^(e-7). */
double orc_e4m3_to_f64(uint8_t c)
{
    int sign = (c >> 7) & 1;
    int e = (c >> 3) & 0xf;
    int m = c & 7;
    double v;
    if (e == 15 && m == 7)
        return NAN;
    if (e == 0)
        v = ldexp((double)m / 8.0, -6);
    else
        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

/*
 * binary32 -> OCP E4M3, round to nearest, ties to even mantissa, saturating at
 * +-448.  The sign bit is kept (so -0 -> 0x80).  NaN -> 0x7F.
 */
uint8_t orc_f32_to_e4m3(float y)
{
    uint8_t sign = signbit(y) ? 0x80 : 0x00;
    double a = fabs((double)y);
    if (isnan(y))
        return 0x7f;
    if (a >= 448.0)
        return sign | 0x7e;
    if (a < ldexp(1.0, -6)) {
        /* subnormal grid, spacing 2^-9; rint() is ties-to-even in the default mode.
           A result of 8 is the code 0x08 = 2^-6, the first normal, as it should be. */
        int r = (int)rint(ldexp(a, 9));
        return sign | (uint8_t)r;
    }
    int ex;
    double fr = frexp(a, &ex);      /* a = fr * 2^ex, fr in [0.5,1) */
    double mant = fr * 2.0;         /* in [1,2) */
    int e = ex - 1;
    int r = (int)rint((mant - 1.0) * 8.0);   /* 0..8, ties to even r */
    if (r == 8) {
        r = 0;
        e += 1;
    }
    int field = e + 7;
    if (field > 15 || (field == 15 && r == 7))
        return sign | 0x7e;         /* cannot happen for a < 448, kept for safety */
    return sign | (uint8_t)((field << 3) | r);
}

void orc_f32_to_e4m3_array(const float *y, uint8_t *out, size_t n)
{
    for (size_t i = 0; i < n; i++)
        out[i] = orc_f32_to_e4m3(y[i]);
}

/* OCP E5M2 code -> double.  exponent field 0: (m/4)*2^-14; 31: infinity (m = 0) or NaN;
 * else (1+m/4)*2^(e-15). */
double orc_e5m2_to_f64(uint8_t c)
{
    int sign = (c >> 7) & 1;
    int e = (c >> 2) & 0x1f;
    int m = c & 3;
    double v;
    if (e == 31)
        v = m ? NAN : INFINITY;
    else if (e == 0)
        v = ldexp((double)m / 4.0, -14);
    else
        v = ldexp(1.0 + (double)m / 4.0, e - 15);
    return sign ? -v : v;
}

/*
 * binary32 -> OCP E5M2, round to nearest, ties to even mantissa, saturating at
 * +-57344 (never an infinity).  The sign bit is kept.  NaN -> 0x7F.
 */
uint8_t orc_f32_to_e5m2(float y)
{
    uint8_t sign = signbit(y) ? 0x80 : 0x00;
    double a = fabs((double)y);
    if (isnan(y))
        return 0x7f;
    if (a >= 57344.0)
        return sign | 0x7b;
    if (a < ldexp(1.0, -14)) {
        /* subnormal grid, spacing 2^-16; a result of 4 is the code 0x04 = 2^-14, the first normal */
        int r = (int)rint(ldexp(a, 16));
        return sign | (uint8_t)r;
    }
    int ex;
    double fr = frexp(a, &ex);      /* a = fr * 2^ex, fr in [0.5,1) */
    double mant = fr * 2.0;         /* in [1,2) */
    int e = ex - 1;
    int r = (int)rint((mant - 1.0) * 4.0);   /* 0..4, ties to even r */
    if (r == 4) {
        r = 0;
        e += 1;
    }
    int field = e + 15;
    if (field >= 31)
        return sign | 0x7b;         /* cannot happen for a < 57344, kept for safety */
    return sign | (uint8_t)((field << 2) | r);
}

void orc_f32_to_e5m2_array(const float *y, uint8_t *out, size_t n)
{
    for (size_t i = 0; i < n; i++)
        out[i] = orc_f32_to_e5m2(y[i]);
}

/* Largest finite value of a one-byte code, and its decode / encode, by kv_dtype (1 or 2). */
static float code_max(int kv_dtype)
{
    return kv_dtype == 2 ? 57344.0f : 448.0f;
}
static double code_to_f64(uint8_t c, int kv_dtype)
{
    return kv_dtype == 2 ? orc_e5m2_to_f64(c) : orc_e4m3_to_f64(c);
}
static uint8_t f32_to_code(float y, int kv_dtype)
{
    return kv_dtype == 2 ? orc_f32_to_e5m2(y) : orc_f32_to_e4m3(y);
}

/* ------------------------------------------------------------ index functions */

/* E = elements per 16 bytes: 16 for one-byte codes, 8 for fp16.
 * K tile [d/E][B][E]: the 16-byte chunks of a token's row, chunk-major. */
static size_t idx_kcache(int blk, int head, int off, int dim, int H_k, int B, int d, int E)
{
    size_t tile = (size_t)blk * H_k + head;
    return tile * (size_t)(B * d) + (size_t)(((dim / E) * B + off) * E + dim % E);
}
/* V tile [d/(4E)][B/4][16][E/4][4]: tokens innermost in runs of 4, then W = E/4 groups of 16 dims. */
static size_t idx_vcache(int blk, int head, int off, int dim, int H_k, int B, int d, int E)
{
    size_t tile = (size_t)blk * H_k + head;
    int W = E / 4, c = dim / 16, n = dim % 16;
    int inner = ((((c / W) * (B / 4) + off / 4) * 16 + n) * W + c % W) * 4 + off % 4;
    return tile * (size_t)(B * d) + (size_t)inner;
}
static size_t idx_scale(int blk, int head, int off, int H_k, int B)
{
    return ((size_t)blk * H_k + head) * B + off;
}

/* ------------------------------------------------------------------- write */

/* Absmax of one row (fp16 is exact in binary32). */
static float row_absmax(const uint16_t *x16, int d)
{
    float amax = 0.0f;
    for (int i = 0; i < d; i++) {
        float a = fabsf((float)orc_f16_to_f64(x16[i]));
        if (a > amax)
            amax = a;
    }
    return amax;
}

/* The scale that maps absmax amax to the code's largest value; an all-zero row gets 1. */
static float scale_of_absmax(float amax, int kv_dtype)
{
    return (amax == 0.0f) ? 1.0f : amax / code_max(kv_dtype);      /* binary32 division */
}

/* One row (one token, one KV head, K or V) under a given scale: the codes. */
static void quantise_row_scaled(const uint16_t *x16, int d, float scale, int kv_dtype, uint8_t *codes)
{
    float cmax = code_max(kv_dtype);
    for (int i = 0; i < d; i++) {
        float x = (float)orc_f16_to_f64(x16[i]);
        float y = x / scale;                                   /* binary32 division */
        if (y > cmax)
            y = cmax;
        if (y < -cmax)
            y = -cmax;
        codes[i] = f32_to_code(y, kv_dtype);
    }
}

/* One row with its own (dynamic) scale = absmax / 448: scale and E4M3 codes. */
static void quantise_row(const uint16_t *x16, int d, float *scale_out, uint8_t *codes)
{
    float scale = scale_of_absmax(row_absmax(x16, d), 1);
    quantise_row_scaled(x16, d, scale, 1, codes);
    *scale_out = scale;
}

/* Membership of token index i in the SkipSet of Eq. 5, given as a bitmap over the call's token
 * indices (bit i%32 of word i/32); a NULL bitmap is the empty set. */
static int in_skip_set(const uint32_t *skip_set, int i)
{
    return skip_set != NULL && ((skip_set[i >> 5] >> (i & 31)) & 1u);
}

/* Opt-KV Alg. 1 phase 1 with the E4M3 store: tokens in order; a token is left out if its index
 * is in the SkipSet (Eq. 5) or its slot is negative. */
void orc_kv_cache_write_fp8(const uint16_t *k, const uint16_t *v, const int64_t *slot_mapping,
                            const uint32_t *skip_set, int T, uint8_t *k_cache, uint8_t *v_cache,
                            float *k_scale, float *v_scale, int H_k, int d, int B)
{
    uint8_t *codes = (uint8_t *)malloc((size_t)d);
    for (int i = 0; i < T; i++) {
        int64_t slot = slot_mapping[i];
        if (slot < 0 || in_skip_set(skip_set, i))
            continue;
        int blk = (int)(slot / B);
        int off = (int)(slot % B);
        for (int h = 0; h < H_k; h++) {
            const uint16_t *krow = k + ((size_t)i * H_k + h) * d;
            const uint16_t *vrow = v + ((size_t)i * H_k + h) * d;
            float s;
            quantise_row(krow, d, &s, codes);
            k_scale[idx_scale(blk, h, off, H_k, B)] = s;
            for (int x = 0; x < d; x++)
                k_cache[idx_kcache(blk, h, off, x, H_k, B, d, 16)] = codes[x];
            quantise_row(vrow, d, &s, codes);
            v_scale[idx_scale(blk, h, off, H_k, B)] = s;
            for (int x = 0; x < d; x++)
                v_cache[idx_vcache(blk, h, off, x, H_k, B, d, 16)] = codes[x];
        }
    }
    free(codes);
}

/*
 * The same write under another code and another scale rule (the schemes the dynamic per-token
 * E4M3 scale stands against).  kv_dtype 1 = E4M3, 2 = E5M2.  scale_mode:
 *   0  every row's own scale, absmax / max code (with kv_dtype 1 this is orc_kv_cache_write_fp8);
 *   1  one scale per (cache block, KV head) for the rows of THIS call: the largest absmax among
 *      the call's written tokens whose slot lies in the block, / max code;
 *   2  static: k_static[h] / v_static[h], whatever the rows hold (larger values saturate).
 * The scale arrays keep one entry per (token, head) in every mode.
 */
void orc_kv_cache_write_fp8_scaled(const uint16_t *k, const uint16_t *v, const int64_t *slot_mapping,
                                   const uint32_t *skip_set, int T, uint8_t *k_cache,
                                   uint8_t *v_cache, float *k_scale, float *v_scale, int H_k, int d,
                                   int B, int kv_dtype, int scale_mode, const float *k_static,
                                   const float *v_static)
{
    uint8_t *codes = (uint8_t *)malloc((size_t)d);
    for (int i = 0; i < T; i++) {
        int64_t slot = slot_mapping[i];
        if (slot < 0 || in_skip_set(skip_set, i))
            continue;
        int blk = (int)(slot / B);
        int off = (int)(slot % B);
        for (int h = 0; h < H_k; h++) {
            const uint16_t *krow = k + ((size_t)i * H_k + h) * d;
            const uint16_t *vrow = v + ((size_t)i * H_k + h) * d;
            float ks, vs;
            if (scale_mode == 2) {
                ks = k_static[h];
                vs = v_static[h];
            } else {
                float ka = row_absmax(krow, d), va = row_absmax(vrow, d);
                if (scale_mode == 1)
                    for (int i2 = 0; i2 < T; i2++) {           /* the call's other rows of this block */
                        int64_t s2 = slot_mapping[i2];
                        if (s2 < 0 || in_skip_set(skip_set, i2) || s2 / B != blk)
                            continue;
                        float a = row_absmax(k + ((size_t)i2 * H_k + h) * d, d);
                        if (a > ka)
                            ka = a;
                        a = row_absmax(v + ((size_t)i2 * H_k + h) * d, d);
                        if (a > va)
                            va = a;
                    }
                ks = scale_of_absmax(ka, kv_dtype);
                vs = scale_of_absmax(va, kv_dtype);
            }
            quantise_row_scaled(krow, d, ks, kv_dtype, codes);
            k_scale[idx_scale(blk, h, off, H_k, B)] = ks;
            for (int x = 0; x < d; x++)
                k_cache[idx_kcache(blk, h, off, x, H_k, B, d, 16)] = codes[x];
            quantise_row_scaled(vrow, d, vs, kv_dtype, codes);
            v_scale[idx_scale(blk, h, off, H_k, B)] = vs;
            for (int x = 0; x < d; x++)
                v_cache[idx_vcache(blk, h, off, x, H_k, B, d, 16)] = codes[x];
        }
    }
    free(codes);
}

/* Same scatter with the fp16 pattern stored unchanged (the unquantised comparison case). */
void orc_kv_cache_write_fp16(const uint16_t *k, const uint16_t *v, const int64_t *slot_mapping,
                             const uint32_t *skip_set, int T, uint16_t *k_cache, uint16_t *v_cache,
                             int H_k, int d, int B)
{
    for (int i = 0; i < T; i++) {
        int64_t slot = slot_mapping[i];
        if (slot < 0 || in_skip_set(skip_set, i))
            continue;
        int blk = (int)(slot / B);
        int off = (int)(slot % B);
        for (int h = 0; h < H_k; h++)
            for (int x = 0; x < d; x++) {
                k_cache[idx_kcache(blk, h, off, x, H_k, B, d, 8)] = k[((size_t)i * H_k + h) * d + x];
                v_cache[idx_vcache(blk, h, off, x, H_k, B, d, 8)] = v[((size_t)i * H_k + h) * d + x];
            }
    }
}

/* ------------------------------------------------------------- cache reads */

/* Dequantised key element of logical token j of sequence s (Eq. 6, Eq. 9).
 * kv_dtype 0 = fp16 cache, 1 = E4M3 codes, 2 = E5M2 codes (both with scales). */
static double load_k(const void *k_cache, const float *k_scale, const int32_t *bt_row, int j,
                     int g, int x, int H_k, int d, int B, int kv_dtype)
{
    int pb = bt_row[j / B];
    int off = j % B;
    if (kv_dtype != 0)
        return code_to_f64(((const uint8_t *)k_cache)[idx_kcache(pb, g, off, x, H_k, B, d, 16)], kv_dtype) *
               (double)k_scale[idx_scale(pb, g, off, H_k, B)];
    return orc_f16_to_f64(((const uint16_t *)k_cache)[idx_kcache(pb, g, off, x, H_k, B, d, 8)]);
}
static double load_v(const void *v_cache, const float *v_scale, const int32_t *bt_row, int j,
                     int g, int x, int H_k, int d, int B, int kv_dtype)
{
    int pb = bt_row[j / B];
    int off = j % B;
    if (kv_dtype != 0)
        return code_to_f64(((const uint8_t *)v_cache)[idx_vcache(pb, g, off, x, H_k, B, d, 16)], kv_dtype) *
               (double)v_scale[idx_scale(pb, g, off, H_k, B)];
    return orc_f16_to_f64(((const uint16_t *)v_cache)[idx_vcache(pb, g, off, x, H_k, B, d, 8)]);
}

/*
 * Attention of one query row over logical tokens [j0, j1) of one sequence:
 *   z_j = softmax_scale * sum_x q_x k~_{j,x};  M = max z;  l = sum exp(z-M);
 *   o = sum exp(z_j-M) v~_j / l.
 * Returns M and l through pointers (used by the partitioned form).  j0 == j1 gives zeros.
 */
static void attend_range(const uint16_t *q_row, const void *k_cache, const void *v_cache,
                         const float *k_scale, const float *v_scale, const int32_t *bt_row,
                         int j0, int j1, int g, int H_k, int d, int B, int kv_dtype,
                         double softmax_scale, double *o, double *M_out, double *l_out)
{
    int n = j1 - j0;
    for (int x = 0; x < d; x++)
        o[x] = 0.0;
    if (n <= 0) {
        *M_out = -INFINITY;
        *l_out = 0.0;
        return;
    }
    double *z = (double *)malloc(sizeof(double) * (size_t)n);
    double M = -INFINITY;
    for (int j = j0; j < j1; j++) {
        double dot = 0.0;
        for (int x = 0; x < d; x++)
            dot += orc_f16_to_f64(q_row[x]) *
                   load_k(k_cache, k_scale, bt_row, j, g, x, H_k, d, B, kv_dtype);
        z[j - j0] = softmax_scale * dot;
        if (z[j - j0] > M)
            M = z[j - j0];
    }
    double l = 0.0;
    for (int j = 0; j < n; j++) {
        z[j] = exp(z[j] - M);
        l += z[j];
    }
    for (int j = j0; j < j1; j++) {
        double p = z[j - j0] / l;
        for (int x = 0; x < d; x++)
            o[x] += p * load_v(v_cache, v_scale, bt_row, j, g, x, H_k, d, B, kv_dtype);
    }
    free(z);
    *M_out = M;
    *l_out = l;
}

/* ------------------------------------------------------------------ decode */

/* out [S, H_q, d] float64.  context_lens[s] == 0 gives a zero row. */
void orc_paged_gqa_decode(const uint16_t *q, const void *k_cache, const void *v_cache,
                          const float *k_scale, const float *v_scale,
                          const int32_t *block_tables, const int32_t *context_lens, double *out,
                          int S, int H_q, int H_k, int d, int B, int max_blocks, int kv_dtype,
                          double softmax_scale)
{
    int H_g = H_q / H_k;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int s = 0; s < S; s++)
        for (int h = 0; h < H_q; h++) {
            int g = h / H_g;
            double M, l;
            attend_range(q + ((size_t)s * H_q + h) * d, k_cache, v_cache, k_scale, v_scale,
                         block_tables + (size_t)s * max_blocks, 0, context_lens[s], g, H_k, d, B,
                         kv_dtype, softmax_scale, out + ((size_t)s * H_q + h) * d, &M, &l);
        }
}

/*
 * Partition p of sequence s covers tokens [p*P, min((p+1)*P, t_s)).
 * tmp_out [S, H_q, max_parts, d] holds the normalised partial o_p, max_logits / exp_sums
 * [S, H_q, max_parts] hold m_p and l_p = sum exp(z - m_p).  Unused partitions are left untouched.
 */
void orc_paged_gqa_decode_partitioned(const uint16_t *q, const void *k_cache, const void *v_cache,
                                      const float *k_scale, const float *v_scale,
                                      const int32_t *block_tables, const int32_t *context_lens,
                                      int P, int max_parts, double *tmp_out, double *max_logits,
                                      double *exp_sums, int S, int H_q, int H_k, int d, int B,
                                      int max_blocks, int kv_dtype, double softmax_scale)
{
    int H_g = H_q / H_k;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int s = 0; s < S; s++)
        for (int h = 0; h < H_q; h++) {
            int t = context_lens[s];
            int nparts = (t + P - 1) / P;
            for (int p = 0; p < nparts && p < max_parts; p++) {
                int j0 = p * P;
                int j1 = (p + 1) * P < t ? (p + 1) * P : t;
                size_t row = ((size_t)s * H_q + h) * max_parts + p;
                attend_range(q + ((size_t)s * H_q + h) * d, k_cache, v_cache, k_scale, v_scale,
                             block_tables + (size_t)s * max_blocks, j0, j1, h / H_g, H_k, d, B,
                             kv_dtype, softmax_scale, tmp_out + row * d, max_logits + row,
                             exp_sums + row);
            }
        }
}

/* M = max_p m_p; w_p = l_p exp(m_p - M); out = sum_p w_p o_p / sum_p w_p. */
void orc_paged_gqa_reduce(const double *tmp_out, const double *max_logits, const double *exp_sums,
                          const int32_t *context_lens, int P, int max_parts, double *out, int S,
                          int H_q, int d)
{
    for (int s = 0; s < S; s++)
        for (int h = 0; h < H_q; h++) {
            int t = context_lens[s];
            int nparts = (t + P - 1) / P;
            if (nparts > max_parts)
                nparts = max_parts;
            double *o = out + ((size_t)s * H_q + h) * d;
            for (int x = 0; x < d; x++)
                o[x] = 0.0;
            if (nparts == 0)
                continue;
            size_t row0 = ((size_t)s * H_q + h) * max_parts;
            double M = -INFINITY;
            for (int p = 0; p < nparts; p++)
                if (max_logits[row0 + p] > M)
                    M = max_logits[row0 + p];
            double W = 0.0;
            for (int p = 0; p < nparts; p++)
                W += exp_sums[row0 + p] * exp(max_logits[row0 + p] - M);
            for (int p = 0; p < nparts; p++) {
                double w = exp_sums[row0 + p] * exp(max_logits[row0 + p] - M) / W;
                for (int x = 0; x < d; x++)
                    o[x] += w * tmp_out[(row0 + p) * d + x];
            }
        }
}

/* ---------------------------------------------------------- chunked prefill */

/*
 * Causal attention of new-chunk query rows over the paged cache, which already holds the
 * chunk's own K/V.  Sequence s owns query rows query_start[s] .. query_start[s+1]-1; with
 * C_s = that count and t_s = context_lens[s] (chunk included), local row i sees tokens
 * j < t_s - C_s + i + 1.
 *
 * rows == NULL: all rows are computed, out is [query_start[S], H_q, d].
 * rows != NULL: only the n_rows listed global row numbers, out is [n_rows, H_q, d].
 */
void orc_paged_gqa_prefill_chunk(const uint16_t *q, const void *k_cache, const void *v_cache,
                                 const float *k_scale, const float *v_scale,
                                 const int32_t *block_tables, const int32_t *context_lens,
                                 const int32_t *query_start, const int32_t *rows, int n_rows,
                                 double *out, int S, int H_q, int H_k, int d, int B,
                                 int max_blocks, int kv_dtype, double softmax_scale)
{
    int H_g = H_q / H_k;
    int total = rows ? n_rows : query_start[S];
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int r = 0; r < total; r++)
        for (int h = 0; h < H_q; h++) {
            int row = rows ? rows[r] : r;
            int s = 0;
            while (!(query_start[s] <= row && row < query_start[s + 1]))
                s++;
            int C = query_start[s + 1] - query_start[s];
            int i = row - query_start[s];
            int visible = context_lens[s] - C + i + 1;
            double M, l;
            attend_range(q + ((size_t)row * H_q + h) * d, k_cache, v_cache, k_scale, v_scale,
                         block_tables + (size_t)s * max_blocks, 0, visible, h / H_g, H_k, d, B,
                         kv_dtype, softmax_scale, out + ((size_t)r * H_q + h) * d, &M, &l);
        }
}

/* ------------------------------------------------- dequantising gather (Eq. 6) */

/*
 * Contiguous dequantised K and V of logical tokens [j0, j1) of sequence s:
 * k_out, v_out [j1-j0, H_k, d] float64.  This is the paper's gather step on its own.
 */
void orc_gather_cached_kv(const void *k_cache, const void *v_cache, const float *k_scale,
                          const float *v_scale, const int32_t *block_tables, int s, int j0,
                          int j1, double *k_out, double *v_out, int H_k, int d, int B,
                          int max_blocks, int kv_dtype)
{
    const int32_t *bt_row = block_tables + (size_t)s * max_blocks;
    for (int j = j0; j < j1; j++)
        for (int g = 0; g < H_k; g++)
            for (int x = 0; x < d; x++) {
                size_t o = (((size_t)(j - j0)) * H_k + g) * d + x;
                k_out[o] = load_k(k_cache, k_scale, bt_row, j, g, x, H_k, d, B, kv_dtype);
                v_out[o] = load_v(v_cache, v_scale, bt_row, j, g, x, H_k, d, B, kv_dtype);
            }
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
