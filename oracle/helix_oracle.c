/*
 * CPU oracle for Helix Parallelism's attention phase (Sec. 2.1.1 "KV partitioning (KVP)", Fig. 4 top).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is a plain, slow, fp64 statement of what the
 * GPU path must compute.  It shares no code, header, table or helper with the HIP library and only
 * tests, the smoke check and the bench's cpu_baseline leg may call it.
 *
 * The paper gives the attention phase in prose only: every KVP rank runs exact softmax attention of
 * the decode query against its own KV-sequence shard and emits a partial output plus one
 * log-sum-exp scalar per (token, head); the ranks' fragments are then rescaled and summed into the
 * exact softmax-normalised attention of the unsharded cache (Sec. 2.1.1; Fig. 4 caption; Sec. 2.2).
 * The oracle is therefore the textbook definition written out:
 *
 *     s_t  = scale * sum_d q[d] * k_t[d]                    (every token t the query may see)
 *     m    = max_t s_t ,  l = sum_t exp(s_t - m)
 *     o[j] = ( sum_t exp(s_t - m) * v_t[j] ) / l ,  lse = m + ln l
 *
 * two passes over the tokens, no tiling, no running rescale, no shards.  GQA: query head h reads KV
 * head h / (Q/K) (Sec. 1: Q query heads share K KV heads).  MLA: one latent row serves as the key
 * (all dk entries) and as the value (its first dv entries) for all query heads (Sec. 1, Sec. 3).
 *
 * Pins (tests/test_oracle_pins.py): brute force against a high-precision evaluator, shard-split
 * identity, constant V, equal keys, single token, zero query, duplicated cache, key shift, GQA/MLA
 * structure, the e4m3 / e2m1 / e8m0 code tables against the format definitions, MXFP4 input against the
 * same values given as bf16, the combine's closed forms, and a float64 library softmax.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_KV_BF16 0
#define ORACLE_KV_FP8_E4M3 1
#define ORACLE_KV_MXFP4 2

/* bfloat16: the upper 16 bits of an IEEE binary32. */
static double bf16_value(uint16_t bits)
{
    uint32_t w = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* OCP 8-bit float E4M3 ("fn" flavour): 1 sign, 4 exponent (bias 7), 3 mantissa bits; no infinity;
 * exponent 15 with mantissa 7 is NaN; exponent 0 is subnormal: m/8 * 2^-6; largest finite is 448. */
double helix_oracle_e4m3_value(uint8_t code)
{
    int sign = code >> 7;
    int e = (code >> 3) & 0xF;
    int m = code & 0x7;
    double mag;
    if (e == 0xF && m == 0x7)
        return NAN;
    if (e == 0)
        mag = ldexp((double)m / 8.0, -6);
    else
        mag = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -mag : mag;
}

/* OCP microscaling FP4 element E2M1: 1 sign, 2 exponent (bias 1), 1 mantissa bit; no infinity, no
 * NaN; exponent 0 is subnormal: m/2 * 2^0.  The magnitudes are 0, 0.5, 1, 1.5, 2, 3, 4, 6. */
double helix_oracle_e2m1_value(uint8_t code)
{
    int sign = (code >> 3) & 1;
    int e = (code >> 1) & 0x3;
    int m = code & 0x1;
    double mag = e == 0 ? (double)m / 2.0 : ldexp(1.0 + (double)m / 2.0, e - 1);
    return sign ? -mag : mag;
}

/* OCP microscaling shared scale E8M0: an unsigned power of two 2^(code - 127); code 255 is NaN. */
double helix_oracle_e8m0_value(uint8_t code)
{
    if (code == 0xFF)
        return NAN;
    return ldexp(1.0, (int)code - 127);
}

typedef struct {
    int32_t B, Q, K, dk, dv;
    int32_t v_aliases_k;      /* 1: value row = first dv entries of the key row (MLA latent) */
    int32_t kv_dtype;         /* ORACLE_KV_* */
    double scale;             /* softmax scale, multiplies q.k */
    const uint16_t *q;        /* bf16 bits, [B,Q,dk] contiguous */
    const void *k, *v;        /* element (b,kh,t,d) at index b*sb + kh*sh + (tok_off[b]+t)*st + d */
    int64_t k_sb, k_sh, k_st;
    int64_t v_sb, v_sh, v_st;
    const float *kv_scale;    /* fp8 only: per-token factor at b*s_sb + kh*s_sh + (tok_off[b]+t) */
    int64_t s_sb, s_sh;
    const int64_t *tok_off;   /* [B] first token row of sequence b, or NULL for 0 */
    const int32_t *len;       /* [B] number of tokens sequence b attends to */
    /* MXFP4 only (the FP4 of the paper's evaluation, Sec. 3: microscaling formats): k / v hold E2M1
     * codes, two per byte, element index idx in the low (idx even) or high (idx odd) nibble of byte
     * idx/2; every 32 consecutive elements of a row share the E8M0 scale at index idx/32 of
     * k_mx / v_mx (strides are multiples of 32 elements) */
    const uint8_t *k_mx, *v_mx;
} oracle_problem;

static double kv_elem(const oracle_problem *p, const void *base, const uint8_t *mx, int64_t idx)
{
    if (p->kv_dtype == ORACLE_KV_BF16)
        return bf16_value(((const uint16_t *)base)[idx]);
    if (p->kv_dtype == ORACLE_KV_MXFP4) {
        uint8_t byte = ((const uint8_t *)base)[idx / 2];
        uint8_t code = (idx & 1) ? (uint8_t)(byte >> 4) : (uint8_t)(byte & 0xF);
        return helix_oracle_e8m0_value(mx[idx / 32]) * helix_oracle_e2m1_value(code);
    }
    return helix_oracle_e4m3_value(((const uint8_t *)base)[idx]);
}

/* One (b,h) row of the definition.  t_lo/t_hi restrict the tokens (a shard); o has dv entries.
 * An empty token set has no softmax: o = 0, lse = -inf. */
static void attend_row(const oracle_problem *p, int b, int h, int64_t t_lo, int64_t t_hi,
                       double *o, double *lse, int inner_parallel)
{
    const int g = p->Q / p->K;
    const int kh = h / g;
    const int64_t n = t_hi - t_lo;
    const int64_t row0 = (p->tok_off ? p->tok_off[b] : 0) + t_lo;
    const uint16_t *qrow = p->q + ((int64_t)b * p->Q + h) * p->dk;
    const int dk = p->dk, dv = p->dv;

    for (int j = 0; j < dv; j++)
        o[j] = 0.0;
    if (n <= 0) {
        *lse = -INFINITY;
        return;
    }
    /* threads over the tokens of one row only pay off (and only reorder the sums) on long rows */
    inner_parallel = inner_parallel && n >= 32768;
    double *s = (double *)malloc((size_t)n * sizeof(double));
    double *qd = (double *)malloc((size_t)dk * sizeof(double));
    for (int d = 0; d < dk; d++)
        qd[d] = bf16_value(qrow[d]);

    /* pass 1: scores and their maximum */
    double m = -INFINITY;
#pragma omp parallel for reduction(max : m) if (inner_parallel)
    for (int64_t t = 0; t < n; t++) {
        int64_t kidx = (int64_t)b * p->k_sb + (int64_t)kh * p->k_sh + (row0 + t) * p->k_st;
        double dot = 0.0;
        for (int d = 0; d < dk; d++)
            dot += qd[d] * kv_elem(p, p->k, p->k_mx, kidx + d);
        if (p->kv_dtype == ORACLE_KV_FP8_E4M3)
            dot *= (double)p->kv_scale[(int64_t)b * p->s_sb + (int64_t)kh * p->s_sh + row0 + t];
        s[t] = p->scale * dot;
        if (s[t] > m)
            m = s[t];
    }

    /* pass 2: normaliser and weighted value sum */
    double l = 0.0;
#pragma omp parallel for reduction(+ : l) reduction(+ : o[:dv]) if (inner_parallel)
    for (int64_t t = 0; t < n; t++) {
        double w = exp(s[t] - m);
        const void *vbase = p->v_aliases_k ? p->k : p->v;
        const uint8_t *vmx = p->v_aliases_k ? p->k_mx : p->v_mx;
        int64_t vidx = p->v_aliases_k
                           ? (int64_t)b * p->k_sb + (int64_t)kh * p->k_sh + (row0 + t) * p->k_st
                           : (int64_t)b * p->v_sb + (int64_t)kh * p->v_sh + (row0 + t) * p->v_st;
        double f = 1.0;
        if (p->kv_dtype == ORACLE_KV_FP8_E4M3)
            f = (double)p->kv_scale[(int64_t)b * p->s_sb + (int64_t)kh * p->s_sh + row0 + t];
        l += w;
        for (int j = 0; j < dv; j++)
            o[j] += w * (f * kv_elem(p, vbase, vmx, vidx + j));
    }
    for (int j = 0; j < dv; j++)
        o[j] /= l;
    *lse = m + log(l);
    free(s);
    free(qd);
}

/*
 * Attention of the query against tokens [t_lo[b], t_hi[b]) of every sequence (t_lo/t_hi NULL: all
 * len[b] tokens, i.e. the unsharded cache).  With n_rows > 0 only the listed (rows_b[i], rows_h[i])
 * pairs are evaluated and o is [n_rows,dv], lse [n_rows]; otherwise o is [B,Q,dv], lse [B,Q].
 * Returns 0, or -1 on arguments that make no sense.
 */
int helix_oracle_attention(const oracle_problem *p, const int64_t *t_lo, const int64_t *t_hi,
                           int32_t n_rows, const int32_t *rows_b, const int32_t *rows_h,
                           double *o, double *lse)
{
    if (!p || !p->q || !p->k || !p->len || !o || !lse)
        return -1;
    if (p->K <= 0 || p->Q % p->K != 0 || (p->v_aliases_k && p->dv > p->dk))
        return -1;
    if (!p->v_aliases_k && !p->v)
        return -1;
    if (p->kv_dtype == ORACLE_KV_FP8_E4M3 && !p->kv_scale)
        return -1;
    if (p->kv_dtype == ORACLE_KV_MXFP4) {
        if (!p->k_mx || (!p->v_aliases_k && !p->v_mx))
            return -1;
        if (p->k_sb % 32 || p->k_sh % 32 || p->k_st % 32 || p->v_sb % 32 || p->v_sh % 32 || p->v_st % 32)
            return -1;
    }
    const int64_t total = n_rows > 0 ? n_rows : (int64_t)p->B * p->Q;
    int nth = 1;
#ifdef _OPENMP
    nth = omp_get_max_threads();
#endif
    /* few rows and many tokens: spread the tokens of one row over the threads instead */
    const int inner = total < nth;
#pragma omp parallel for schedule(dynamic, 1) if (!inner)
    for (int64_t r = 0; r < total; r++) {
        int b = n_rows > 0 ? rows_b[r] : (int)(r / p->Q);
        int h = n_rows > 0 ? rows_h[r] : (int)(r % p->Q);
        int64_t lo = t_lo ? t_lo[b] : 0;
        int64_t hi = t_hi ? t_hi[b] : p->len[b];
        attend_row(p, b, h, lo, hi, o + r * p->dv, lse + r, inner);
    }
    return 0;
}

/*
 * Combine of N shard partials (Sec. 2.1.1: every rank rescales the received fragments and adds them up):
 *     lse* = max_i lse_i ; w_i = exp(lse_i - lse*) ; O = sum_i w_i O_i / sum_i w_i ;
 *     LSE = lse* + ln sum_i w_i .
 * It follows from exp(lse_i) = sum over shard i of exp(s_t): the shard's share of the global
 * normaliser.  A shard with lse = -inf (no tokens) has weight zero; if all are empty O = 0,
 * LSE = -inf.  o_parts [N,R,dv], lse_parts [N,R] -> o [R,dv], lse [R].
 */
int helix_oracle_combine(int32_t N, int64_t R, int32_t dv, const double *o_parts,
                         const double *lse_parts, double *o, double *lse)
{
    if (N < 1 || !o_parts || !lse_parts || !o || !lse)
        return -1;
    for (int64_t r = 0; r < R; r++) {
        double top = -INFINITY;
        for (int i = 0; i < N; i++)
            if (lse_parts[(int64_t)i * R + r] > top)
                top = lse_parts[(int64_t)i * R + r];
        for (int j = 0; j < dv; j++)
            o[r * dv + j] = 0.0;
        if (top == -INFINITY) {
            lse[r] = -INFINITY;
            continue;
        }
        double wsum = 0.0;
        for (int i = 0; i < N; i++) {
            double li = lse_parts[(int64_t)i * R + r];
            if (li == -INFINITY)
                continue;
            double w = exp(li - top);
            wsum += w;
            for (int j = 0; j < dv; j++)
                o[r * dv + j] += w * o_parts[((int64_t)i * R + r) * dv + j];
        }
        for (int j = 0; j < dv; j++)
            o[r * dv + j] /= wsum;
        lse[r] = top + log(wsum);
    }
    return 0;
}

/* Index of the shard holding the largest stored fp32 LSE (lowest index on ties; 0 if all -inf).
 * The decision is taken on the fp32 values exactly as the GPU stored them. */
int helix_oracle_argmax_f32(int32_t N, int64_t R, const float *lse_parts, int32_t *argmax)
{
    if (N < 1 || !lse_parts || !argmax)
        return -1;
    for (int64_t r = 0; r < R; r++) {
        int best = 0;
        for (int i = 1; i < N; i++)
            if (lse_parts[(int64_t)i * R + r] > lse_parts[(int64_t)best * R + r])
                best = i;
        argmax[r] = best;
    }
    return 0;
}

int helix_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
