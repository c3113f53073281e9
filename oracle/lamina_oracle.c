/*
 * CPU oracle for the decode attention operator -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, obviously-correct fp64 definition that the GPU library is
 * checked against.  Nothing in the product path may link, load or call it; only the
 * tests, the smoke check and the benchmark's cpu_baseline leg do.  It shares no code,
 * header, table or helper with the HIP sources.
 *
 * What it computes (paper Sec. 2.1, the starred equation, read per head; grouped-query
 * attention as described in Sec. 2.2.2): for request r, query head h, kv head
 * g = h div G, context length n = seq_lens[r]
 *
 *     s_j  = scale * sum_c q[r][h][c] * K[r][g][j][c]        j = 0..n-1
 *     m    = max_j s_j
 *     w_j  = exp(s_j - m),   S = sum_j w_j
 *     out[r][h][c] = (sum_j w_j * V[r][g][j][c]) / S
 *     lse[r][h]    = m + ln S      ( = ln S_q(I) of Sec. 4.2.2 )
 *
 * Two passes (max first, then the sums), plain left-to-right fp64 accumulation, no
 * blocking, no online recurrence.  n == 0 gives out = 0 and lse = -inf.
 *
 * Inputs are the very bit patterns the GPU sees, widened exactly: bf16 -> fp64 by
 * placing the 16 bits in the top half of an fp32; fp8 (OCP e4m3fn) through the
 * decoder below, times the per-(request, kv head) fp32 scale widened to fp64.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- exact widening of storage formats -------------------------------------------- */

static double bf16_to_f64(uint16_t bits)
{
    uint32_t w = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/*
 * OCP 8-bit float, e4m3fn flavour: 1 sign, 4 exponent (bias 7), 3 mantissa bits.
 * No infinities; S.1111.111 is NaN; exponent field 0 is subnormal: (m/8) * 2^-6.
 * Largest finite magnitude is S.1111.110 = 1.75 * 2^8 = 448.
 */
double oracle_e4m3fn_decode(uint8_t byte)
{
    int sign = (byte >> 7) & 1;
    int expo = (byte >> 3) & 0xF;
    int mant = byte & 0x7;
    double mag;
    if (expo == 0xF && mant == 0x7)
        return NAN;
    if (expo == 0)
        mag = ldexp((double)mant / 8.0, -6);
    else
        mag = ldexp(1.0 + (double)mant / 8.0, expo - 7);
    return sign ? -mag : mag;
}

/*
 * Round-to-nearest-even quantiser onto the e4m3fn grid, saturating at +-448.
 * Used only to pin the decoder (round trips) -- the GPU path never encodes.
 * Written as an explicit search over the 127 non-negative finite codes so that it is
 * independent of any bit trickery: the nearest grid point wins, ties go to the code
 * with an even mantissa bit pattern (even code value).
 */
uint8_t oracle_e4m3fn_encode(double x)
{
    uint8_t sign = 0;
    int best = 0, code;
    double bestd;
    if (isnan(x))
        return 0x7F;
    if (x < 0.0 || (x == 0.0 && signbit(x))) {
        sign = 0x80;
        x = -x;
    }
    if (x >= 448.0)
        return (uint8_t)(sign | 0x7E);
    bestd = fabs(x - oracle_e4m3fn_decode(0));
    for (code = 1; code <= 0x7E; ++code) {
        double d = fabs(x - oracle_e4m3fn_decode((uint8_t)code));
        if (d < bestd || (d == bestd && (code & 1) == 0)) {
            bestd = d;
            best = code;
        }
    }
    return (uint8_t)(sign | best);
}

/* ---- the operator ------------------------------------------------------------------ */

typedef struct {
    int32_t num_q_heads;          /* Hq                                                   */
    int32_t num_kv_heads;         /* Hkv, divides Hq; G = Hq / Hkv                         */
    int32_t head_dim;             /* D                                                     */
    int32_t kv_is_fp8;            /* 0: K/V are bf16 bit patterns; 1: e4m3fn bytes         */
    int32_t block_size;           /* 0: contiguous strided cache; >0: paged, tokens/block  */
    int32_t block_table_stride;   /* entries per request row of block_table                */
    int64_t stride_req;           /* contiguous: elements between requests                 */
    int64_t stride_head;          /* contiguous: elements between kv heads                 */
    int64_t stride_tok;           /* contiguous: elements between tokens                   */
    int64_t pool_stride_block;    /* paged: elements between pool blocks                   */
    int64_t pool_stride_head;     /* paged: elements between kv heads inside a block       */
    double  scale;                /* softmax scale, e.g. 1/sqrt(D)                          */
} oracle_layout;

static int64_t token_offset(const oracle_layout *L, const int32_t *block_table,
                            int r, int g, int j)
{
    if (L->block_size > 0) {
        int64_t blk = block_table[(int64_t)r * L->block_table_stride + j / L->block_size];
        return blk * L->pool_stride_block + (int64_t)g * L->pool_stride_head
             + (int64_t)(j % L->block_size) * L->head_dim;
    }
    return (int64_t)r * L->stride_req + (int64_t)g * L->stride_head
         + (int64_t)j * L->stride_tok;
}

/* All 256 decoded byte values, filled once from the decoder above (a lookup is the
 * same exact value, only cheaper than ldexp per element). */
static double e4m3fn_table[256];
static int e4m3fn_table_ready = 0;

static void fill_e4m3fn_table(void)
{
    int b;
    if (e4m3fn_table_ready)
        return;
    for (b = 0; b < 256; ++b)
        e4m3fn_table[b] = oracle_e4m3fn_decode((uint8_t)b);
    e4m3fn_table_ready = 1;
}

static double kv_elem(const oracle_layout *L, const void *base, int64_t idx)
{
    if (L->kv_is_fp8)
        return e4m3fn_table[((const uint8_t *)base)[idx]];
    return bf16_to_f64(((const uint16_t *)base)[idx]);
}

/*
 * Evaluate `num_pairs` (request, query head) rows.  pairs = [r0, h0, r1, h1, ...];
 * pass NULL to mean "all R x Hq rows in order" (then num_pairs must equal R * Hq).
 * out is [num_pairs][D] fp64, lse is [num_pairs] fp64.  k_scale / v_scale are
 * [R][Hkv] fp32 (fp8 only, else NULL).  Returns 0, or -1 on a bad argument.
 */
int oracle_decode_attention(const oracle_layout *L, int32_t num_requests,
                            const uint16_t *q,          /* bf16 bits [R][Hq][D] */
                            const void *k_cache, const void *v_cache,
                            const int32_t *seq_lens, const int32_t *block_table,
                            const float *k_scale, const float *v_scale,
                            const int32_t *pairs, int64_t num_pairs,
                            double *out, double *lse)
{
    const int D = L->head_dim, Hq = L->num_q_heads, Hkv = L->num_kv_heads;
    int64_t p;
    if (D <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0)
        return -1;
    if (L->block_size > 0 && block_table == NULL)
        return -1;
    if (L->kv_is_fp8 && (k_scale == NULL || v_scale == NULL))
        return -1;
    if (pairs == NULL && num_pairs != (int64_t)num_requests * Hq)
        return -1;
    fill_e4m3fn_table();
    {
        const int G = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1)
        for (p = 0; p < num_pairs; ++p) {
            const int r = pairs ? pairs[2 * p] : (int)(p / Hq);
            const int h = pairs ? pairs[2 * p + 1] : (int)(p % Hq);
            const int g = h / G;
            const int n = seq_lens[r];
            const double ks = L->kv_is_fp8 ? (double)k_scale[(int64_t)r * Hkv + g] : 1.0;
            const double vs = L->kv_is_fp8 ? (double)v_scale[(int64_t)r * Hkv + g] : 1.0;
            const uint16_t *qrow = q + ((int64_t)r * Hq + h) * D;
            double *orow = out + p * D;
            double *s = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
            double m = -INFINITY, S = 0.0;
            int j, c;
            for (c = 0; c < D; ++c)
                orow[c] = 0.0;
            /* pass 1: scores and their maximum */
            for (j = 0; j < n; ++j) {
                const int64_t off = token_offset(L, block_table, r, g, j);
                double dot = 0.0;
                for (c = 0; c < D; ++c)
                    dot += bf16_to_f64(qrow[c]) * (kv_elem(L, k_cache, off + c) * ks);
                s[j] = L->scale * dot;
                if (s[j] > m)
                    m = s[j];
            }
            /* pass 2: weights, their sum, and the weighted sum of V rows */
            for (j = 0; j < n; ++j) {
                const int64_t off = token_offset(L, block_table, r, g, j);
                const double w = exp(s[j] - m);
                S += w;
                for (c = 0; c < D; ++c)
                    orow[c] += w * (kv_elem(L, v_cache, off + c) * vs);
            }
            if (n > 0) {
                for (c = 0; c < D; ++c)
                    orow[c] /= S;
                lse[p] = m + log(S);
            } else {
                lse[p] = -INFINITY;
            }
            free(s);
        }
    }
    return 0;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
