/*
 * CPU oracle for sparse MLA decode attention over the OmniAttn retained set.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP library is checked against.  It shares no code with that library, is
 * never used to produce a product result, and is loaded only by the tests, by
 * the smoke check and by the benchmark's CPU-baseline leg.
 *
 * What it computes, for every sequence b and head h (paper section 3.2.1):
 *
 *   retained set   M_b = {1..N_sink} u {M - N_recent + 1 .. M}   (second
 *                  equation of 3.2.1), here 0-based over the L_b cached tokens
 *                  of sequence b:  j is kept iff 0 <= j < L_b and
 *                  (j < S or j >= L_b - W).  It is a set: a position inside
 *                  both ranges counts once.
 *   output         softmax(q K_M^T * scale) V_M   (left-hand side of the first
 *                  equation of 3.2.1), one query row per (b, h).
 *
 * The paper names MLA only as a compatible architecture; the MLA reading used
 * here is the absorbed decode form: every cached token is one latent row of
 * 576 numbers, the key is the whole row, the value is its first 512 numbers,
 * and the query already carries the key up-projection.  `scale` is supplied by
 * the caller.  lse = ln sum_j exp(scale * q.k_j) over the retained j; an empty
 * retained set gives out = 0 and lse = -inf.
 *
 * All arithmetic is IEEE double.  Stored inputs (bf16 queries, bf16 or OCP
 * e4m3 cache bytes, fp32 per-token scales) are widened exactly.  There is no
 * blocking and no online softmax: logits are materialised, then max, then
 * sum, then the weighted sum, in that order.
 *
 * Pinned by tests/test_oracle_*.py: dense reduction against a library
 * softmax, brute force over explicit index lists, closed forms, invariants,
 * a hand-computed worked example, decoder tables.  The paper's accuracy claim
 * (sparse ~ dense on a trained model) needs weights and suites that are not
 * available: parity unpinned for that claim only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define QK_DIM 576
#define V_DIM 512
#define PAGE 128

enum { ORACLE_KV_BF16 = 0, ORACLE_KV_FP8_E4M3 = 1 };

/* bf16 is the upper half of an IEEE binary32. */
double oracle_bf16_to_double(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* OCP 8-bit float E4M3: 1 sign, 4 exponent (bias 7), 3 mantissa bits; no
 * infinities; S.1111.111 is NaN; exponent 0 is subnormal (m/8 * 2^-6). */
double oracle_fp8_e4m3_to_double(uint8_t bits)
{
    int sign = bits >> 7;
    int e = (bits >> 3) & 0xF;
    int m = bits & 0x7;
    double v;
    if (e == 0xF && m == 0x7)
        return NAN;
    if (e == 0)
        v = ldexp((double)m / 8.0, -6);
    else
        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

/* Is logical position j of a sequence of length L retained? */
int oracle_is_retained(int64_t j, int64_t L, int64_t S, int64_t W)
{
    if (j < 0 || j >= L)
        return 0;
    return (j < S) || (j >= L - W);
}

/*
 * Compute out/lse for n_pairs (b, h) pairs.  pairs == NULL means every pair
 * of the B x H grid in row-major order (then n_pairs must equal B*H).
 *
 * Several queries per sequence (the first equation of section 3.2.1 has a
 * query matrix of K rows): q_len >= 1 consecutive tokens, the last q_len of
 * the sequence, each attend causally.  The H rows of a sequence are then
 * q_len groups of H / q_len heads, group t belonging to the query at position
 * L - q_len + t, which sees the keys 0 .. L - q_len + t, i.e. a sequence of
 * length L - (q_len - 1 - t) to which the retained-set rule is applied as is.
 *
 *   q          bf16 bits  [B, H, 576]
 *   cache      bf16 bits or e4m3 bytes [num_pages, 128, 576]
 *   scales     fp32 [num_pages, 128], used only for e4m3
 *   page_table int32 [B, max_pages]: logical page i of sequence b
 *   out        double [n_pairs, 512];  lse  double [n_pairs]
 *   probs      optional double [n_pairs, max_L]: softmax weight of logical
 *              position j (0 where not retained); NULL to skip
 *
 * Returns 0, or -1 on bad arguments / allocation failure, or -2 when a
 * retained position maps to a page id outside [0, num_pages).
 */
int omniattn_oracle(int32_t B, int32_t H, const uint16_t *q, const void *cache,
                    int32_t kv_dtype, const float *scales, int64_t num_pages,
                    const int32_t *page_table, int32_t max_pages,
                    const int32_t *seq_lens, int32_t S, int32_t W, double scale,
                    const int32_t *pairs, int64_t n_pairs, double *out,
                    double *lse, double *probs, int64_t max_L, int32_t q_len)
{
    if (B < 0 || H < 0 || S < 0 || W < 0 || !out || !lse)
        return -1;
    if (q_len < 1 || H % q_len != 0)
        return -1;
    if (!pairs && n_pairs != (int64_t)B * H)
        return -1;
    if (kv_dtype != ORACLE_KV_BF16 && kv_dtype != ORACLE_KV_FP8_E4M3)
        return -1;
    int status = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n_pairs; ++i) {
        int32_t b = pairs ? pairs[2 * i] : (int32_t)(i / H);
        int32_t h = pairs ? pairs[2 * i + 1] : (int32_t)(i % H);
        int64_t L_seq = seq_lens[b];
        int32_t Hq = H / q_len;                /* heads per query */
        int32_t t = h / Hq;                    /* which of the q_len queries this row is */
        int64_t L = L_seq - (q_len - 1 - t);   /* the keys this query sees: 0 .. L-1 */
        if (L < 0)
            L = 0;
        double *o = out + i * V_DIM;
        for (int c = 0; c < V_DIM; ++c)
            o[c] = 0.0;
        if (probs)
            for (int64_t j = 0; j < max_L; ++j)
                probs[i * max_L + j] = 0.0;

        double qd[QK_DIM];
        for (int d = 0; d < QK_DIM; ++d)
            qd[d] = oracle_bf16_to_double(q[((int64_t)b * H + h) * QK_DIM + d]);

        /* retained positions, one by one */
        int64_t n = 0;
        for (int64_t j = 0; j < L; ++j)
            n += oracle_is_retained(j, L, S, W);
        if (n == 0) {
            lse[i] = -INFINITY;
            continue;
        }
        int64_t *idx = (int64_t *)malloc((size_t)n * sizeof *idx);
        double *s = (double *)malloc((size_t)n * sizeof *s);
        double *kv = (double *)malloc((size_t)n * QK_DIM * sizeof *kv);
        if (!idx || !s || !kv) {
            {
#pragma omp atomic write
                status = -1;
            }
            free(idx); free(s); free(kv);
            continue;
        }
        n = 0;
        for (int64_t j = 0; j < L; ++j)
            if (oracle_is_retained(j, L, S, W))
                idx[n++] = j;

        /* gather through the page table and widen */
        int bad = 0;
        for (int64_t t = 0; t < n; ++t) {
            int64_t j = idx[t];
            int64_t page = page_table[(int64_t)b * max_pages + j / PAGE];
            int64_t slot = j % PAGE;
            if (page < 0 || page >= num_pages) {
                bad = 1;
                break;
            }
            int64_t row = (page * PAGE + slot) * QK_DIM;
            if (kv_dtype == ORACLE_KV_BF16) {
                const uint16_t *c16 = (const uint16_t *)cache;
                for (int d = 0; d < QK_DIM; ++d)
                    kv[t * QK_DIM + d] = oracle_bf16_to_double(c16[row + d]);
            } else {
                const uint8_t *c8 = (const uint8_t *)cache;
                double sc = (double)scales[page * PAGE + slot];
                for (int d = 0; d < QK_DIM; ++d)
                    kv[t * QK_DIM + d] = oracle_fp8_e4m3_to_double(c8[row + d]) * sc;
            }
        }
        if (bad) {
            {
#pragma omp atomic write
                status = -2;
            }
            free(idx); free(s); free(kv);
            continue;
        }

        /* logits */
        for (int64_t t = 0; t < n; ++t) {
            double acc = 0.0;
            for (int d = 0; d < QK_DIM; ++d)
                acc += qd[d] * kv[t * QK_DIM + d];
            s[t] = scale * acc;
        }
        /* softmax: max, sum, normalise */
        double m = s[0];
        for (int64_t t = 1; t < n; ++t)
            m = fmax(m, s[t]);   /* fmax ignores NaN; NaN logits poison Z below */
        double Z = 0.0;
        for (int64_t t = 0; t < n; ++t)
            Z += exp(s[t] - m);
        /* weighted sum of values = first 512 numbers of each row */
        for (int64_t t = 0; t < n; ++t) {
            double p = exp(s[t] - m) / Z;
            if (probs && idx[t] < max_L)
                probs[i * max_L + idx[t]] = p;
            for (int c = 0; c < V_DIM; ++c)
                o[c] += p * kv[t * QK_DIM + c];
        }
        lse[i] = m + log(Z);
        free(idx); free(s); free(kv);
    }
    return status;
}
