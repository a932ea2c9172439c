/* Host-sanitizer driver for the oracle: the two-token worked example (values from the
 * definition: weights 1/(1+e) and e/(1+e)) and a small paged fp8 problem with an empty
 * sequence, both walked under ASan / UBSan.  Prints "ok" when the worked example's
 * numbers come out. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int omniattn_oracle(int32_t B, int32_t H, const uint16_t *q, const void *cache, int32_t kv_dtype,
                    const float *scales, int64_t num_pages, const int32_t *page_table, int32_t max_pages,
                    const int32_t *seq_lens, int32_t S, int32_t W, double scale, const int32_t *pairs,
                    int64_t n_pairs, double *out, double *lse, double *probs, int64_t max_L, int32_t q_len);

static uint16_t bf16(float f) { uint32_t u; memcpy(&u, &f, 4); return (uint16_t)(u >> 16); }

int main(void)
{
    enum { QK = 576, V = 512, PAGE = 128 };
    /* 1. one sequence of two tokens, one head: q = e_0, k_0 = 0, k_1 = e_0 (logits 0 and 1),
     *    values 1 and 5 in column 0 */
    uint16_t *q = calloc(QK, sizeof *q), *cache = calloc((size_t)PAGE * QK, sizeof *cache);
    int32_t pt[1] = {0}, lens[1] = {2};
    double out[V], lse[1], probs[2];
    if (!q || !cache) return 2;
    q[0] = bf16(1.0f);
    cache[0 * QK + 0] = bf16(0.0f);
    cache[0 * QK + 1] = bf16(1.0f);
    cache[1 * QK + 0] = bf16(1.0f);
    cache[1 * QK + 1] = bf16(5.0f);
    if (omniattn_oracle(1, 1, q, cache, 0, NULL, 1, pt, 1, lens, 1, 1, 1.0, NULL, 1, out, lse, probs, 2, 1)) return 3;
    const double e = exp(1.0);
    if (fabs(probs[0] - 1 / (1 + e)) > 1e-15 || fabs(lse[0] - log(1 + e)) > 1e-15) return 4;
    if (fabs(out[0] - e / (1 + e)) > 1e-15 || fabs(out[1] - (1 + 5 * e) / (1 + e)) > 1e-15) return 5;
    /* 2. three sequences (lengths 0, 5, 130) over two pages each, fp8 codes, shuffled pages */
    int B = 3, H = 2, pages = 6;
    uint8_t *c8 = malloc((size_t)pages * PAGE * QK);
    float *sc = malloc((size_t)pages * PAGE * sizeof *sc);
    uint16_t *q2 = malloc((size_t)B * H * QK * sizeof *q2);
    int32_t pt2[6] = {5, 3, 1, 4, 2, 0}, lens2[3] = {0, 5, 130};
    double *out2 = malloc((size_t)B * H * V * sizeof *out2), lse2[6];
    if (!c8 || !sc || !q2 || !out2) return 6;
    for (size_t i = 0; i < (size_t)pages * PAGE * QK; ++i) c8[i] = (uint8_t)((i * 37u + 11u) % 0x78u);
    for (int i = 0; i < pages * PAGE; ++i) sc[i] = 0.01f * (float)(1 + i % 7);
    for (int i = 0; i < B * H * QK; ++i) q2[i] = bf16((float)((i % 13) - 6) / 64.0f);
    if (omniattn_oracle(B, H, q2, c8, 1, sc, pages, pt2, 2, lens2, 2, 3, 0.07, NULL, (int64_t)B * H, out2, lse2, NULL, 0, 1)) return 7;
    if (!(lse2[0] == -INFINITY) || !isfinite(lse2[2]) || !isfinite(lse2[5])) return 8;
    free(q); free(cache); free(c8); free(sc); free(q2); free(out2);
    puts("ok");
    return 0;
}
