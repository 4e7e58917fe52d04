/*
 * sanitize_main.c -- TEST INFRASTRUCTURE: drives every entry point of krul_oracle.c on small ragged
 * inputs (all three storage types, the causal reading, masks, ties, NaN scores) in a build with
 * -fsanitize=address,undefined, so that an out-of-bounds access, a leak or undefined arithmetic in the
 * oracle fails a test instead of passing unnoticed.  It includes the oracle's source to reach the
 * static functions as well.  It checks no values: the pins do that.
 */
#include "krul_oracle.c"
#include <stdio.h>

static uint32_t rng_state = 12345u;
static uint32_t next_u32(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return rng_state;
}
static float next_unit(void) { return (float)(next_u32() >> 8) / 16777216.0f * 2.0f - 1.0f; }

static void fill(void *p, int dtype, size_t n)
{
    for (size_t i = 0; i < n; ++i) {
        const float v = next_unit();
        if (dtype == ORACLE_F32) {
            ((float *)p)[i] = v;
        } else if (dtype == ORACLE_BF16) {
            uint32_t bits;
            memcpy(&bits, &v, 4);
            ((uint16_t *)p)[i] = (uint16_t)(bits >> 16);
        } else {   /* binary16 patterns with exponents 12..15: values in [2^-3, 2) and their negatives */
            ((uint16_t *)p)[i] = (uint16_t)((next_u32() & 0x8000u) | ((12u + (next_u32() & 3u)) << 10) | (next_u32() & 1023u));
        }
    }
}

int main(void)
{
    int fails = 0;
    const int shapes[][7] = {   /* B, L, Hq, Hkv, d, S, Tq */
        {1, 2, 1, 1, 8, 1, 1}, {2, 3, 4, 2, 16, 37, 5}, {1, 5, 6, 3, 8, 19, 19}, {3, 4, 2, 2, 24, 7, 3}};
    for (int dtype = 0; dtype < 3; ++dtype)
        for (unsigned si = 0; si < sizeof shapes / sizeof shapes[0]; ++si)
            for (int causal = 0; causal < 2; ++causal) {
                const int *sh = shapes[si];
                oracle_shape_t s = {sh[0], sh[1], sh[2], sh[3], sh[4], sh[5], sh[6], dtype, 0.0, causal};
                if (causal && s.n_hist < s.n_query) continue;
                const size_t es = dtype == ORACLE_F32 ? 4 : 2;
                const size_t nq = (size_t)s.batch * s.n_layers * s.n_q_heads * s.n_query * s.head_dim;
                const size_t nk = (size_t)s.batch * s.n_layers * s.n_kv_heads * s.n_hist * s.head_dim;
                void *q = malloc(nq * es), *k = malloc(nk * es);
                fill(q, dtype, nq);
                fill(k, dtype, nk);
                const int B = s.batch, L = s.n_layers, H = s.n_q_heads, NP = L - 1;
                double *ps = malloc(sizeof(double) * B * NP), *hs = malloc(sizeof(double) * B * NP * H);
                double *pd = malloc(sizeof(double) * B * NP), *hd = malloc(sizeof(double) * B * NP * H);
                fails += krul_oracle_pair_similarity(&s, q, k, ps, hs, pd, hd) != 0;
                fails += krul_oracle_pair_similarity(&s, q, k, ps, NULL, NULL, NULL) != 0;
                int32_t units[6] = {0, 0, 0, B - 1, NP - 1, H - 1};
                double uc[2], ud[2];
                fails += krul_oracle_units(&s, q, k, 2, units, uc, ud) != 0;
                int32_t *pairs = malloc(sizeof(int32_t) * B * (L / 2 + 1)), *count = malloc(sizeof(int32_t) * B);
                uint8_t *el = malloc((size_t)B * L);
                for (int i = 0; i < B * L; ++i) el[i] = (uint8_t)(next_u32() % 4 != 0);
                for (int ns = 0; ns <= L / 2; ++ns) {
                    fails += krul_oracle_select_pairs(ps, NULL, B, L, ns, pairs, count) != 0;
                    fails += krul_oracle_select_pairs(ps, el, B, L, ns, pairs, count) != 0;
                }
                ps[0] = NAN;
                fails += krul_oracle_select_pairs(ps, el, B, L, L / 2, pairs, count) != 0;
                if (!causal) {
                    double *mass = malloc(sizeof(double) * B * L);
                    fails += krul_oracle_ir_mass(&s, q, k, 0.2, mass, el) != 0;
                    free(mass);
                }
                double *pc2 = malloc(sizeof(double) * B * L * L), *pd2 = malloc(sizeof(double) * B * L * L);
                double *hc2 = malloc(sizeof(double) * B * H * L * L), *hd2 = malloc(sizeof(double) * B * H * L * L);
                fails += krul_oracle_all_pairs(&s, q, k, pc2, pd2, hc2, hd2) != 0;
                int32_t heads[2] = {B - 1, H - 1};
                fails += krul_oracle_all_pairs_heads(&s, q, k, 1, heads, hc2, hd2) != 0;
                int32_t *pairs2 = malloc(sizeof(int32_t) * B * (L / 2 + 1) * 2);
                for (int ns = 0; ns <= L / 2; ++ns)
                    for (int smaller = 0; smaller < 2; ++smaller)
                        fails += krul_oracle_select_pairs_all(smaller ? pd2 : pc2, smaller, ns & 1 ? el : NULL, B, L, ns, pairs2, count) != 0;
                pd2[(size_t)1 * L + 0] = NAN;
                fails += krul_oracle_select_pairs_all(pd2, 1, NULL, B, L, L / 2, pairs2, count) != 0;
                free(q); free(k); free(ps); free(hs); free(pd); free(hd); free(pairs); free(count); free(el);
                free(pc2); free(pd2); free(hc2); free(hd2); free(pairs2);
            }
    /* argument errors must be refused, not crash */
    oracle_shape_t bad = {0, 1, 1, 1, 8, 1, 1, 0, 0.0, 0};
    fails += krul_oracle_pair_similarity(&bad, &bad, &bad, NULL, NULL, NULL, NULL) == 0;
    fails += krul_oracle_select_pairs(NULL, NULL, 1, 2, 1, NULL, NULL) == 0;
    printf("oracle sanitizer drive: %d unexpected return codes, %d threads\n", fails, krul_oracle_num_threads());
    return fails != 0;
}
