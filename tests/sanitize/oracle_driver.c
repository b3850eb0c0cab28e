/* Host-only exerciser for the C oracle (oracle/tree_attention_oracle.c), built with
 * -fsanitize=address,undefined by tests/test_sanitizers.py. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_tree_attention(const float *q, const float *k, const float *v, double *out, const int32_t *node_tok_begin,
                          const int32_t *node_tok_len, const int32_t *node_parent, int32_t n_nodes,
                          const int32_t *query_node, int32_t nq, int32_t ntok, int32_t Hq, int32_t Hkv, int32_t d,
                          double scale, int32_t nthreads, int32_t *used_threads);

static uint64_t state = 12345;
static uint32_t rnd(void) {
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(state >> 33);
}

int main(void) {
    for (int it = 0; it < 40; ++it) {
        const int32_t n = 1 + (int32_t)(rnd() % 9), nq = (int32_t)(rnd() % 7), Hkv = 1 + (int32_t)(rnd() % 3);
        const int32_t G = 1 + (int32_t)(rnd() % 3), Hq = Hkv * G, d = 8 * (1 + (int32_t)(rnd() % 4));
        int32_t begin[16], len[16], parent[16], qn[8], cur = 0;
        for (int32_t u = 0; u < n; ++u) {
            parent[u] = u == 0 ? -1 : (int32_t)(rnd() % (uint32_t)u);
            len[u] = (int32_t)(rnd() % 30);
            begin[u] = cur;
            cur += len[u] + (int32_t)(rnd() % 3);
        }
        const int32_t ntok = cur + 1;
        for (int32_t j = 0; j < nq; ++j) qn[j] = (int32_t)(rnd() % (uint32_t)n);
        float *q = malloc(sizeof(float) * (size_t)(nq ? nq : 1) * Hq * d);
        float *k = malloc(sizeof(float) * (size_t)ntok * Hkv * d), *v = malloc(sizeof(float) * (size_t)ntok * Hkv * d);
        double *o = malloc(sizeof(double) * (size_t)(nq ? nq : 1) * Hq * d);
        for (size_t i = 0; i < (size_t)nq * Hq * d; ++i) q[i] = (float)(rnd() % 2001) / 1000.f - 1.f;
        for (size_t i = 0; i < (size_t)ntok * Hkv * d; ++i) {
            k[i] = (float)(rnd() % 2001) / 1000.f - 1.f;
            v[i] = (float)(rnd() % 2001) / 1000.f - 1.f;
        }
        int32_t used = 0;
        const int rc = oracle_tree_attention(q, k, v, o, begin, len, parent, n, qn, nq, ntok, Hq, Hkv, d, 0.25, 2, &used);
        if (rc != 0) return 2;
        for (size_t i = 0; i < (size_t)nq * Hq * d; ++i)
            if (!(o[i] > -4.0 && o[i] < 4.0)) return 3; /* a convex combination of values in [-1, 1] */
        free(q); free(k); free(v); free(o);
    }
    puts("oracle ok");
    return 0;
}
