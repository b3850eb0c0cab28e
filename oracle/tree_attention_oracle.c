/*
 * TEST INFRASTRUCTURE ONLY -- the fp64 oracle for tree-attention decode.
 *
 * Only the test-suite, the smoke check and the benchmark's cpu_baseline leg may
 * build or call this file.  The product (libdeft.so) shares no code with it.
 *
 * What it computes is the plain definition the method must reproduce exactly
 * (the paper states the method is mathematically equivalent to vanilla
 * attention; Section 3.1 defines <q,k,v> = Softmax(q k^T / sqrt(d)) v):
 * for every query j and query head h,
 *
 *     path(j) = all tokens of all nodes from the root down to query_node[j], inclusive
 *     kvh     = h / (Hq / Hkv)
 *     s_t     = scale * sum_c Q[j,h,c] * K[t,kvh,c]           t in path(j)
 *     O[j,h,:] = sum_t softmax_t(s) * V[t,kvh,:]
 *
 * There is no chunking, no merge, no reordering: one query, one path, one
 * max-subtracted softmax, all in double precision.  Inputs are float (every
 * bf16 value is exactly representable) and are widened to double on use.
 *
 * Pinned by tests/test_oracle_attention.py against a library SDPA on
 * single-branch trees, a dense reachability-mask formulation, closed forms and
 * invariances.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/*
 * Core: node u owns extents ext_ptr[u] .. ext_ptr[u+1]-1, each a run of physical rows
 * [ext_begin, ext_begin + ext_len); its tokens are those runs in order.  A contiguous cache has one
 * extent per node, a paged cache one per page.
 * Returns 0 on success; -1 bad argument; -2 malformed tree (cycle / bad index); -3 out of memory.
 */
int oracle_tree_attention_extents(const float *Q, const float *K, const float *V, double *O,
                                  const int32_t *ext_ptr, const int32_t *ext_begin, const int32_t *ext_len,
                                  const int32_t *node_parent, int32_t n_nodes,
                                  const int32_t *query_node, int32_t nq, int32_t ntok,
                                  int32_t Hq, int32_t Hkv, int32_t d, double scale, int32_t nthreads,
                                  int32_t *threads_used)
{
    if (!Q || !K || !V || !O || !ext_ptr || n_nodes <= 0 || nq < 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv != 0)
        return -1;
    const int group = Hq / Hkv;
    int status = 0;
    int used = 1;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif

#pragma omp parallel
    {
#ifdef _OPENMP
#pragma omp single
        used = omp_get_num_threads();
#endif
        double *s = NULL;      /* scores of one (query, head) over its path */
        int64_t *tok = NULL;   /* physical token index of each path position */
        int64_t cap = 0;

#pragma omp for schedule(dynamic, 1)
        for (int64_t jh = 0; jh < (int64_t)nq * Hq; ++jh) {
            const int j = (int)(jh / Hq), h = (int)(jh % Hq);
            const int kvh = h / group;

            /* walk parent pointers from the query's node up to the root */
            int64_t n = 0;
            int steps = 0, bad = 0;
            for (int u = query_node[j]; u != -1; u = node_parent[u]) {
                if (u < 0 || u >= n_nodes || ++steps > n_nodes) { bad = 1; break; }
                for (int32_t e = ext_ptr[u]; e < ext_ptr[u + 1]; ++e) {
                    if (ext_len[e] < 0 || ext_begin[e] < 0 || (int64_t)ext_begin[e] + ext_len[e] > ntok) { bad = 1; break; }
                    n += ext_len[e];
                }
                if (bad) break;
            }
            if (bad) {
#pragma omp atomic write
                status = -2;
                continue;
            }
            if (n > cap) {
                free(s); free(tok);
                cap = n;
                s = (double *)malloc(sizeof(double) * (size_t)cap);
                tok = (int64_t *)malloc(sizeof(int64_t) * (size_t)cap);
                if (!s || !tok) {
#pragma omp atomic write
                    status = -3;
                    cap = 0; free(s); free(tok); s = NULL; tok = NULL;
                    continue;
                }
            }
            int64_t p = 0;
            for (int u = query_node[j]; u != -1; u = node_parent[u])
                for (int32_t e = ext_ptr[u]; e < ext_ptr[u + 1]; ++e)
                    for (int32_t t = 0; t < ext_len[e]; ++t)
                        tok[p++] = (int64_t)ext_begin[e] + t;

            const float *q = Q + ((int64_t)j * Hq + h) * d;
            double *o = O + ((int64_t)j * Hq + h) * d;
            for (int c = 0; c < d; ++c) o[c] = 0.0;
            if (n == 0) continue; /* empty path: output defined as zero */

            double smax = -INFINITY;
            for (int64_t i = 0; i < n; ++i) {
                const float *k = K + (tok[i] * Hkv + kvh) * d;
                double acc = 0.0;
                for (int c = 0; c < d; ++c) acc += (double)q[c] * (double)k[c];
                s[i] = acc * scale;
                if (s[i] > smax) smax = s[i];
            }
            double denom = 0.0;
            for (int64_t i = 0; i < n; ++i) {
                s[i] = exp(s[i] - smax);
                denom += s[i];
            }
            for (int64_t i = 0; i < n; ++i) {
                const float *v = V + (tok[i] * Hkv + kvh) * d;
                const double w = s[i] / denom;
                for (int c = 0; c < d; ++c) o[c] += w * (double)v[c];
            }
        }
        free(s);
        free(tok);
    }
    if (threads_used) *threads_used = used;
    return status;
}

/* Node-contiguous cache: node u owns rows [node_tok_begin[u], +node_tok_len[u]). */
int oracle_tree_attention(const float *Q, const float *K, const float *V, double *O,
                          const int32_t *node_tok_begin, const int32_t *node_tok_len,
                          const int32_t *node_parent, int32_t n_nodes,
                          const int32_t *query_node, int32_t nq, int32_t ntok,
                          int32_t Hq, int32_t Hkv, int32_t d, double scale, int32_t nthreads,
                          int32_t *threads_used)
{
    if (!node_tok_begin || !node_tok_len || n_nodes <= 0) return -1;
    int32_t *ptr = (int32_t *)malloc(sizeof(int32_t) * ((size_t)n_nodes + 1));
    if (!ptr) return -3;
    for (int32_t u = 0; u <= n_nodes; ++u) ptr[u] = u; /* one extent per node */
    const int rc = oracle_tree_attention_extents(Q, K, V, O, ptr, node_tok_begin, node_tok_len, node_parent, n_nodes,
                                                 query_node, nq, ntok, Hq, Hkv, d, scale, nthreads, threads_used);
    free(ptr);
    return rc;
}
