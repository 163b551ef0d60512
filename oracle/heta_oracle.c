/*
 * CPU oracle, edge-loop part.  TEST INFRASTRUCTURE ONLY: the product path (the HIP
 * library and its Python binding) never includes, links or calls anything in this
 * directory, and this file shares no code with it.
 *
 * It states the relation-specific aggregation of the HGNN layer (Eq. 1, first line,
 * with AGG_r a GCN-style neighbour sum or mean; Algorithm 1, the per-worker
 * "aggregate neighbour features of S_B^l" step) and its transposed backward
 * (Algorithm 1, the workers' local backpropagation) directly over an explicit edge
 * list {(u_e, v_e)}: one loop over edges, fp64 accumulators, no blocking, no CSR/CSC
 * traversal, no reordering.  Every function is pinned by tests that compare it with a
 * dense count-matrix product, with closed forms and with finite differences.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* deg_r(v) = number of edges whose destination is v (multi-edges counted). */
void oracle_in_degree(int64_t n_edges, const int32_t *dst, int64_t n_dst, int64_t *deg)
{
    memset(deg, 0, (size_t)n_dst * sizeof(int64_t));
    for (int64_t e = 0; e < n_edges; ++e)
        deg[dst[e]] += 1;
}

/*
 * M_r[v] = sum over edges e with v_e = v of H0[row(u_e)],  row(u) = gid[u] if gid else u;
 * with mean != 0 the row is divided by deg_r(v) when deg_r(v) > 0 and stays 0 otherwise.
 * H0 is [*, ld]; M is [n_dst, d] fp64.  Two instances of the same loop: one reads a float32
 * table (the same bytes the GPU path reads, widened to fp64 on load), one an fp64 table
 * (used when H0 is itself an fp64 product of a feature table with a fixed matrix).
 */
#define ORACLE_AGGREGATE_FWD(NAME, T)                                                              \
    void NAME(int64_t n_edges, const int32_t *src, const int32_t *dst, int64_t n_dst, const T *H0, \
              int64_t ld, int32_t d, const int64_t *gid, int32_t mean, double *M)                  \
    {                                                                                              \
        memset(M, 0, (size_t)n_dst * (size_t)d * sizeof(double));                                  \
        for (int64_t e = 0; e < n_edges; ++e) {                                                    \
            int64_t u = gid ? gid[src[e]] : (int64_t)src[e];                                       \
            const T *h = H0 + u * ld;                                                              \
            double *m = M + (int64_t)dst[e] * d;                                                   \
            for (int32_t j = 0; j < d; ++j)                                                        \
                m[j] += (double)h[j];                                                              \
        }                                                                                          \
        if (mean) {                                                                                \
            int64_t *deg = (int64_t *)malloc((size_t)(n_dst > 0 ? n_dst : 1) * sizeof(int64_t));   \
            oracle_in_degree(n_edges, dst, n_dst, deg);                                            \
            for (int64_t v = 0; v < n_dst; ++v) {                                                  \
                if (deg[v] > 0) {                                                                  \
                    double *m = M + v * d;                                                         \
                    double dv = (double)deg[v];                                                    \
                    for (int32_t j = 0; j < d; ++j)                                                \
                        m[j] /= dv;                                                                \
                }                                                                                  \
            }                                                                                      \
            free(deg);                                                                             \
        }                                                                                          \
    }

ORACLE_AGGREGATE_FWD(oracle_aggregate_fwd, float)
ORACLE_AGGREGATE_FWD(oracle_aggregate_fwd_f64, double)

/*
 * Backward of the aggregation: for every edge e,  dH0[u_e] += c_e * dM[v_e],
 * c_e = 1 (sum) or 1/deg_r(v_e) (mean).  dH0 is [n_src, d] fp64 and is ACCUMULATED into,
 * so that the relations sharing a source type add up.  dM is [n_dst, d] fp64.
 */
void oracle_aggregate_bwd(int64_t n_edges, const int32_t *src, const int32_t *dst, int64_t n_dst,
                          const double *dM, int32_t d, int32_t mean, double *dH0)
{
    int64_t *deg = NULL;
    if (mean) {
        deg = (int64_t *)malloc((size_t)(n_dst > 0 ? n_dst : 1) * sizeof(int64_t));
        oracle_in_degree(n_edges, dst, n_dst, deg);
    }
    for (int64_t e = 0; e < n_edges; ++e) {
        const double *g = dM + (int64_t)dst[e] * d;
        double *o = dH0 + (int64_t)src[e] * d;
        double c = mean ? 1.0 / (double)deg[dst[e]] : 1.0;
        for (int32_t j = 0; j < d; ++j)
            o[j] += c * g[j];
    }
    free(deg);
}

/*
 * The transposed adjacency as a CSC: column u lists the destinations of u's out-edges
 * in ascending original edge position (which makes the result unique): count the edges of
 * every column, then walk the edge list once in order and append each edge to its column.
 */
void oracle_csc(int64_t n_edges, const int32_t *src, const int32_t *dst, int64_t n_src,
                int64_t *colptr, int32_t *row)
{
    memset(colptr, 0, (size_t)(n_src + 1) * sizeof(int64_t));
    for (int64_t e = 0; e < n_edges; ++e)
        colptr[src[e] + 1] += 1;
    for (int64_t u = 0; u < n_src; ++u)
        colptr[u + 1] += colptr[u];
    int64_t *fill = (int64_t *)malloc((size_t)(n_src > 0 ? n_src : 1) * sizeof(int64_t));
    memcpy(fill, colptr, (size_t)n_src * sizeof(int64_t));
    for (int64_t e = 0; e < n_edges; ++e)
        row[fill[src[e]]++] = dst[e];
    free(fill);
}
