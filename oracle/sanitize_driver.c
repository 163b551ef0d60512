/*
 * Driver that runs every function of heta_oracle.c on inputs read from a file, for builds with
 * -fsanitize=address,undefined.  TEST INFRASTRUCTURE ONLY (tests/test_oracle_sanitizers.py builds and
 * runs it on the CPU); it adds no arithmetic: it reads arrays, calls the oracle, writes the results.
 *
 * Input file (native endianness):  int64 n_edges, n_src, n_dst, n_table_rows, ld, d, has_gid, mean;
 *   int32 src[n_edges]; int32 dst[n_edges]; float table[n_table_rows * ld]; int64 gid[n_src] (if has_gid);
 *   double dM[n_dst * d].
 * Output file: int64 deg[n_dst]; double M[n_dst * d]; double dH0[n_src * d]; int64 colptr[n_src + 1];
 *   int32 row[n_edges].
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void oracle_in_degree(int64_t n_edges, const int32_t *dst, int64_t n_dst, int64_t *deg);
void oracle_aggregate_fwd(int64_t n_edges, const int32_t *src, const int32_t *dst, int64_t n_dst, const float *H0,
                          int64_t ld, int32_t d, const int64_t *gid, int32_t mean, double *M);
void oracle_aggregate_bwd(int64_t n_edges, const int32_t *src, const int32_t *dst, int64_t n_dst, const double *dM,
                          int32_t d, int32_t mean, double *dH0);
void oracle_csc(int64_t n_edges, const int32_t *src, const int32_t *dst, int64_t n_src, int64_t *colptr, int32_t *row);

static void *alloc_exact(size_t bytes) { return malloc(bytes ? bytes : 1); } /* exact sizes: the sanitizer sees any overrun */

static int read_all(FILE *f, void *p, size_t bytes) { return bytes == 0 || fread(p, 1, bytes, f) == bytes; }

int main(int argc, char **argv)
{
    if (argc != 3) return 2;
    FILE *f = fopen(argv[1], "rb");
    if (!f) return 3;
    int64_t h[8];
    if (!read_all(f, h, sizeof h)) return 4;
    const int64_t n_edges = h[0], n_src = h[1], n_dst = h[2], n_rows = h[3], ld = h[4], d = h[5], has_gid = h[6], mean = h[7];
    int32_t *src = alloc_exact((size_t)n_edges * 4), *dst = alloc_exact((size_t)n_edges * 4);
    float *table = alloc_exact((size_t)(n_rows * ld) * 4);
    int64_t *gid = has_gid ? alloc_exact((size_t)n_src * 8) : NULL;
    double *dM = alloc_exact((size_t)(n_dst * d) * 8);
    if (!read_all(f, src, (size_t)n_edges * 4) || !read_all(f, dst, (size_t)n_edges * 4) ||
        !read_all(f, table, (size_t)(n_rows * ld) * 4) || (has_gid && !read_all(f, gid, (size_t)n_src * 8)) ||
        !read_all(f, dM, (size_t)(n_dst * d) * 8))
        return 5;
    fclose(f);
    int64_t *deg = alloc_exact((size_t)n_dst * 8);
    double *M = alloc_exact((size_t)(n_dst * d) * 8);
    double *dH0 = calloc((size_t)(n_src * d) ? (size_t)(n_src * d) : 1, 8);
    int64_t *colptr = alloc_exact((size_t)(n_src + 1) * 8);
    int32_t *row = alloc_exact((size_t)n_edges * 4);
    oracle_in_degree(n_edges, dst, n_dst, deg);
    oracle_aggregate_fwd(n_edges, src, dst, n_dst, table, ld, (int32_t)d, gid, (int32_t)mean, M);
    oracle_aggregate_bwd(n_edges, src, dst, n_dst, dM, (int32_t)d, (int32_t)mean, dH0);
    oracle_csc(n_edges, src, dst, n_src, colptr, row);
    FILE *o = fopen(argv[2], "wb");
    if (!o) return 6;
    fwrite(deg, 8, (size_t)n_dst, o);
    fwrite(M, 8, (size_t)(n_dst * d), o);
    fwrite(dH0, 8, (size_t)(n_src * d), o);
    fwrite(colptr, 8, (size_t)(n_src + 1), o);
    fwrite(row, 4, (size_t)n_edges, o);
    fclose(o);
    free(src); free(dst); free(table); free(gid); free(dM); free(deg); free(M); free(dH0); free(colptr); free(row);
    return 0;
}
