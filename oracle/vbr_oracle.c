/*
 * CPU oracle for the blocked sparse-times-dense path (1-SA reordering, VBR index, C = A.B).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, written to be checked against the paper by eye.
 * It shares no code, header, table or helper with the HIP library; nothing in the product
 * path calls it.  Only tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * What follows the paper step by step (the blocking is a greedy heuristic whose result depends
 * on the visiting order, so the steps are taken in the paper's order):
 *   - quotient rows                     : section 3.1, Eq. 4
 *   - grouping of identical quotient rows: Algorithm 1 applied to quotient rows (section 3.1);
 *                                          the hash of Eq. 5 is only a device to find identical
 *                                          rows ("can be replaced by any hash"), so the oracle
 *                                          finds them by sorting the patterns themselves
 *   - greedy merge with pattern update  : Algorithm 2 (section 3.1)
 *   - merge condition                   : section 3.2, conditions 1 and 2 (Jaccard, Eq. 3)
 * What is a plain definition written out:
 *   - C = A.B and the bound matrix S = |A|.|B| in binary64 straight from the CSR matrix
 *     (section 4.4.1: the blocked routine multiplies A by a dense B; fill-in zeros add nothing).
 *
 * Readings taken where the paper is silent (each is listed in the design notes of the repo):
 *   similarity "at least tau" (the proof of Theorem 1 uses >=); I/U evaluated as one binary64
 *   division; the merge limit floor(lambda0 / (1 - tau/2)) evaluated once per seed in binary64;
 *   lambda0 counts column blocks (quotient nonzeros); two empty patterns are similar; classes of
 *   identical quotient rows are visited in order of their smallest row; groups are numbered in
 *   seed order; rows inside a group ascend; every stored CSR entry counts as a nonzero.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

/* ------------------------------------------------------------------ quotient rows (Eq. 4) */
/* pat_ptr[i]..pat_ptr[i+1] delimit the ascending list of column blocks row i touches. */
static int build_patterns(int64_t n_rows, const int64_t *row_ptr, const int32_t *col_idx,
                          int32_t col_block, int64_t **pat_ptr_out, int32_t **pat_out)
{
    int64_t *pat_ptr = (int64_t *)malloc((size_t)(n_rows + 1) * sizeof(int64_t));
    int32_t *pat = (int32_t *)malloc((size_t)(row_ptr[n_rows] > 0 ? row_ptr[n_rows] : 1) * sizeof(int32_t));
    if (!pat_ptr || !pat) { free(pat_ptr); free(pat); return -1; }
    int64_t w = 0;
    pat_ptr[0] = 0;
    for (int64_t i = 0; i < n_rows; ++i) {
        int32_t last = -1;
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            int32_t j = col_idx[p] / col_block;     /* block Q_j holding this column */
            if (j != last) { pat[w++] = j; last = j; }
        }
        pat_ptr[i + 1] = w;
    }
    *pat_ptr_out = pat_ptr;
    *pat_out = pat;
    return 0;
}

/* ------------------------------------------------------------------ identical quotient rows */
static const int64_t *g_pat_ptr;
static const int32_t *g_pat;

static int cmp_pattern_then_row(const void *a, const void *b)
{
    int64_t ra = *(const int64_t *)a, rb = *(const int64_t *)b;
    int64_t la = g_pat_ptr[ra + 1] - g_pat_ptr[ra], lb = g_pat_ptr[rb + 1] - g_pat_ptr[rb];
    const int32_t *pa = g_pat + g_pat_ptr[ra], *pb = g_pat + g_pat_ptr[rb];
    int64_t l = la < lb ? la : lb;
    for (int64_t t = 0; t < l; ++t)
        if (pa[t] != pb[t]) return pa[t] < pb[t] ? -1 : 1;
    if (la != lb) return la < lb ? -1 : 1;
    return ra < rb ? -1 : (ra > rb ? 1 : 0);
}

static int same_pattern(int64_t ra, int64_t rb)
{
    int64_t la = g_pat_ptr[ra + 1] - g_pat_ptr[ra], lb = g_pat_ptr[rb + 1] - g_pat_ptr[rb];
    if (la != lb) return 0;
    return memcmp(g_pat + g_pat_ptr[ra], g_pat + g_pat_ptr[rb], (size_t)la * sizeof(int32_t)) == 0;
}

/*
 * 1-SA.  similarity_only != 0 drops condition 2 of section 3.2 (used only to reproduce the
 * pathological example of that section).
 * perm[new position] = old row; row_groups[g] = first position of group g; row_groups[G] = n_rows.
 */
int oracle_sa1(int64_t n_rows, int64_t n_cols, const int64_t *row_ptr, const int32_t *col_idx,
               int32_t col_block, double tau, int32_t similarity_only,
               int32_t *perm, int32_t *row_groups, int32_t *n_groups)
{
    if (n_rows < 0 || col_block <= 0 || n_cols % col_block != 0 || !(tau >= 0.0 && tau <= 1.0)) return -1;
    int64_t kb = n_cols / col_block;
    int64_t *pat_ptr; int32_t *pat;
    if (build_patterns(n_rows, row_ptr, col_idx, col_block, &pat_ptr, &pat)) return -2;

    /* classes of identical quotient rows; rep[c] = smallest row of class c, classes by rising rep */
    int64_t *order = (int64_t *)malloc((size_t)(n_rows + 1) * sizeof(int64_t));
    int64_t *class_of = (int64_t *)malloc((size_t)(n_rows + 1) * sizeof(int64_t)); /* row -> rep row */
    for (int64_t i = 0; i < n_rows; ++i) order[i] = i;
    g_pat_ptr = pat_ptr; g_pat = pat;
    qsort(order, (size_t)n_rows, sizeof(int64_t), cmp_pattern_then_row);
    for (int64_t t = 0; t < n_rows; ++t) {
        /* equal patterns are adjacent and, among them, rows ascend: the first one is the smallest */
        if (t > 0 && same_pattern(order[t - 1], order[t])) class_of[order[t]] = class_of[order[t - 1]];
        else class_of[order[t]] = order[t];
    }
    int64_t n_cls = 0;
    int64_t *rep = (int64_t *)malloc((size_t)(n_rows + 1) * sizeof(int64_t));
    for (int64_t i = 0; i < n_rows; ++i) if (class_of[i] == i) rep[n_cls++] = i;   /* rising */

    /* Algorithm 2 over the classes */
    int64_t *grp = (int64_t *)malloc((size_t)(n_cls + 1) * sizeof(int64_t));      /* class -> group */
    unsigned char *inP = (unsigned char *)calloc((size_t)(kb + 1), 1);             /* current pattern */
    int32_t *Plist = (int32_t *)malloc((size_t)(kb + 1) * sizeof(int32_t));
    for (int64_t c = 0; c < n_cls; ++c) grp[c] = -1;
    int64_t G = 0;
    for (int64_t i = 0; i < n_cls; ++i) {
        if (grp[i] != -1) continue;
        grp[i] = G;
        int64_t sizeP = 0;
        for (int64_t p = pat_ptr[rep[i]]; p < pat_ptr[rep[i] + 1]; ++p) { inP[pat[p]] = 1; Plist[sizeP++] = pat[p]; }
        int64_t lambda0 = sizeP;
        int64_t lam_max = (int64_t)floor((double)lambda0 / (1.0 - 0.5 * tau));
        for (int64_t j = i + 1; j < n_cls; ++j) {
            if (grp[j] != -1) continue;
            const int32_t *v = pat + pat_ptr[rep[j]];
            int64_t sizeV = pat_ptr[rep[j] + 1] - pat_ptr[rep[j]];
            int64_t I = 0;
            for (int64_t t = 0; t < sizeV; ++t) I += inP[v[t]];
            int64_t U = sizeP + sizeV - I;
            int similar = (U == 0) ? 1 : ((double)I / (double)U >= tau);
            int within = similarity_only ? 1 : (U <= lam_max);
            if (similar && within) {
                grp[j] = G;
                for (int64_t t = 0; t < sizeV; ++t)
                    if (!inP[v[t]]) { inP[v[t]] = 1; Plist[sizeP++] = v[t]; }      /* pattern <- OR */
            }
        }
        for (int64_t t = 0; t < sizeP; ++t) inP[Plist[t]] = 0;
        ++G;
    }

    /* rows sorted by group (stable in the row index) */
    int64_t *count = (int64_t *)calloc((size_t)(G + 1), sizeof(int64_t));
    int64_t *cls_index = (int64_t *)malloc((size_t)(n_rows + 1) * sizeof(int64_t)); /* rep row -> class */
    for (int64_t c = 0; c < n_cls; ++c) cls_index[rep[c]] = c;
    for (int64_t r = 0; r < n_rows; ++r) count[grp[cls_index[class_of[r]]]]++;
    row_groups[0] = 0;
    for (int64_t g = 0; g < G; ++g) row_groups[g + 1] = row_groups[g] + (int32_t)count[g];
    for (int64_t g = 0; g < G; ++g) count[g] = row_groups[g];
    for (int64_t r = 0; r < n_rows; ++r) perm[count[grp[cls_index[class_of[r]]]]++] = (int32_t)r;
    *n_groups = (int32_t)G;

    free(pat_ptr); free(pat); free(order); free(class_of); free(rep); free(grp); free(inP);
    free(Plist); free(count); free(cls_index);
    return 0;
}

/*
 * VBR index for a given row partition: per group the ascending list of column blocks that hold
 * at least one stored entry of the group's rows (only nonzero blocks are kept, section 3.1),
 * and the running element offset of each block (a block of group g holds h_g * col_block
 * elements, zero-filled).  blk_col and blk_off must have room for the worst case
 * (min(nnz, n_groups * n_cols / col_block) blocks, +1 for blk_off).
 */
int oracle_vbr_index(int64_t n_rows, int64_t n_cols, const int64_t *row_ptr, const int32_t *col_idx,
                     int32_t col_block, const int32_t *perm, const int32_t *row_groups, int32_t n_groups,
                     int64_t *blk_ptr, int32_t *blk_col, int64_t *blk_off, int64_t *n_blocks)
{
    if (col_block <= 0 || n_cols % col_block != 0) return -1;
    int64_t kb = n_cols / col_block;
    unsigned char *seen = (unsigned char *)calloc((size_t)(kb + 1), 1);
    if (!seen) return -2;
    int64_t nb = 0, off = 0;
    blk_ptr[0] = 0;
    blk_off[0] = 0;
    for (int32_t g = 0; g < n_groups; ++g) {
        int64_t h = row_groups[g + 1] - row_groups[g];
        for (int64_t q = row_groups[g]; q < row_groups[g + 1]; ++q) {
            int64_t r = perm[q];
            for (int64_t p = row_ptr[r]; p < row_ptr[r + 1]; ++p) seen[col_idx[p] / col_block] = 1;
        }
        for (int64_t j = 0; j < kb; ++j) {
            if (!seen[j]) continue;
            seen[j] = 0;
            blk_col[nb] = (int32_t)j;
            off += h * col_block;
            blk_off[++nb] = off;
        }
        blk_ptr[g + 1] = nb;
    }
    (void)n_rows;
    *n_blocks = nb;
    free(seen);
    return 0;
}

/*
 * C = A.B and S = |A|.|B| in binary64 from the CSR matrix, for the listed rows only
 * (rows == NULL: all rows, n_sel = n_rows).  vals and B are the 16-bit inputs already
 * converted exactly to binary64.  C and S are n_sel x N, row-major; S may be NULL.
 * One output row is one sequential sum over the row's entries in CSR order.
 */
int oracle_spmm(int64_t n_rows, const int64_t *row_ptr, const int32_t *col_idx, const double *vals,
                const double *B, int64_t N, const int64_t *rows, int64_t n_sel, double *C, double *S)
{
    if (N < 0) return -1;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t q = 0; q < n_sel; ++q) {
        int64_t i = rows ? rows[q] : q;
        double *c = C + q * N;
        double *s = S ? S + q * N : 0;
        for (int64_t n = 0; n < N; ++n) c[n] = 0.0;
        if (s) for (int64_t n = 0; n < N; ++n) s[n] = 0.0;
        if (i < 0 || i >= n_rows) continue;
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            double a = vals[p];
            const double *b = B + (int64_t)col_idx[p] * N;
            for (int64_t n = 0; n < N; ++n) c[n] += a * b[n];
            if (s) {
                double aa = fabs(a);
                for (int64_t n = 0; n < N; ++n) s[n] += aa * fabs(b[n]);
            }
        }
    }
    return 0;
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
