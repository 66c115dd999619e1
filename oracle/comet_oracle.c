/*
 * CPU oracle for the sparse x dense contractions (TEST INFRASTRUCTURE ONLY).
 *
 * This file is the plain, slow, obviously-correct statement of what the GPU
 * library must compute.  It is used by the tests, by the smoke check and by the
 * benchmark's CPU-baseline leg -- never by the product path -- and it shares no
 * code with the HIP sources.
 *
 * Every operation is the paper's defining sum (Section 8.2, "Sparse Tensor
 * Operations") evaluated by one loop over a coordinate list (i, j[, k], value),
 * in storage order, one term at a time.  The result is exact up to rounding, so
 * the oracle is the definition written out; nothing is blocked, fused or
 * reordered.  Sums use Neumaier's compensated summation in fp64, and next to
 * every output element the oracle returns A = sum |term|, which the tests use as
 * the scale of the absolute error floor.
 *
 * The level walker at the end expands per-level pos/crd storage into a
 * coordinate list by the access rules of Section 4 and Table "Generated code to
 * access nonzeros coordinates" (D, CU, CN, S).
 *
 * All pointers are host pointers; int32 indices, fp64 values (Section 6.1,
 * "Sparse Tensor Data Type").  Return value 0 = ok, negative = bad argument.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef int64_t i64;

/* Neumaier compensated accumulation: (s, c) carries sum = s + c. */
static inline void acc_add(double *s, double *c, double x) {
    double t = *s + x;
    if (fabs(*s) >= fabs(x)) *c += (*s - t) + x;
    else                     *c += (x - t) + *s;
    *s = t;
}

/* out[n] = s[n] + c[n] */
static void acc_finish(double *s, const double *c, i64 n) {
    for (i64 p = 0; p < n; ++p) s[p] += c[p];
}

/* SpMV: y_i = sum_j x_ij v_j   (Section 8.2, SpMV) */
int oracle_spmv(i64 nnz, const int32_t *ri, const int32_t *ci, const double *a,
                i64 I, i64 J, const double *v, double *y, double *yabs) {
    double *c = (double *)calloc((size_t)(I > 0 ? I : 1), sizeof(double));
    if (!c) return -2;
    memset(y, 0, (size_t)I * sizeof(double));
    memset(yabs, 0, (size_t)I * sizeof(double));
    for (i64 p = 0; p < nnz; ++p) {
        i64 i = ri[p], j = ci[p];
        if (i < 0 || i >= I || j < 0 || j >= J) { free(c); return -1; }
        double t = a[p] * v[j];
        acc_add(&y[i], &c[i], t);
        yabs[i] += fabs(t);
    }
    acc_finish(y, c, I);
    free(c);
    return 0;
}

/* SpMM: y_ir = sum_j x_ij u_jr, U and Y row-major (Section 8.2, SpMM; Section 6.2 Step II
 * for the row-major linearisation of dense operands). */
int oracle_spmm(i64 nnz, const int32_t *ri, const int32_t *ci, const double *a,
                i64 I, i64 J, i64 R, const double *U, double *Y, double *Yabs) {
    double *c = (double *)calloc((size_t)(I * R > 0 ? I * R : 1), sizeof(double));
    if (!c) return -2;
    memset(Y, 0, (size_t)(I * R) * sizeof(double));
    memset(Yabs, 0, (size_t)(I * R) * sizeof(double));
    for (i64 p = 0; p < nnz; ++p) {
        i64 i = ri[p], j = ci[p];
        if (i < 0 || i >= I || j < 0 || j >= J) { free(c); return -1; }
        for (i64 r = 0; r < R; ++r) {
            double t = a[p] * U[j * R + r];
            acc_add(&Y[i * R + r], &c[i * R + r], t);
            Yabs[i * R + r] += fabs(t);
        }
    }
    acc_finish(Y, c, I * R);
    free(c);
    return 0;
}

/* Distinct (i, j) pairs of a coordinate list, in lexicographic order.
 * gid[p] receives the rank of nonzero p's pair; gi/gj (capacity nnz) the pairs.
 * Returns the number of distinct pairs. */
typedef struct { int32_t i, j; i64 p; } pair_rec;
static int pair_cmp(const void *x, const void *y) {
    const pair_rec *a = (const pair_rec *)x, *b = (const pair_rec *)y;
    if (a->i != b->i) return a->i < b->i ? -1 : 1;
    if (a->j != b->j) return a->j < b->j ? -1 : 1;
    return a->p < b->p ? -1 : (a->p > b->p ? 1 : 0);
}
i64 oracle_group_pairs(i64 nnz, const int32_t *ci, const int32_t *cj,
                       i64 *gid, int32_t *gi, int32_t *gj) {
    if (nnz == 0) return 0;
    pair_rec *rec = (pair_rec *)malloc((size_t)nnz * sizeof(pair_rec));
    if (!rec) return -2;
    for (i64 p = 0; p < nnz; ++p) { rec[p].i = ci[p]; rec[p].j = cj[p]; rec[p].p = p; }
    qsort(rec, (size_t)nnz, sizeof(pair_rec), pair_cmp);
    i64 g = -1;
    for (i64 q = 0; q < nnz; ++q) {
        if (q == 0 || rec[q].i != rec[q - 1].i || rec[q].j != rec[q - 1].j) {
            ++g; gi[g] = rec[q].i; gj[g] = rec[q].j;
        }
        gid[rec[q].p] = g;
    }
    free(rec);
    return g + 1;
}

/* TTV along the last mode: y_ij = sum_k x_ijk v_k   (Section 8.2, SpTTV, with the contracted
 * mode being the third one).  Output element g belongs to the g-th distinct (i, j) pair. */
int oracle_ttv(i64 nnz, const i64 *gid, const int32_t *ck, const double *a,
               i64 K, const double *v, i64 ngroups, double *y, double *yabs) {
    double *c = (double *)calloc((size_t)(ngroups > 0 ? ngroups : 1), sizeof(double));
    if (!c) return -2;
    memset(y, 0, (size_t)ngroups * sizeof(double));
    memset(yabs, 0, (size_t)ngroups * sizeof(double));
    for (i64 p = 0; p < nnz; ++p) {
        i64 g = gid[p], k = ck[p];
        if (g < 0 || g >= ngroups || k < 0 || k >= K) { free(c); return -1; }
        double t = a[p] * v[k];
        acc_add(&y[g], &c[g], t);
        yabs[g] += fabs(t);
    }
    acc_finish(y, c, ngroups);
    free(c);
    return 0;
}

/* TTM along the last mode: y_ijr = sum_k x_ijk u_kr   (Section 8.2, SpTTM; R takes the place
 * of the contracted mode).  Row g of Y (R entries, row-major) belongs to the g-th pair. */
int oracle_ttm(i64 nnz, const i64 *gid, const int32_t *ck, const double *a,
               i64 K, i64 R, const double *U, i64 ngroups, double *Y, double *Yabs) {
    double *c = (double *)calloc((size_t)(ngroups * R > 0 ? ngroups * R : 1), sizeof(double));
    if (!c) return -2;
    memset(Y, 0, (size_t)(ngroups * R) * sizeof(double));
    memset(Yabs, 0, (size_t)(ngroups * R) * sizeof(double));
    for (i64 p = 0; p < nnz; ++p) {
        i64 g = gid[p], k = ck[p];
        if (g < 0 || g >= ngroups || k < 0 || k >= K) { free(c); return -1; }
        for (i64 r = 0; r < R; ++r) {
            double t = a[p] * U[k * R + r];
            acc_add(&Y[g * R + r], &c[g * R + r], t);
            Yabs[g * R + r] += fabs(t);
        }
    }
    acc_finish(Y, c, ngroups * R);
    free(c);
    return 0;
}

/* MTTKRP for the first mode: m_ir = sum_{j,k} x_ijk b_jr c_kr.  The paper only names the
 * operation (Section 8.3, last paragraph); this is the standard definition of the
 * matricised-tensor-times-Khatri-Rao product with the output indexed by mode 1. */
int oracle_mttkrp(i64 nnz, const int32_t *ci, const int32_t *cj, const int32_t *ck, const double *a,
                  i64 I, i64 J, i64 K, i64 R, const double *B, const double *C,
                  double *M, double *Mabs) {
    double *c = (double *)calloc((size_t)(I * R > 0 ? I * R : 1), sizeof(double));
    if (!c) return -2;
    memset(M, 0, (size_t)(I * R) * sizeof(double));
    memset(Mabs, 0, (size_t)(I * R) * sizeof(double));
    for (i64 p = 0; p < nnz; ++p) {
        i64 i = ci[p], j = cj[p], k = ck[p];
        if (i < 0 || i >= I || j < 0 || j >= J || k < 0 || k >= K) { free(c); return -1; }
        for (i64 r = 0; r < R; ++r) {
            double t = (a[p] * B[j * R + r]) * C[k * R + r];
            acc_add(&M[i * R + r], &c[i * R + r], t);
            Mabs[i * R + r] += fabs(t);
        }
    }
    acc_finish(M, c, I * R);
    free(c);
    return 0;
}

/* Scaled / accumulating result: out = alpha * prod + beta * old, element by element.  Step III of the
 * code generation algorithm (Section 6.2) updates the output element in place, i.e. the product is added
 * to what the output holds (beta = 1); alpha and beta generalise that the usual way.  beta == 0: `old` is
 * not read (it may hold NaN); alpha == 0: `prod` is not read.  out_abs = |alpha| * prod_abs + |beta * old|
 * is the sum of absolute values of everything that was added, for the error bound of a comparison. */
int oracle_axpby(i64 n, double alpha, const double *prod, const double *prod_abs, double beta,
                 const double *old, double *out, double *out_abs) {
    for (i64 p = 0; p < n; ++p) {
        double v = 0.0, a = 0.0;
        if (alpha != 0.0) { v = alpha * prod[p]; a = fabs(alpha) * prod_abs[p]; }
        if (beta != 0.0) { const double o = beta * old[p]; v = v + o; a += fabs(o); }
        out[p] = v;
        out_abs[p] = a;
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Level walker (Section 4; Table "Generated code to access nonzeros coordinates").
 *
 *   D : for i in 0 .. pos[0]            coordinate i,      child position m*pos[0] + i
 *   CU: for p in pos[m] .. pos[m+1]     coordinate crd[p], child position p
 *   CN: for p in pos[0] .. pos[1]       coordinate crd[p], child position p
 *   S :                                 coordinate crd[m], child position m
 *
 * where m is the position handed down by the level above (0 at the root).  The position
 * reached below the last level indexes the value array.  coords[q*order + l] receives the
 * level-l coordinate of value position q; seen[q] counts how often position q was reached
 * (a well-formed tensor reaches each exactly once).
 * ------------------------------------------------------------------------------------------ */
enum { TAG_D = 0, TAG_CU = 1, TAG_CN = 2, TAG_S = 3 };

typedef struct {
    int order;
    const int32_t *tags;
    const int32_t *const *pos; const i64 *pos_len;
    const int32_t *const *crd; const i64 *crd_len;
    i64 nvals;
    int32_t *coords; int32_t *seen;
    int32_t cur[8];
    int err;
} walk_ctx;

static void walk_level(walk_ctx *w, int l, i64 m) {
    if (w->err) return;
    if (l == w->order) {
        if (m < 0 || m >= w->nvals) { w->err = -3; return; }
        for (int q = 0; q < w->order; ++q) w->coords[m * w->order + q] = w->cur[q];
        w->seen[m] += 1;
        return;
    }
    const int32_t *pos = w->pos[l], *crd = w->crd[l];
    switch (w->tags[l]) {
    case TAG_D: {
        if (w->pos_len[l] < 1) { w->err = -4; return; }
        i64 size = pos[0];
        for (i64 i = 0; i < size; ++i) { w->cur[l] = (int32_t)i; walk_level(w, l + 1, m * size + i); }
        break; }
    case TAG_CU: {
        if (m + 1 >= w->pos_len[l]) { w->err = -5; return; }
        for (i64 p = pos[m]; p < pos[m + 1]; ++p) {
            if (p < 0 || p >= w->crd_len[l]) { w->err = -6; return; }
            w->cur[l] = crd[p]; walk_level(w, l + 1, p);
        }
        break; }
    case TAG_CN: {
        if (w->pos_len[l] < 2) { w->err = -7; return; }
        for (i64 p = pos[0]; p < pos[1]; ++p) {
            if (p < 0 || p >= w->crd_len[l]) { w->err = -6; return; }
            w->cur[l] = crd[p]; walk_level(w, l + 1, p);
        }
        break; }
    case TAG_S: {
        if (m < 0 || m >= w->crd_len[l]) { w->err = -8; return; }
        w->cur[l] = crd[m]; walk_level(w, l + 1, m);
        break; }
    default: w->err = -9;
    }
}

int oracle_walk(int order, const int32_t *tags,
                const int32_t *const *pos, const i64 *pos_len,
                const int32_t *const *crd, const i64 *crd_len,
                i64 nvals, int32_t *coords, int32_t *seen) {
    if (order < 1 || order > 8) return -1;
    walk_ctx w;
    memset(&w, 0, sizeof w);
    w.order = order; w.tags = tags; w.pos = pos; w.pos_len = pos_len; w.crd = crd; w.crd_len = crd_len;
    w.nvals = nvals; w.coords = coords; w.seen = seen;
    memset(seen, 0, (size_t)nvals * sizeof(int32_t));
    walk_level(&w, 0, 0);
    return w.err;
}
