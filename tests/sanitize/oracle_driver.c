/* Runs every entry point of oracle/comet_oracle.c once on small hand-made inputs (including empty
 * inputs and a coordinate out of range) so that a build with -fsanitize=address,undefined can
 * flag reads or writes outside the arrays, leaks, and undefined arithmetic.  Expected values are
 * worked out by hand from the definitions of Section 8.2 of the paper.  Exit status 0 = all good. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef int64_t i64;
int oracle_spmv(i64, const int32_t *, const int32_t *, const double *, i64, i64, const double *, double *, double *);
int oracle_spmm(i64, const int32_t *, const int32_t *, const double *, i64, i64, i64, const double *, double *, double *);
i64 oracle_group_pairs(i64, const int32_t *, const int32_t *, i64 *, int32_t *, int32_t *);
int oracle_ttv(i64, const i64 *, const int32_t *, const double *, i64, const double *, i64, double *, double *);
int oracle_ttm(i64, const i64 *, const int32_t *, const double *, i64, i64, const double *, i64, double *, double *);
int oracle_mttkrp(i64, const int32_t *, const int32_t *, const int32_t *, const double *, i64, i64, i64, i64,
                  const double *, const double *, double *, double *);
int oracle_axpby(i64, double, const double *, const double *, double, const double *, double *, double *);
int oracle_walk(int, const int32_t *, const int32_t *const *, const i64 *, const int32_t *const *, const i64 *, i64,
                int32_t *, int32_t *);

static int fails = 0;
static void check(int ok, const char *what) {
    if (!ok) { fprintf(stderr, "FAILED: %s\n", what); ++fails; }
}
static int near(double a, double b) { return fabs(a - b) <= 1e-14 * (1.0 + fabs(b)); }

/* heap copies so that the sanitizer sees the exact array bounds */
static void *dup_bytes(const void *src, size_t n) { void *p = malloc(n ? n : 1); if (n) memcpy(p, src, n); return p; }
#define DUP(arr) dup_bytes(arr, sizeof(arr))

int main(void) {
    /* 3 x 4 matrix: (0,1)=2 (0,3)=-1 (2,0)=4 (2,1)=0.5; row 1 empty */
    const int32_t ri_[] = {0, 0, 2, 2}, ci_[] = {1, 3, 0, 1};
    const double a_[] = {2.0, -1.0, 4.0, 0.5};
    const double x_[] = {1.0, 2.0, 3.0, 4.0};
    int32_t *ri = DUP(ri_), *ci = DUP(ci_);
    double *a = DUP(a_), *x = DUP(x_);
    double *y = malloc(3 * sizeof(double)), *ya = malloc(3 * sizeof(double));
    check(oracle_spmv(4, ri, ci, a, 3, 4, x, y, ya) == 0, "spmv status");
    check(near(y[0], 2 * 2 - 4) && near(y[1], 0) && near(y[2], 4 + 1), "spmv values");
    check(near(ya[0], 8) && near(ya[1], 0) && near(ya[2], 5), "spmv absolute sums");
    check(oracle_spmv(0, ri, ci, a, 3, 4, x, y, ya) == 0 && y[0] == 0 && y[2] == 0, "spmv without nonzeros");
    check(oracle_spmv(4, ri, ci, a, 3, 3, x, y, ya) == -1, "spmv column out of range is an error");

    const double U_[] = {1, 10, 2, 20, 3, 30, 4, 40};                 /* 4 x 2, row-major */
    double *U = DUP(U_), *Y = malloc(6 * sizeof(double)), *Ya = malloc(6 * sizeof(double));
    check(oracle_spmm(4, ri, ci, a, 3, 4, 2, U, Y, Ya) == 0, "spmm status");
    check(near(Y[0], 0) && near(Y[1], 0) && near(Y[2], 0) && near(Y[3], 0) && near(Y[4], 5) && near(Y[5], 50), "spmm values");
    check(near(Ya[0], 8) && near(Ya[1], 80), "spmm absolute sums");

    /* 2 x 3 x 4 tensor: (0,1,0)=1 (0,1,3)=2 (1,0,2)=3 (1,2,2)=-4 (1,2,3)=5 */
    const int32_t ti_[] = {0, 0, 1, 1, 1}, tj_[] = {1, 1, 0, 2, 2}, tk_[] = {0, 3, 2, 2, 3};
    const double tv_[] = {1, 2, 3, -4, 5};
    int32_t *ti = DUP(ti_), *tj = DUP(tj_), *tk = DUP(tk_);
    double *tv = DUP(tv_);
    i64 *gid = malloc(5 * sizeof(i64));
    int32_t *gi = malloc(5 * sizeof(int32_t)), *gj = malloc(5 * sizeof(int32_t));
    const i64 ng = oracle_group_pairs(5, ti, tj, gid, gi, gj);
    check(ng == 3 && gid[0] == 0 && gid[1] == 0 && gid[2] == 1 && gid[3] == 2 && gid[4] == 2, "pair grouping");
    check(gi[0] == 0 && gj[0] == 1 && gi[1] == 1 && gj[1] == 0 && gi[2] == 1 && gj[2] == 2, "pair list");
    check(oracle_group_pairs(0, ti, tj, gid, gi, gj) == 0, "pair grouping of nothing");
    double *ty = malloc(3 * sizeof(double)), *tya = malloc(3 * sizeof(double));
    check(oracle_ttv(5, gid, tk, tv, 4, x, 3, ty, tya) == 0, "ttv status");
    check(near(ty[0], 1 * 1 + 2 * 4) && near(ty[1], 3 * 3) && near(ty[2], -4 * 3 + 5 * 4), "ttv values");
    check(near(tya[2], 12 + 20), "ttv absolute sums");
    double *TY = malloc(6 * sizeof(double)), *TYa = malloc(6 * sizeof(double));
    check(oracle_ttm(5, gid, tk, tv, 4, 2, U, 3, TY, TYa) == 0, "ttm status");
    check(near(TY[0], 9) && near(TY[1], 90) && near(TY[2], 9) && near(TY[3], 90) && near(TY[4], 8) && near(TY[5], 80), "ttm values");
    const double B_[] = {1, 2, 3, 4, 5, 6};                           /* 3 x 2 */
    double *B = DUP(B_), *M = malloc(4 * sizeof(double)), *Ma = malloc(4 * sizeof(double));
    check(oracle_mttkrp(5, ti, tj, tk, tv, 2, 3, 4, 2, B, U, M, Ma) == 0, "mttkrp status");
    /* row 0: fiber (0,1): (1*1 + 2*4, 1*10 + 2*40) scaled by B[1] = (3, 4) */
    check(near(M[0], 3 * 9) && near(M[1], 4 * 90), "mttkrp row 0");
    /* row 1: B[0] = (1, 2) times (9, 90)  +  B[2] = (5, 6) times (8, 80) */
    check(near(M[2], 9 + 40) && near(M[3], 180 + 480), "mttkrp row 1");
    check(oracle_mttkrp(5, ti, tj, tk, tv, 2, 2, 4, 2, B, U, M, Ma) == -1, "mttkrp coordinate out of range is an error");

    /* y = 2 * (A x) + (-1) * old with old = (1, 1, 1): (0, 0, 5) -> (-1, -1, 9) */
    {
        const double old_[] = {1.0, 1.0, 1.0};
        double *old = DUP(old_), *o = malloc(3 * sizeof(double)), *oa = malloc(3 * sizeof(double));
        check(oracle_spmv(4, ri, ci, a, 3, 4, x, y, ya) == 0, "spmv again");
        check(oracle_axpby(3, 2.0, y, ya, -1.0, old, o, oa) == 0, "axpby status");
        check(near(o[0], -1) && near(o[1], -1) && near(o[2], 9), "axpby values");
        check(near(oa[0], 17) && near(oa[1], 1) && near(oa[2], 11), "axpby absolute sums");
        check(oracle_axpby(3, 2.0, y, ya, 0.0, NULL, o, oa) == 0 && near(o[2], 10), "axpby with beta 0 reads no old values");
        check(oracle_axpby(0, 2.0, y, ya, 1.0, old, o, oa) == 0, "axpby of nothing");
        free(old); free(o); free(oa);
    }

    /* level walker: the 3 x 4 matrix as [D, CU] */
    const int32_t tags_[] = {0, 1};                                    /* D, CU */
    const int32_t pos0_[] = {3}, pos1_[] = {0, 2, 2, 4}, crd1_[] = {1, 3, 0, 1};
    int32_t *tags = DUP(tags_), *pos0 = DUP(pos0_), *pos1 = DUP(pos1_), *crd1 = DUP(crd1_);
    const int32_t *pos[2] = {pos0, pos1}, *crd[2] = {NULL, crd1};
    const i64 pos_len[2] = {1, 4}, crd_len[2] = {0, 4};
    int32_t *coords = malloc(8 * sizeof(int32_t)), *seen = malloc(4 * sizeof(int32_t));
    const int wrc = oracle_walk(2, tags, pos, pos_len, crd, crd_len, 4, coords, seen);
    check(wrc == 0, "walk status");
    if (wrc == 0) {
        int ok = 1;
        for (int p = 0; p < 4; ++p) ok = ok && seen[p] == 1 && coords[2 * p] == ri_[p] && coords[2 * p + 1] == ci_[p];
        check(ok, "walk coordinates");
    }

    free(ri); free(ci); free(a); free(x); free(y); free(ya); free(U); free(Y); free(Ya);
    free(ti); free(tj); free(tk); free(tv); free(gid); free(gi); free(gj); free(ty); free(tya); free(TY); free(TYa);
    free(B); free(M); free(Ma); free(tags); free(pos0); free(pos1); free(crd1); free(coords); free(seen);
    if (fails) return 1;
    puts("oracle sanitize driver: ok");
    return 0;
}
