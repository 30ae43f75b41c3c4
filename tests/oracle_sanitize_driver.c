/*
 * Memory-safety check of the CPU oracle (test infrastructure): every entry point of
 * oracle/preft_oracle.c is called on small batches whose buffers are heap blocks of exactly the
 * documented size, in all three storage types, with empty segments, sequences without an adapter,
 * ids past the pool, padded row strides, row selections and gathered rows.  Built with
 * -fsanitize=address,undefined by tests/test_oracle_sanitize.py: any access outside a buffer, any
 * misaligned or overflowing operation aborts the run.  The values themselves are pinned elsewhere
 * (tests/test_oracle_pins.py); here two calls that must agree are compared as a smoke check.
 * With -DPLANT_SHORT_BUFFER every matrix is one element short, which the instrumented oracle must
 * trip over: that build is expected to abort.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

enum { F64 = 0, F32 = 1, BF16 = 2 };

int ora_positions(int32_t *row_adapter, int64_t T, const int32_t *seg_start, const int32_t *seg_adapter,
                  const int32_t *seg_prompt_len, int32_t S, int32_t N, int position_set);
int ora_lora_batch(double *out, const int64_t *rows, int64_t n_rows, const void *y0, int64_t ldy, const void *x,
                   int64_t ldx, int64_t T, int64_t m, int64_t n, const int32_t *seg_start,
                   const int32_t *seg_adapter, const int32_t *seg_prompt_len, int32_t S,
                   const void *const *A_pool, const void *const *B_pool, int32_t N, int32_t r, double alpha,
                   int position_set, int dt_act, int dt_w, int gathered);
int ora_direft_batch(double *out, const int64_t *rows, int64_t n_rows, const void *h, int64_t ldh, int64_t T,
                     int64_t d, const int32_t *seg_start, const int32_t *seg_adapter,
                     const int32_t *seg_prompt_len, int32_t S, const void *const *A_pool,
                     const void *const *B_pool, const void *const *b_pool, int32_t N, int32_t r, double s,
                     int position_set, int dt_act, int dt_w, int gathered);
int ora_loreft_batch(double *out, const int64_t *rows, int64_t n_rows, const void *h, int64_t ldh, int64_t T,
                     int64_t d, const int32_t *seg_start, const int32_t *seg_adapter,
                     const int32_t *seg_prompt_len, int32_t S, const void *const *W_pool,
                     const void *const *R_pool, const void *const *b_pool, int32_t N, int32_t r, double s,
                     int position_set, int dt_act, int dt_w, int gathered);
int ora_threads(void);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static double rnd(void)                       /* small multiples of 1/8: exact in every storage type */
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)((int)((state >> 33) % 17) - 8) / 8.0;
}
static size_t esize(int dt) { return dt == F64 ? 8 : dt == F32 ? 4 : 2; }
static void put(void *p, int64_t i, int dt, double v)
{
    if (dt == F64) ((double *)p)[i] = v;
    else if (dt == F32) ((float *)p)[i] = (float)v;
    else {
        float f = (float)v;
        uint32_t bits;
        memcpy(&bits, &f, 4);
        ((uint16_t *)p)[i] = (uint16_t)(bits >> 16);
    }
}
/* a heap block of exactly rows x ld elements (the last row is not padded beyond its width) */
static void *matrix(int64_t rows, int64_t width, int64_t ld, int dt)
{
    int64_t count = rows > 0 ? (rows - 1) * ld + width : 0;
#ifdef PLANT_SHORT_BUFFER                          /* the check of the check: one element too few */
    if (count > 1) count -= 1;
#endif
    void *p = malloc((size_t)(count > 0 ? count : 1) * esize(dt));
    for (int64_t i = 0; i < count; ++i) put(p, i, dt, rnd());
    return p;
}
static void fail(const char *what)
{
    fprintf(stderr, "oracle_sanitize_driver: %s\n", what);
    exit(1);
}

static void one_case(int dt_act, int dt_w, int position_set)
{
    enum { S = 7, N = 3, M = 10, NOUT = 6, D = 9, R = 2 };
    /* lengths 4,0,1,3,1,2,5: an empty sequence, decode rows, a sequence without adapter, an id past the pool */
    const int32_t seg_start[S + 1] = {0, 4, 4, 5, 8, 9, 11, 16};
    const int32_t seg_adapter[S] = {1, 0, 2, -1, 0, 7, 2};
    const int32_t seg_prompt[S] = {4, 0, 0, 3, 1, 2, 9};   /* the last one exceeds its length: clamped */
    const int64_t T = 16, ldx = M + 3, ldy = NOUT + 2, ldh = D + 1;
    int32_t *sst = malloc(sizeof seg_start), *sad = malloc(sizeof seg_adapter), *spr = malloc(sizeof seg_prompt);
    memcpy(sst, seg_start, sizeof seg_start);
    memcpy(sad, seg_adapter, sizeof seg_adapter);
    memcpy(spr, seg_prompt, sizeof seg_prompt);

    int32_t *owner = malloc(sizeof(int32_t) * T);
    if (ora_positions(owner, T, sst, sad, spr, S, N, position_set)) fail("positions rejected a valid table");
    if (owner[8] != (position_set ? 0 : 0) || owner[5] != -1 || owner[9] != -1) fail("positions: unexpected owner");

    void *x = matrix(T, M, ldx, dt_act), *y0 = matrix(T, NOUT, ldy, dt_act), *h = matrix(T, D, ldh, dt_act);
    const void *A[N], *B[N], *W1[N], *W2[N], *bias[N];
    for (int a = 0; a < N; ++a) {
        A[a] = matrix(R, M, M, dt_w);
        B[a] = matrix(NOUT, R, R, dt_w);
        W1[a] = matrix(R, D, D, dt_w);
        W2[a] = matrix(R, D, D, dt_w);
        bias[a] = matrix(1, R, R, dt_w);
    }
    const void **Ap = malloc(sizeof A), **Bp = malloc(sizeof B), **W1p = malloc(sizeof W1), **W2p = malloc(sizeof W2),
               **bp = malloc(sizeof bias);
    memcpy(Ap, A, sizeof A); memcpy(Bp, B, sizeof B); memcpy(W1p, W1, sizeof W1); memcpy(W2p, W2, sizeof W2);
    memcpy(bp, bias, sizeof bias);

    /* whole batch */
    double *lo = malloc(sizeof(double) * T * NOUT), *di = malloc(sizeof(double) * T * D), *lr = malloc(sizeof(double) * T * D);
    if (ora_lora_batch(lo, NULL, 0, y0, ldy, x, ldx, T, M, NOUT, sst, sad, spr, S, Ap, Bp, N, R, 0.5, position_set,
                       dt_act, dt_w, 0)) fail("lora batch");
    if (ora_direft_batch(di, NULL, 0, h, ldh, T, D, sst, sad, spr, S, W1p, W2p, bp, N, R, 2.0, position_set, dt_act,
                         dt_w, 0)) fail("direft batch");
    if (ora_direft_batch(lr, NULL, 0, h, ldh, T, D, sst, sad, spr, S, W1p, W2p, NULL, N, R, 2.0, position_set, dt_act,
                         dt_w, 0)) fail("direft batch without bias");
    if (ora_loreft_batch(lr, NULL, 0, h, ldh, T, D, sst, sad, spr, S, W1p, W2p, bp, N, R, 0.25, position_set, dt_act,
                         dt_w, 0)) fail("loreft batch");

    /* a row selection read in place, and the same rows gathered into tight buffers */
    const int64_t pick[5] = {15, 0, 8, 5, 3};
    int64_t *rows = malloc(sizeof pick);
    memcpy(rows, pick, sizeof pick);
    double *sel = malloc(sizeof(double) * 5 * NOUT), *gat = malloc(sizeof(double) * 5 * NOUT);
    if (ora_lora_batch(sel, rows, 5, y0, ldy, x, ldx, T, M, NOUT, sst, sad, spr, S, Ap, Bp, N, R, 0.5, position_set,
                       dt_act, dt_w, 0)) fail("lora selection");
    void *xg = malloc(5 * M * esize(dt_act)), *yg = malloc(5 * NOUT * esize(dt_act));
    for (int q = 0; q < 5; ++q) {
        memcpy((char *)xg + q * M * esize(dt_act), (char *)x + pick[q] * ldx * esize(dt_act), M * esize(dt_act));
        memcpy((char *)yg + q * NOUT * esize(dt_act), (char *)y0 + pick[q] * ldy * esize(dt_act), NOUT * esize(dt_act));
    }
    if (ora_lora_batch(gat, rows, 5, yg, NOUT, xg, M, T, M, NOUT, sst, sad, spr, S, Ap, Bp, N, R, 0.5, position_set,
                       dt_act, dt_w, 1)) fail("lora gathered");
    for (int q = 0; q < 5; ++q)
        for (int i = 0; i < NOUT; ++i)
            if (sel[q * NOUT + i] != gat[q * NOUT + i] || sel[q * NOUT + i] != lo[pick[q] * NOUT + i])
                fail("selection, gathered rows and the whole batch disagree");
    double *dsel = malloc(sizeof(double) * 5 * D);
    if (ora_direft_batch(dsel, rows, 5, h, ldh, T, D, sst, sad, spr, S, W1p, W2p, bp, N, R, 2.0, position_set, dt_act,
                         dt_w, 0)) fail("direft selection");
    for (int q = 0; q < 5; ++q)
        for (int j = 0; j < D; ++j)
            if (dsel[q * D + j] != di[pick[q] * D + j]) fail("direft selection and the whole batch disagree");

    /* empty batch; malformed tables are refused, not read past */
    if (ora_lora_batch(lo, NULL, 0, y0, ldy, x, ldx, 0, M, NOUT, sst, sad, spr, 0, Ap, Bp, N, R, 0.5, position_set,
                       dt_act, dt_w, 0)) fail("empty batch");
    sst[3] = 2;                                    /* decreasing offsets */
    if (!ora_positions(owner, T, sst, sad, spr, S, N, position_set)) fail("non-monotone offsets accepted");
    sst[3] = 5;
    sst[S] = 17;                                   /* offsets past T */
    if (!ora_positions(owner, T, sst, sad, spr, S, N, position_set)) fail("offsets past T accepted");

    for (int a = 0; a < N; ++a) {
        free((void *)A[a]); free((void *)B[a]); free((void *)W1[a]); free((void *)W2[a]); free((void *)bias[a]);
    }
    free(Ap); free(Bp); free(W1p); free(W2p); free(bp);
    free(x); free(y0); free(h); free(xg); free(yg);
    free(lo); free(di); free(lr); free(sel); free(gat); free(dsel); free(rows);
    free(owner); free(sst); free(sad); free(spr);
}

int main(void)
{
    if (ora_threads() < 1) fail("thread count");
    for (int dt_act = 0; dt_act < 3; ++dt_act)
        for (int dt_w = 0; dt_w < 3; ++dt_w)
            for (int position_set = 0; position_set < 2; ++position_set) one_case(dt_act, dt_w, position_set);
    puts("oracle_sanitize_driver: ok");
    return 0;
}
