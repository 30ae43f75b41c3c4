/*
 * PreFT CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 statement of what the prefill-only adapter path computes,
 * written from the paper's definitions.  It exists so that the GPU library can be
 * checked against something that can be verified by eye; it is never part of the
 * product path, shares no code with the HIP sources, and must only be used by the
 * tests, the smoke check and the CPU-baseline leg of the benchmark.
 *
 * What is implemented (paper's column-vector notation throughout):
 *   - Eq. 1  masked replacement: a row keeps f(x)_i unless its position i is in P.
 *   - Eq. 2  LoRA:    Phi(f(x)) = f(x) + alpha * B A x,  A in R^{r x m}, B in R^{n x r}.
 *   - Eq. 3  DiReFT:  Phi(h) = h + B^T (A h + b),        A, B in R^{r x d}, b in R^r,
 *            with the scalar prefactor s_r of App. C.2 (s_r = 1 gives Eq. 3 itself);
 *            the prefactor multiplies the whole B^T(Ah + b) term, bias included.
 *   - App. C.2 LoReFT: Phi(h) = h + s_r R^T (W h + b - R h),  W, R in R^{r x d}, b in R^r
 *            (R is the materialised rotation, rows orthonormal in the method; the
 *            arithmetic below does not assume it).
 *   - Eq. 4  P^PreFT = {1..p}: the first p rows of a sequence (its prompt positions);
 *            the all-position set P^A of Sec. 3.2 is every row of the sequence.
 *
 * Batch layout (App. D.3: the flattened token batch delimited by cumulative
 * per-sequence offsets): rows seg_start[s] .. seg_start[s+1]-1 belong to sequence s,
 * which carries adapter seg_adapter[s] (negative or >= N: no adapter) and whose first
 * seg_prompt_len[s] rows are prompt positions.
 *
 * All tensors are read in their storage type (fp64, fp32 or bf16) and widened exactly
 * to fp64; every sum is a left-to-right fp64 loop; outputs are fp64.  No blocking, no
 * fusion, no reordering.
 *
 * Parity pins for every function here live in tests/test_oracle_pins.py.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORA_F64 = 0, ORA_F32 = 1, ORA_BF16 = 2 };
enum { ORA_PROMPT_ONLY = 0, ORA_ALL_POSITIONS = 1 };

/* exact widening of element i of a typed array */
static double ld(const void *p, int64_t i, int dt)
{
    if (dt == ORA_F64) return ((const double *)p)[i];
    if (dt == ORA_F32) return (double)((const float *)p)[i];
    /* bf16 = upper 16 bits of an IEEE fp32 */
    uint32_t bits = ((uint32_t)((const uint16_t *)p)[i]) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static int64_t elem_size(int dt) { return dt == ORA_F64 ? 8 : dt == ORA_F32 ? 4 : 2; }

static const void *row_ptr(const void *base, int64_t row, int64_t ld_elems, int dt)
{
    return (const char *)base + row * ld_elems * elem_size(dt);
}

/*
 * Eq. 1 + Eq. 4: for every row t of the flattened batch, the adapter that acts on it,
 * or -1 if the row is not in the position set (or its sequence has no adapter).
 * Returns 0, or -1 if the segment table is malformed.
 */
int ora_positions(int32_t *row_adapter, int64_t T,
                  const int32_t *seg_start, const int32_t *seg_adapter,
                  const int32_t *seg_prompt_len, int32_t S, int32_t N, int position_set)
{
    for (int64_t t = 0; t < T; ++t) row_adapter[t] = -1;
    if (S > 0 && (seg_start[0] != 0 || seg_start[S] != T)) return -1;
    for (int32_t s = 0; s < S; ++s) {
        int64_t lo = seg_start[s], hi = seg_start[s + 1];
        if (hi < lo) return -1;
        int32_t a = seg_adapter[s];
        if (a < 0 || a >= N) continue;                       /* no adapter: identity  */
        int64_t len = hi - lo;
        int64_t p = seg_prompt_len[s];
        if (p < 0) p = 0;
        if (p > len) p = len;
        int64_t n_in_P = (position_set == ORA_ALL_POSITIONS) ? len : p;   /* Eq. 4 / P^A */
        for (int64_t t = lo; t < lo + n_in_P; ++t) row_adapter[t] = a;
    }
    return 0;
}

/* Eq. 2 on one position: out = y0 + alpha * B (A x).  A is [r,m], B is [n,r], row-major. */
void ora_lora_row(double *out, const void *y0, const void *x,
                  const void *A, const void *B,
                  int64_t m, int64_t n, int32_t r, double alpha, int dt_act, int dt_w)
{
    double *z = (double *)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
    for (int32_t k = 0; k < r; ++k) {                        /* z = A x                */
        double acc = 0.0;
        for (int64_t j = 0; j < m; ++j) acc += ld(A, (int64_t)k * m + j, dt_w) * ld(x, j, dt_act);
        z[k] = acc;
    }
    for (int64_t i = 0; i < n; ++i) {                        /* out = y0 + alpha B z   */
        double acc = 0.0;
        for (int32_t k = 0; k < r; ++k) acc += ld(B, i * r + k, dt_w) * z[k];
        out[i] = ld(y0, i, dt_act) + alpha * acc;
    }
    free(z);
}

/* Eq. 3 (scaled, App. C.2) on one position: out = h + s * B^T (A h + b).  A, B are [r,d]. */
void ora_direft_row(double *out, const void *h,
                    const void *A, const void *B, const void *b,
                    int64_t d, int32_t r, double s, int dt_act, int dt_w)
{
    double *a = (double *)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
    for (int32_t k = 0; k < r; ++k) {                        /* a = A h + b            */
        double acc = 0.0;
        for (int64_t j = 0; j < d; ++j) acc += ld(A, (int64_t)k * d + j, dt_w) * ld(h, j, dt_act);
        a[k] = acc + (b ? ld(b, k, dt_w) : 0.0);
    }
    for (int64_t j = 0; j < d; ++j) {                        /* out = h + s B^T a      */
        double acc = 0.0;
        for (int32_t k = 0; k < r; ++k) acc += ld(B, (int64_t)k * d + j, dt_w) * a[k];
        out[j] = ld(h, j, dt_act) + s * acc;
    }
    free(a);
}

/* App. C.2, LoReFT on one position: out = h + s * R^T (W h + b - R h).  W, R are [r,d]. */
void ora_loreft_row(double *out, const void *h,
                    const void *W, const void *R, const void *b,
                    int64_t d, int32_t r, double s, int dt_act, int dt_w)
{
    double *a = (double *)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
    for (int32_t k = 0; k < r; ++k) {                        /* a = W h + b - R h      */
        double wh = 0.0, rh = 0.0;
        for (int64_t j = 0; j < d; ++j) wh += ld(W, (int64_t)k * d + j, dt_w) * ld(h, j, dt_act);
        for (int64_t j = 0; j < d; ++j) rh += ld(R, (int64_t)k * d + j, dt_w) * ld(h, j, dt_act);
        a[k] = wh + (b ? ld(b, k, dt_w) : 0.0) - rh;
    }
    for (int64_t j = 0; j < d; ++j) {                        /* out = h + s R^T a      */
        double acc = 0.0;
        for (int32_t k = 0; k < r; ++k) acc += ld(R, (int64_t)k * d + j, dt_w) * a[k];
        out[j] = ld(h, j, dt_act) + s * acc;
    }
    free(a);
}

/*
 * LoRA over a batch.  If rows == NULL every row t in [0,T) is produced into out[t];
 * otherwise out[q] holds row rows[q], q < n_rows.  Rows outside the position set are
 * the widened copy of y0 (Eq. 1, "otherwise" branch).
 * x:[T,m] (row stride ldx), y0:[T,n] (row stride ldy), A_pool[a]:[r,m], B_pool[a]:[n,r].
 * With rows != NULL and gathered != 0 the caller has already gathered the selected rows:
 * x and y0 then hold n_rows rows, row q being batch row rows[q] (for batches too large
 * to copy whole); positions and adapters still come from the full segment table.
 */
int ora_lora_batch(double *out, const int64_t *rows, int64_t n_rows,
                   const void *y0, int64_t ldy, const void *x, int64_t ldx,
                   int64_t T, int64_t m, int64_t n,
                   const int32_t *seg_start, const int32_t *seg_adapter,
                   const int32_t *seg_prompt_len, int32_t S,
                   const void *const *A_pool, const void *const *B_pool, int32_t N,
                   int32_t r, double alpha, int position_set, int dt_act, int dt_w, int gathered)
{
    int32_t *row_adapter = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    if (ora_positions(row_adapter, T, seg_start, seg_adapter, seg_prompt_len, S, N, position_set)) {
        free(row_adapter);
        return -1;
    }
    int64_t count = rows ? n_rows : T;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < count; ++q) {
        int64_t t = rows ? rows[q] : q;
        double *o = out + q * n;
        int32_t a = row_adapter[t];
        int64_t src = (rows && gathered) ? q : t;            /* where row t's data sits */
        const void *y0_t = row_ptr(y0, src, ldy, dt_act);
        if (a < 0) {
            for (int64_t i = 0; i < n; ++i) o[i] = ld(y0_t, i, dt_act);
        } else {
            ora_lora_row(o, y0_t, row_ptr(x, src, ldx, dt_act), A_pool[a], B_pool[a],
                         m, n, r, alpha, dt_act, dt_w);
        }
    }
    free(row_adapter);
    return 0;
}

/* DiReFT over a batch; same row-selection and gathering convention.  h:[T,d] (row stride ldh). */
int ora_direft_batch(double *out, const int64_t *rows, int64_t n_rows,
                     const void *h, int64_t ldh, int64_t T, int64_t d,
                     const int32_t *seg_start, const int32_t *seg_adapter,
                     const int32_t *seg_prompt_len, int32_t S,
                     const void *const *A_pool, const void *const *B_pool,
                     const void *const *b_pool, int32_t N,
                     int32_t r, double s, int position_set, int dt_act, int dt_w, int gathered)
{
    int32_t *row_adapter = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    if (ora_positions(row_adapter, T, seg_start, seg_adapter, seg_prompt_len, S, N, position_set)) {
        free(row_adapter);
        return -1;
    }
    int64_t count = rows ? n_rows : T;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < count; ++q) {
        int64_t t = rows ? rows[q] : q;
        double *o = out + q * d;
        int32_t a = row_adapter[t];
        const void *h_t = row_ptr(h, (rows && gathered) ? q : t, ldh, dt_act);
        if (a < 0) {
            for (int64_t j = 0; j < d; ++j) o[j] = ld(h_t, j, dt_act);
        } else {
            ora_direft_row(o, h_t, A_pool[a], B_pool[a], b_pool ? b_pool[a] : NULL,
                           d, r, s, dt_act, dt_w);
        }
    }
    free(row_adapter);
    return 0;
}

/* LoReFT over a batch; same conventions as ora_direft_batch. */
int ora_loreft_batch(double *out, const int64_t *rows, int64_t n_rows,
                     const void *h, int64_t ldh, int64_t T, int64_t d,
                     const int32_t *seg_start, const int32_t *seg_adapter,
                     const int32_t *seg_prompt_len, int32_t S,
                     const void *const *W_pool, const void *const *R_pool,
                     const void *const *b_pool, int32_t N,
                     int32_t r, double s, int position_set, int dt_act, int dt_w, int gathered)
{
    int32_t *row_adapter = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    if (ora_positions(row_adapter, T, seg_start, seg_adapter, seg_prompt_len, S, N, position_set)) {
        free(row_adapter);
        return -1;
    }
    int64_t count = rows ? n_rows : T;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < count; ++q) {
        int64_t t = rows ? rows[q] : q;
        double *o = out + q * d;
        int32_t a = row_adapter[t];
        const void *h_t = row_ptr(h, (rows && gathered) ? q : t, ldh, dt_act);
        if (a < 0) {
            for (int64_t j = 0; j < d; ++j) o[j] = ld(h_t, j, dt_act);
        } else {
            ora_loreft_row(o, h_t, W_pool[a], R_pool[a], b_pool ? b_pool[a] : NULL,
                           d, r, s, dt_act, dt_w);
        }
    }
    free(row_adapter);
    return 0;
}

int ora_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
