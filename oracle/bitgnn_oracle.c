/*
 * CPU oracle for binarized GNN layer inference (BitGNN, ICS '23).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition of what
 * the HIP library must compute.  It works on UNPACKED arrays: +-1 values in
 * int8, neighbour lists in CSR, int64 accumulators.  It uses no bit tricks, no
 * popcount, no packed words, and shares no code with the HIP path.  Only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * Every function states the passage of the paper it follows.  OpenMP only
 * splits the outermost (row) loop; every output element is still produced by
 * the literal sum of its definition.
 */
#include <stdint.h>
#include <stddef.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Binarization (Section 2.2, sign function): v = +1 if x >= tau else -1.
 * The paper has tau = 0; a per-column tau is BatchNorm folded into the
 * comparison.  The tie x == tau gives +1.  x: [n][ldx] floats, K used. */
void orc_bin_f32(const float *x, int64_t n, int64_t K, int64_t ldx,
                 const float *tau_or_null, int8_t *v)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t k = 0; k < K; ++k) {
            float tau = tau_or_null ? tau_or_null[k] : 0.0f;
            v[i * K + k] = (x[i * ldx + k] >= tau) ? (int8_t)1 : (int8_t)-1;
        }
}

/* Same for int8 input (x >= 0 -> +1). */
void orc_bin_i8(const int8_t *x, int64_t n, int64_t K, int64_t ldx, int8_t *v)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t k = 0; k < K; ++k)
            v[i * K + k] = (x[i * ldx + k] >= 0) ? (int8_t)1 : (int8_t)-1;
}

/* Feature transformation X W of a layer (Section 2.1, GCNConv equation) with
 * both operands binarized to +-1 (Section 3.1.1, Bi-GCN):
 *     Z[i][c] = sum_k vx[i][k] * vw[k][c]
 * vx: [n][K], vw: [K][M], Z: [n][M]. */
void orc_bmm(const int8_t *vx, int64_t n, int64_t K, const int8_t *vw,
             int64_t M, int64_t *Z)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        int64_t *z = Z + i * M;
        for (int64_t c = 0; c < M; ++c)
            z[c] = 0;
        for (int64_t k = 0; k < K; ++k) {
            int64_t xv = vx[i * K + k];
            const int8_t *w = vw + k * M;
            for (int64_t c = 0; c < M; ++c)
                z[c] += xv * (int64_t)w[c];
        }
    }
}

/* Neighbour aggregation of +-1 activations over a 0/1 adjacency
 * (Section 3.2.2, method 1: walk the non-zeros of the adjacency row; a stored
 * 1 adds +1, a stored -1 adds -1; zeros of the adjacency are skipped):
 *     S[i][c] = sum_{j in N(i)} v[j][c]
 * rowptr: [n+1], col: [nnz], v: [n_src][C], S: [n][C]. */
void orc_spmm_pm1(const int64_t *rowptr, const int32_t *col, int64_t n,
                  const int8_t *v, int64_t C, int64_t *S)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n; ++i) {
        int64_t *s = S + i * C;
        for (int64_t c = 0; c < C; ++c)
            s[c] = 0;
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            const int8_t *vj = v + (int64_t)col[e] * C;
            for (int64_t c = 0; c < C; ++c) {
                if (vj[c] > 0)
                    s[c] += 1;
                else
                    s[c] -= 1;
            }
        }
    }
}

/* Re-binarization of an integer accumulator (Algorithm 1, the c[n] >= 0 test
 * before the store, with the folded BatchNorm threshold T_c in place of 0):
 *     v[i][c] = +1 if acc[i][c] >= T[c] else -1 */
void orc_rebin(const int64_t *acc, int64_t n, int64_t C, const int32_t *T,
               int8_t *v)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t c = 0; c < C; ++c)
            v[i * C + c] = (acc[i * C + c] >= (int64_t)T[c]) ? (int8_t)1 : (int8_t)-1;
}

/* Aggregation of integer (non-binarized) activations over the 0/1 adjacency:
 * the second-layer aggregation of the "binary aggregation" model
 * (Table 3 caption: MM.BBF + BSpMM.FBF), kept in exact integers:
 *     Y[i][c] = sum_{j in N(i)} Z[j][c] */
void orc_spmm_i64(const int64_t *rowptr, const int32_t *col, int64_t n,
                  const int64_t *Z, int64_t M, int64_t *Y)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n; ++i) {
        int64_t *y = Y + i * M;
        for (int64_t c = 0; c < M; ++c)
            y[c] = 0;
        for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            const int64_t *zj = Z + (int64_t)col[e] * M;
            for (int64_t c = 0; c < M; ++c)
                y[c] += zj[c];
        }
    }
}

/* Scaling (SCL, Section 3.1.1) of the last layer: one positive per-class
 * factor.  It commutes with the 0/1 column sum, so it is applied once to the
 * exact integer: logit = (float)((double)alpha[c] * Y[i][c]). */
void orc_scale(const int64_t *Y, int64_t n, int64_t M, const float *alpha,
               float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t c = 0; c < M; ++c)
            out[i * M + c] = (float)((double)alpha[c] * (double)Y[i * M + c]);
}

/* Concatenation [a | b] along the feature axis (auxiliary CONCAT operation,
 * Section 3.1.2, third group of low-level functions). */
void orc_concat(const int8_t *a, int64_t Ka, const int8_t *b, int64_t Kb,
                int64_t n, int8_t *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t k = 0; k < Ka; ++k)
            out[i * (Ka + Kb) + k] = a[i * Ka + k];
        for (int64_t k = 0; k < Kb; ++k)
            out[i * (Ka + Kb) + Ka + k] = b[i * Kb + k];
    }
}

/* Weighted / full-precision aggregation (Section 3.1.1: the BSpMM variants with a
 * full-precision activation operand or output, and the weighted adjacency written as
 * a 0/1 matrix times its factorisation vectors):
 *   Y[i][c] = r[i] * sum_{j in N(i)} f[j] * x[j][c]
 * in double precision: the plain definition.  r or f may be NULL (= 1). */
void orc_spmm_weighted(const int64_t *rowptr, const int32_t *col, int64_t n,
                       const double *x, int64_t C, const double *r,
                       const double *f, double *Y)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t c = 0; c < C; ++c) {
            double s = 0.0;
            for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k) {
                const int64_t j = col[k];
                s += (f ? f[j] : 1.0) * x[j * C + c];
            }
            Y[i * C + c] = (r ? r[i] : 1.0) * s;
        }
    }
}

/* The same sum as single precision takes it when every step is rounded once: neighbour
 * by neighbour in stored order, one multiply and one add each (no fused multiply-add),
 * then one multiply by r[i].  This is the value that decides a bit when the output of
 * a weighted aggregation is binarized again; `volatile` keeps the compiler from
 * contracting or widening the steps. */
void orc_spmm_weighted_f32(const int64_t *rowptr, const int32_t *col, int64_t n,
                           const float *x, int64_t C, const float *r,
                           const float *f, float *Y)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t c = 0; c < C; ++c) {
            volatile float s = 0.0f;
            for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k) {
                const int64_t j = col[k];
                volatile float p = (f ? f[j] : 1.0f) * x[j * C + c];
                s = s + p;
            }
            volatile float y = (r ? r[i] : 1.0f) * s;
            Y[i * C + c] = y;
        }
    }
}

/* Re-binarization of a full-precision value: +1 if y >= tau_c else -1
 * (Section 2.2 with a threshold in place of 0; ties give +1). */
void orc_rebin_f32(const float *y, int64_t n, int64_t C, const float *tau,
                   int8_t *v)
{
    for (int64_t i = 0; i < n; ++i)
        for (int64_t c = 0; c < C; ++c)
            v[i * C + c] = (y[i * C + c] >= tau[c]) ? 1 : -1;
}
