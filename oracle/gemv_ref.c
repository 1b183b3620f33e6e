/*
 * Test infrastructure, not product code: the reference result of the hot path.
 *
 * The executor under test reaches, faster, exactly the textbook matrix-vector
 * product of the paper's running example O = M @ N (Section 3, "Execution
 * Example").  This file is that definition written out as plain loops:
 * fp32 inputs, every product and every sum in fp64, no blocking, no
 * reordering, one thread.  It shares nothing with the HIP path.
 *
 * Only tests, the smoke check and the bench's cpu_baseline leg may call it.
 */
#include <stdint.h>
#include <stddef.h>
#include <math.h>

/* Dense:  Y[b][i] = sum_j M[i][j] * X[b][j]      (M row-major, leading dimension ld >= K)
 * Yabs[b][i] = sum_j |M[i][j] * X[b][j]|  (the scale of the error bound); may be NULL. */
void gemv_ref_dense(const float *M, int64_t rows, int64_t K, int64_t ld,
                    const float *X, int32_t B, double *Y, double *Yabs)
{
    for (int32_t b = 0; b < B; b++) {
        for (int64_t i = 0; i < rows; i++) {
            double s = 0.0, a = 0.0;
            for (int64_t j = 0; j < K; j++) {
                double p = (double)M[i * ld + j] * (double)X[(int64_t)b * K + j];
                s += p;
                a += fabs(p);
            }
            Y[(int64_t)b * rows + i] = s;
            if (Yabs) Yabs[(int64_t)b * rows + i] = a;
        }
    }
}

/* Ragged: n_seg independent row segments stacked in M (rows row_off[s] .. row_off[s+1]-1,
 * each row K contiguous floats); segment s is multiplied by its own vector X[s][0..K).
 *         Y[row_off[s] + i] = sum_j M[row_off[s] + i][j] * X[s][j]                       */
void gemv_ref_ragged(const float *M, const int64_t *row_off, int32_t n_seg, int64_t K,
                     const float *X, double *Y, double *Yabs)
{
    for (int32_t s = 0; s < n_seg; s++) {
        for (int64_t i = row_off[s]; i < row_off[s + 1]; i++) {
            double acc = 0.0, a = 0.0;
            for (int64_t j = 0; j < K; j++) {
                double p = (double)M[i * K + j] * (double)X[(int64_t)s * K + j];
                acc += p;
                a += fabs(p);
            }
            Y[i] = acc;
            if (Yabs) Yabs[i] = a;
        }
    }
}
