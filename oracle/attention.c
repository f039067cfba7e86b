/*
 * CPU oracle for ragged-cache attention -- TEST INFRASTRUCTURE ONLY.
 *
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may call
 * this file.  It shares no code with the HIP library and the HIP library never
 * calls it.
 *
 * What it computes: the plain definition of scaled-dot-product attention
 * (paper Sec. 2.1, Eq. 1), applied to ONE head whose key/value sequence has
 * already been assembled by the caller as the concatenation of that head's
 * selected history frames followed by the current chunk (paper Sec. 2.2, Eq. 2;
 * per-head effective length, Sec. 4.3 "Ragged-Cache Attention").
 *
 *   s_j   = scale * sum_d q[i][d] * K[j][d]
 *   p_j   = exp(s_j - max_j s_j) / sum_j exp(s_j - max_j s_j)
 *   out_i = sum_j p_j * V[j][:]
 *
 * Inputs are float32 (bf16-rounded values widened by the caller), every sum is
 * carried in double, the result is rounded once to float32.  No tiling, no
 * running-max recurrence, no reordering: three nested loops per query row.
 */
#include <math.h>
#include <stdlib.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int pfo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * q     [n_q_total][D]   queries of this head
 * K, V  [Lkv][D]         this head's assembled key / value sequence
 * rows  [n_rows] or NULL query-row indices to evaluate (NULL = rows 0..n_rows-1)
 * out   [n_rows][D]      row r of out is attention of query rows[r]
 * w_out [n_rows][Lkv] or NULL: softmax weights p_j (for the "rows sum to one" pin)
 * returns 0, or -1 on a bad argument.
 */
int pfo_attn_head(const float *q, const float *K, const float *V,
                  const int32_t *rows, int n_rows, int Lkv, int D,
                  double scale, float *out, double *w_out)
{
    if (!q || !K || !V || !out || n_rows < 0 || Lkv < 1 || D < 1) return -1;
    int fail = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)Lkv);
        double *acc = (double *)malloc(sizeof(double) * (size_t)D);
        if (!s || !acc) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(dynamic, 4)
            for (int r = 0; r < n_rows; ++r) {
                const int i = rows ? rows[r] : r;
                const float *qi = q + (size_t)i * D;
                double smax = -INFINITY;
                for (int j = 0; j < Lkv; ++j) {
                    const float *kj = K + (size_t)j * D;
                    double dot = 0.0;
                    for (int d = 0; d < D; ++d) dot += (double)qi[d] * (double)kj[d];
                    s[j] = scale * dot;
                    if (s[j] > smax) smax = s[j];
                }
                double denom = 0.0;
                for (int j = 0; j < Lkv; ++j) {
                    s[j] = exp(s[j] - smax);
                    denom += s[j];
                }
                for (int d = 0; d < D; ++d) acc[d] = 0.0;
                for (int j = 0; j < Lkv; ++j) {
                    const double p = s[j] / denom;
                    const float *vj = V + (size_t)j * D;
                    for (int d = 0; d < D; ++d) acc[d] += p * (double)vj[d];
                    if (w_out) w_out[(size_t)r * Lkv + j] = p;
                }
                for (int d = 0; d < D; ++d) out[(size_t)r * D + d] = (float)acc[d];
            }
        }
        free(s);
        free(acc);
    }
    return fail ? -1 : 0;
}
