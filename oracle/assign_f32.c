/* TEST INFRASTRUCTURE ONLY -- CPU oracle for the k-means assignment step.
 *
 * The paper clusters Q and K with k-means (Methodology, "Problem Formulation") and fixes
 * neither the metric nor the arithmetic. This oracle takes squared Euclidean distance
 * (the clustering error of Proposition 1 is an l2 error and centroids are cluster means)
 * and evaluates it in a single fixed fp32 order so that the integer label it decides is
 * reproducible bit for bit by any implementation that follows the same order:
 *
 *   dot   = 0;  for t = 0..d-1:  dot = fma(x[t], c[t], dot)
 *   cn    = 0;  for t = 0..d-1:  cn  = fma(c[t], c[t], cn)
 *   score = fma(-2, dot, cn)            (||x||^2 is the same for every centroid: dropped)
 *   label = lowest index attaining the minimum score (strict '<' while scanning upward)
 *
 * Build with -ffp-contract=off: every rounding below is an explicit fmaf.
 * Nothing in the HIP library includes, links or calls this file.
 */
#include <math.h>
#include <stdint.h>

void svgear_oracle_assign_f32(const float* x, int64_t n, int d, const float* c, int C,
                              int32_t* labels, float* best_score) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    const float* xi = x + i * (int64_t)d;
    float best = INFINITY;
    int32_t arg = 0;
    for (int j = 0; j < C; ++j) {
      const float* cj = c + (int64_t)j * d;
      float dot = 0.0f, cn = 0.0f;
      for (int t = 0; t < d; ++t) dot = fmaf(xi[t], cj[t], dot);
      for (int t = 0; t < d; ++t) cn = fmaf(cj[t], cj[t], cn);
      float score = fmaf(-2.0f, dot, cn);
      if (j == 0 || score < best) {
        best = score;
        arg = j;
      }
    }
    labels[i] = arg;
    if (best_score) best_score[i] = best;
  }
}

int svgear_oracle_max_threads(void) {
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  return omp_get_max_threads();
#else
  return 1;
#endif
}
