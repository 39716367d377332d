/*
 * CPU oracle: see dll_oracle.h.  TEST INFRASTRUCTURE ONLY; shares nothing with the
 * GPU library.  Build: gcc -O2 -fopenmp -shared -fPIC dll_oracle.c -lm
 */
#include "dll_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* Shape rules: positive sizes, the padded input at least as large as the filter,
 * pad no larger than the filter allows for a well-defined full convolution, and an
 * even pre-pool map when 2x2 pooling is on. */
static int oracle_desc_ok(const oracle_conv_desc *d) {
  if (!d) return 0;
  if (d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0) return 0;
  if (d->pad < 0 || d->pad > d->R - 1 || d->pad > d->S - 1) return 0;
  const int Ho = d->H + 2 * d->pad - d->R + 1, Wo = d->W + 2 * d->pad - d->S + 1;
  if (Ho <= 0 || Wo <= 0) return 0;
  if (d->act < ORACLE_ACT_IDENTITY || d->act > ORACLE_ACT_RELU) return 0;
  if (d->pool != 1 && d->pool != 2) return 0;
  if (d->pool == 2 && ((Ho & 1) || (Wo & 1))) return 0;
  return 1;
}

#define REAL float
#define FN(name) oracle_##name
#include "dll_oracle_core.inc"
#undef REAL
#undef FN

#define REAL double
#define FN(name) oracle64_##name
#include "dll_oracle_core.inc"
#undef REAL
#undef FN
