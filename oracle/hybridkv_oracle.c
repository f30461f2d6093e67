/*
 * TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.
 *
 * CPU oracle of the hybrid-cache decode step (LayerNorm -> K/V projection of
 * the activation checkpoints -> concatenation with the cached K/V -> softmax
 * attention for one decode query).  The arithmetic lives in
 * hybridkv_oracle_impl.h; this file instantiates it in fp64 (symbols *_f64,
 * the reference the GPU path is compared with) and in fp32 (symbols *_f32,
 * the plain single-precision CPU baseline that the bench times).
 *
 * Build: gcc -O2 -fopenmp -fPIC -shared hybridkv_oracle.c -o libhybridkv_oracle.so -lm
 * (-O2 without -ffast-math: no reassociation, the sums run in index order.)
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define REAL double
#define SUFFIX _f64
#define HKO_SQRT sqrt
#define HKO_EXP exp
#define HKO_INF ((double)INFINITY)
#include "hybridkv_oracle_impl.h"
#undef REAL
#undef SUFFIX
#undef HKO_SQRT
#undef HKO_EXP
#undef HKO_INF

#define REAL float
#define SUFFIX _f32
#define HKO_SQRT sqrtf
#define HKO_EXP expf
#define HKO_INF ((float)INFINITY)
#include "hybridkv_oracle_impl.h"
#undef REAL
#undef SUFFIX
#undef HKO_SQRT
#undef HKO_EXP
#undef HKO_INF

/* Number of threads the OpenMP loops above will use (1 without OpenMP). */
int hko_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
