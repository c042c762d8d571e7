/*
 * TEST INFRASTRUCTURE ONLY -- see layer_ops_impl.h.  Builds the CPU oracle's
 * layer operations in two precisions: _f64 (the reference values) and _f32
 * (to show how reconstruction error behaves in the paper's float32 setting,
 * Section 3.2 "Numerical error").
 *
 *   gcc -O2 -fopenmp -shared -fPIC layer_ops.c -o liboracle_layer_ops.so -lm
 */
#include <math.h>
#include <stddef.h>

#define REAL double
#define FN(name) name##_f64
#include "layer_ops_impl.h"
#undef REAL
#undef FN

#define REAL float
#define FN(name) name##_f32
#include "layer_ops_impl.h"
#undef REAL
#undef FN

#ifdef _OPENMP
#include <omp.h>
int orc_num_threads(void) { return omp_get_max_threads(); }
#else
int orc_num_threads(void) { return 1; }
#endif
