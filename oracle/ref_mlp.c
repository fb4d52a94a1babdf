/*
 * CPU oracle for the one-hidden-layer MLP gradient (paper section 4.2, with a softmax / cross-entropy
 * output stage).  TEST INFRASTRUCTURE ONLY: see ref_mlp_body.inc for what is computed and the citations.
 *
 * The body is compiled twice:
 *   ref_mlp_grad_f64 / ref_mlp_loss_f64   every operation in double: the reference value for parity (fed
 *                                         the fp32 inputs widened exactly) and for finite differences
 *   ref_mlp_grad_f32 / ref_mlp_loss_f32   every operation in float, the paper's precision (section 4.2
 *                                         reports 32 bits to be enough): the timed CPU baseline
 * Only tests, the smoke check and the bench's cpu_baseline leg may use this file.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#define REAL double
#define FN(name) name##_f64
#define R_TANH tanh
#define R_EXP exp
#define R_LOG log
#include "ref_mlp_body.inc"
#undef REAL
#undef FN
#undef R_TANH
#undef R_EXP
#undef R_LOG

#define REAL float
#define FN(name) name##_f32
#define R_TANH tanhf
#define R_EXP expf
#define R_LOG logf
#include "ref_mlp_body.inc"
#undef REAL
#undef FN
#undef R_TANH
#undef R_EXP
#undef R_LOG

/* Number of threads the `omp parallel for` loops use (reported beside the timed baseline). */
#ifdef _OPENMP
#include <omp.h>
int ref_threads(void) { return omp_get_max_threads(); }
#else
int ref_threads(void) { return 1; }
#endif
