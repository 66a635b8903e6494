/*
 * CPU oracle for the per-GPU ResNet-50 SGD iteration -- TEST INFRASTRUCTURE ONLY.
 * Built by oracle/build.py into oracle/librn50_oracle.so; only tests, the smoke
 * check and the benchmark's cpu_baseline leg load it.  It shares no code with
 * the HIP library.  Every function exists in an fp32 (_f32) and an fp64 (_f64)
 * instantiation of the same plain text in rn50_oracle_impl.inc.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>

/* Nearest IEEE-754 binary16 value of v, ties to even, returned as a double.
 * binary16: 10 fraction bits, normal exponents -14..15, subnormal quantum 2^-24,
 * largest finite value 65504; anything that rounds above it becomes infinity.
 * rint() rounds to nearest-even in the default floating-point environment.      */
double oracle_round_binary16(double v)
{
    if (isnan(v) || isinf(v) || v == 0.0) return v;
    const double a = fabs(v);
    int e;
    (void)frexp(a, &e);          /* a = m * 2^e with m in [0.5, 1): leading bit has weight 2^(e-1) */
    int lead = e - 1;
    if (lead < -14) lead = -14;  /* subnormals share the quantum of the smallest normal binade */
    const double quantum = ldexp(1.0, lead - 10);
    double r = rint(a / quantum) * quantum;
    if (r > 65504.0) r = INFINITY;
    return copysign(r, v);
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Number of OpenMP threads later calls use (timing aid for the benchmark's CPU leg; no effect on results). */
void oracle_set_threads(int n)
{
#ifdef _OPENMP
    extern void omp_set_num_threads(int);
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

#define REAL float
#define FN(name) name##_f32
#include "rn50_oracle_impl.inc"
#undef REAL
#undef FN

#define REAL double
#define FN(name) name##_f64
#include "rn50_oracle_impl.inc"
#undef REAL
#undef FN
