/* CPU oracle for structured-grid weighted sums (2D and 3D filter, 2D/3D stencil, Jacobi iteration, scan).
 *
 * TEST INFRASTRUCTURE ONLY: a plain, slow, obviously-correct evaluation of the definitions
 * in Sec. 2.1 and Sec. 2.2 of the paper, used by the tests, by the smoke check and as the
 * timed CPU baseline of the benchmark.  It shares no code, header, table or helper with the
 * GPU library and must never be called from the product path.
 *
 * Precision: float grids are summed in double (every product of two floats is exact in
 * double), double grids in long double (64-bit significand on x86-64); one rounding to the
 * working type per output.  The sum therefore sits within half an ulp or so of the exact
 * value and a GPU result is compared against (nearly) the truth, not against another
 * summation order.
 *
 * The loops over rows are split over OpenMP threads when built with -fopenmp; points are
 * independent, so threading changes no value.
 *
 * Pins (tests/test_oracle_pins.py): exact rational brute force on tiny grids, delta input,
 * constant and linear fields, hand-worked five-point example, scipy.ndimage / torch
 * cross-checks (also with explicit origins / anchors in 3D), separable filters, iteration identities.
 * No function here is unpinned.
 */
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_ZERO = 0, ORACLE_CLAMP = 1 };

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

#define T float
#define ACC double
#define FN(name) name##_f32
#include "ssam_oracle_body.inc"
#undef T
#undef ACC
#undef FN

#define T double
#define ACC long double
#define FN(name) name##_f64
#include "ssam_oracle_body.inc"
#undef T
#undef ACC
#undef FN
