/* CPU oracle for the DaSGD parameter pipeline (Local SGD with delayed averaging, Eq. 2 of the
 * paper): the iteration written out step by step in plain C, in fp64 (reference) and in fp32
 * (the precision the paper's gradients and the GPU path use).
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing here is shared with, included by, or called from the GPU
 * library; only the test-suite, the smoke check and the benchmark's CPU-baseline leg use it.
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC (no fast-math, no contraction, so
 * every operation is rounded once, in the order written).
 *
 * What pins it to something other than itself (tests/oracle_pins.py; each pin must also catch at
 * least one of the mistakes planted by tests/test_oracle_mutants.py):
 *   local update   torch.optim.SGD with momentum and weight decay, incl. a learning-rate change
 *   mean           numpy's fp64 mean; identical rows at power-of-two W come back bit-exactly
 *   merge          hand-worked dyadic example; spread around the replica mean shrinks by exactly xi
 *   step (the iteration, launch and merge steps, FIFO of pending averages)
 *                  hand-worked example; special cases that reduce to plain SGD, to mini-batch SGD
 *                  and to Local SGD built from library routines; the paper's recursion for the
 *                  averaged model; its matrix form as a matrix product; the closed form of the
 *                  noise-free quadratic; the appendix trigger for the launch and merge steps
 * No function is unpinned.  The paper prints no numerical value for whole runs of the benchmark
 * configurations (random gradients, d >= tau): as wholes those are parity unpinned by the paper.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define REAL float
#define NAME(x) x##_f32
#include "dasgd_oracle_impl.h"
#undef REAL
#undef NAME

#define REAL double
#define NAME(x) x##_f64
#include "dasgd_oracle_impl.h"
#undef REAL
#undef NAME

/* Threads used by the elementwise loops (results do not depend on it: every element is
 * independent and the order over replicas is fixed).  Returns the count in effect. */
int dasgd_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
    return omp_get_max_threads();
#else
    (void)n;
    return 1;
#endif
}
