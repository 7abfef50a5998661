/* CPU oracle for the truly sparse MLP training step (CSR weights, dense batches).
 *
 * TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's CPU-baseline leg
 * call it; the HIP library never does and shares no code with it.
 *
 * Plain loops that write out the definitions of the four sparse operations of Section 4
 * (A = S B, A = S^T B, S = A B^T on S's pattern, S = alpha S + beta T), the ReLU of
 * Section 5.1 and the softmax cross-entropy of the Appendix B listing.  fp64 accumulation
 * everywhere; the _f32 entry points store fp32, the _f64 entry points store fp64 (used for
 * finite differences).
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC sparse_mlp_oracle.c -o libsparse_mlp_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define REAL float
#define FN(x) x##_f32
#include "sparse_mlp_oracle_impl.inc"
#undef REAL
#undef FN

#define REAL double
#define FN(x) x##_f64
#include "sparse_mlp_oracle_impl.inc"
#undef REAL
#undef FN

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
