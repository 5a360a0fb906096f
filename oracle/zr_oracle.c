/*
 * CPU oracle, native part: a plain dense matrix product in float64.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this; it
 * shares no code with the HIP library.
 *
 * The resized linear layer multiplies *pruned* matrices exactly as a normal
 * linear layer multiplies full ones (paper Sec. 3.1, "Overview Resizing
 * Design"): the only arithmetic is an ordinary matrix product.  The pruning
 * (extracting the kept slices in ascending index order) and the recovery
 * (placing results back, imputing the missing slices) are done by the Python
 * part of the oracle around this routine.
 *
 * C[I x J] = A[I x Kc] * B[Kc x J], all row-major, contiguous, float64.
 * Textbook triple loop in i-k-j order (each C row accumulates its Kc
 * contributions in ascending k), rows distributed over OpenMP threads.
 * No blocking, no reordering beyond that.  Built with FP contraction off.
 */
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

void zro_matmul_f64(const double* A, const double* B, double* C,
                    int64_t I, int64_t Kc, int64_t J)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < I; ++i) {
        double* c = C + (size_t)i * (size_t)J;
        for (int64_t j = 0; j < J; ++j) c[j] = 0.0;
        for (int64_t k = 0; k < Kc; ++k) {
            const double a = A[(size_t)i * (size_t)Kc + (size_t)k];
            const double* b = B + (size_t)k * (size_t)J;
            for (int64_t j = 0; j < J; ++j) c[j] += a * b[j];
        }
    }
}

/* Number of threads the matmul above runs on (reported beside its timing). */
int zro_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Kept count L*(1-gamma) (Algorithm 1, the L_pri line), rounded half-up to an
 * integer in IEEE double: floor((1-ratio)*n + 0.5). */
int64_t zro_keep_count(int64_t n, double ratio)
{
    volatile double kept = (1.0 - ratio) * (double)n;
    volatile double shifted = kept + 0.5;
    int64_t r = (int64_t)shifted;      /* shifted >= 0 here: truncation == floor */
    if ((double)r > shifted) --r;
    return r;
}
