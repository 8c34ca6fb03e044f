/* TEST INFRASTRUCTURE ONLY -- the plain CPU oracle's loop on all host cores, for the benchmark's
 * reported CPU baseline.
 *
 * Nothing in the product path may call, link or import this file.  It is NOT the parity
 * reference (mttkrp_oracle.c, single thread, fixed summation order, is): this file exists so that
 * the benchmark can also say what the same plain loop does when every host core works on it.
 *
 * Same definition (Section II-C, Eq. 4-7; Algorithm "COO-MTTKRP", Section III-A, whose parallel
 * form "needs atomic operations" as that section says): the loop over the stored nonzeros is split
 * over the threads and every fp64 add into M is an atomic update, so the result equals the
 * single-thread oracle's up to the order of the fp64 additions.
 *
 * Pin (tests/test_oracle_pins.py): equal to oracle_mttkrp within fp64 summation-order noise.
 */
#include <stdint.h>
#include <stddef.h>
#include <omp.h>

#define ORACLE_MAX_ORDER 8

/* out: [dims[mode]][rank] fp64, overwritten.  threads_used receives the team size.
 * Returns 0, -1 on a bad argument, -2 if an index is out of range. */
int oracle_mttkrp_omp(int order, const uint64_t *dims, uint64_t nnz,
                      const uint32_t *const *inds, const float *vals, int rank,
                      const float *const *factors, int mode, double *out, int *threads_used)
{
    if (order < 2 || order > ORACLE_MAX_ORDER || mode < 0 || mode >= order || rank < 1) return -1;
    if (!dims || !inds || !vals || !factors || !out) return -1;
    const uint64_t rows = dims[mode];
    int bad = 0, team = 1;
#pragma omp parallel
    {
#pragma omp single
        team = omp_get_num_threads();
#pragma omp for schedule(static)
        for (uint64_t t = 0; t < rows * (uint64_t)rank; ++t) out[t] = 0.0;
#pragma omp for schedule(static)
        for (uint64_t z = 0; z < nnz; ++z) {
            int ok = 1;
            for (int m = 0; m < order; ++m)
                if (inds[m][z] >= dims[m]) ok = 0;
            if (!ok) {
#pragma omp atomic write
                bad = 1;
                continue;
            }
            double *y = out + (uint64_t)inds[mode][z] * (uint64_t)rank;
            const double v = (double)vals[z];
            for (int r = 0; r < rank; ++r) {
                double p = v;
                for (int m = 0; m < order; ++m) {
                    if (m == mode) continue;
                    p *= (double)factors[m][(uint64_t)inds[m][z] * (uint64_t)rank + (uint64_t)r];
                }
#pragma omp atomic
                y[r] += p;
            }
        }
    }
    if (threads_used) *threads_used = team;
    return bad ? -2 : 0;
}
