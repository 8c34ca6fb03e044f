/* TEST INFRASTRUCTURE ONLY -- the plain CPU oracle for mode-n sparse MTTKRP.
 *
 * Nothing in the product path may call, link or import this file.  It is used
 * by the tests, by the smoke check and by the benchmark's CPU-baseline leg.
 * It shares no code with the GPU library.
 *
 * What it computes (Section II-C, Eq. 4-7; Algorithm "COO-MTTKRP", Section
 * III-A): the hybrid balanced CSF method reaches exactly the plain MTTKRP
 * result (it changes storage and scheduling only; Eq. 7 equals Eq. 8), so the
 * oracle is the plain definition written out, generalised from three modes to
 * N modes and from mode 1 to any target mode n as Section II-C says it can be:
 *
 *   for every stored nonzero z with coordinates (i_1..i_N) and value v:
 *     for r in 0..R-1:
 *       M[i_n][r] += (double)v * prod_{m != n} (double)A_m[i_m][r]
 *
 * M is fp64 and starts at zero; nonzeros are visited in input order; duplicate
 * coordinates are separate nonzeros and simply add up.  Indices are 0-based
 * uint32, values and factor matrices fp32 (Section V-A), factor matrices are
 * row-major [dims[m]][R] (inputs of Algorithm "COO-MTTKRP").
 *
 * oracle_mttkrp_f64 is the same sum with fp64 factor matrices (nothing is
 * widened but the value), the reference for the library's fp64 entry point.
 *
 * Pins (tests/test_oracle_pins.py): dense matricised-tensor times explicit
 * Khatri-Rao product (Eq. 4-5) on tiny tensors, the rank-1 closed form, the
 * cross-mode invariant sum(M^(n) * A_n), nonzero-order and partition
 * invariance, and the sparse-matrix special case K = 1 against scipy.
 */
#include <stdint.h>
#include <stddef.h>

#define ORACLE_MAX_ORDER 8

/* Full result.  out: [dims[mode]][rank] fp64, overwritten.
 * Returns 0, -1 on a bad argument, -2 if an index is out of range. */
int oracle_mttkrp(int order, const uint64_t *dims, uint64_t nnz,
                  const uint32_t *const *inds, const float *vals, int rank,
                  const float *const *factors, int mode, double *out)
{
    if (order < 2 || order > ORACLE_MAX_ORDER || mode < 0 || mode >= order || rank < 1) return -1;
    if (!dims || !inds || !vals || !factors || !out) return -1;
    const uint64_t rows = dims[mode];
    for (uint64_t t = 0; t < rows * (uint64_t)rank; ++t) out[t] = 0.0;
    for (uint64_t z = 0; z < nnz; ++z) {
        for (int m = 0; m < order; ++m)
            if (inds[m][z] >= dims[m]) return -2;
        double *y = out + (uint64_t)inds[mode][z] * (uint64_t)rank;
        const double v = (double)vals[z];
        for (int r = 0; r < rank; ++r) {
            double p = v;
            for (int m = 0; m < order; ++m) {
                if (m == mode) continue;
                p *= (double)factors[m][(uint64_t)inds[m][z] * (uint64_t)rank + (uint64_t)r];
            }
            y[r] += p;
        }
    }
    return 0;
}

/* The same sum restricted to chosen output rows, for checking sampled rows of
 * results too large to hold in fp64 on the host.  slot_of_row[i] is the row of
 * `out` that receives M[i][:], or -1 to skip row i.  out: [nslots][rank]. */
int oracle_mttkrp_rows(int order, const uint64_t *dims, uint64_t nnz,
                       const uint32_t *const *inds, const float *vals, int rank,
                       const float *const *factors, int mode,
                       const int32_t *slot_of_row, uint64_t nslots, double *out)
{
    if (order < 2 || order > ORACLE_MAX_ORDER || mode < 0 || mode >= order || rank < 1) return -1;
    if (!dims || !inds || !vals || !factors || !out || !slot_of_row) return -1;
    for (uint64_t t = 0; t < nslots * (uint64_t)rank; ++t) out[t] = 0.0;
    for (uint64_t z = 0; z < nnz; ++z) {
        const uint32_t i = inds[mode][z];
        if (i >= dims[mode]) return -2;
        const int32_t slot = slot_of_row[i];
        if (slot < 0) continue;
        if ((uint64_t)slot >= nslots) return -1;
        for (int m = 0; m < order; ++m)
            if (inds[m][z] >= dims[m]) return -2;
        double *y = out + (uint64_t)slot * (uint64_t)rank;
        const double v = (double)vals[z];
        for (int r = 0; r < rank; ++r) {
            double p = v;
            for (int m = 0; m < order; ++m) {
                if (m == mode) continue;
                p *= (double)factors[m][(uint64_t)inds[m][z] * (uint64_t)rank + (uint64_t)r];
            }
            y[r] += p;
        }
    }
    return 0;
}

/* The same definition with fp64 factor matrices: M[i_n][r] += (double)v * prod_{m != n} A_m[i_m][r]. */
int oracle_mttkrp_f64(int order, const uint64_t *dims, uint64_t nnz,
                      const uint32_t *const *inds, const float *vals, int rank,
                      const double *const *factors, int mode, double *out)
{
    if (order < 2 || order > ORACLE_MAX_ORDER || mode < 0 || mode >= order || rank < 1) return -1;
    if (!dims || !inds || !vals || !factors || !out) return -1;
    const uint64_t rows = dims[mode];
    for (uint64_t t = 0; t < rows * (uint64_t)rank; ++t) out[t] = 0.0;
    for (uint64_t z = 0; z < nnz; ++z) {
        for (int m = 0; m < order; ++m)
            if (inds[m][z] >= dims[m]) return -2;
        double *y = out + (uint64_t)inds[mode][z] * (uint64_t)rank;
        const double v = (double)vals[z];
        for (int r = 0; r < rank; ++r) {
            double p = v;
            for (int m = 0; m < order; ++m) {
                if (m == mode) continue;
                p *= factors[m][(uint64_t)inds[m][z] * (uint64_t)rank + (uint64_t)r];
            }
            y[r] += p;
        }
    }
    return 0;
}
