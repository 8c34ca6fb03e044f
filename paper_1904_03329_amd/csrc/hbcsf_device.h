// Kernel argument block and launch entry points shared by the kernels and the C-ABI layer.
#ifndef HBCSF_DEVICE_H_
#define HBCSF_DEVICE_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hbcsf {

enum KernelKind { kCooKernel = 0, kCslKernel = 1, kCsfKernel = 2 };

// The B-CSF kernel's dense fiber-row gather: rows its per-wavefront LDS cache holds, the instantiations that
// exist (rank 32, orders 3 and 4, runs of 32 or 64 nonzeros), and the LDS bytes it adds per wavefront.
constexpr int kDenseCacheRows = 32;
inline bool dense_mid_available(int order, int G, uint32_t lshift) {
  return G == 8 && (order == 3 || order == 4) && (lshift == 5 || lshift == 6);
}
inline size_t dense_mid_lds_bytes(int G) { return 256 + (size_t)kDenseCacheRows * 16 * (size_t)G; }

// Device pointers of one slice group of one mode, by tree level (0 = root .. order-1 = leaf).
struct GroupArgs {
  const uint32_t* ind[5];       // index arrays (per slice / segment / nonzero, by group kind)
  const uint32_t* ptr[5];       // starts in the group's nonzero stream (n+1 entries)
  const uint32_t* runFirst[5];  // slice / segment holding the first nonzero of each run
  const float* val;             // values in stream order
  const float* fac[5];          // factor matrix of each tree level (fac[0] unused)
  float* out;                   // [rows][rank]
  uint32_t nnz;                 // nonzeros in the group
  uint32_t runs;                // ceil(nnz / L)
  uint32_t lshift;              // log2 L
  uint32_t nUnits;              // ceil(runs / lane groups per wavefront)
  uint32_t unitsPerWave;        // consecutive units in one span
  uint32_t nSpans;              // ceil(nUnits / unitsPerWave)
  uint32_t streamLevel;         // bit l: the factor rows of fiber level l are gathered with streaming loads
  uint32_t persistent;          // 1: resident wavefronts take spans round-robin; 0: one wavefront per span
  uint32_t denseMid;            // B-CSF kernel: 1 = fiber-level rows gathered once per block of steps for the whole
                                // wavefront through an LDS row cache (needs dense_mid_available and its LDS size)
  // Optional wavefront trace (profiling only, nullptr = off): trace[0] counts records; record i
  // is the four words at trace[4 + 4 i]: {kernel kind, XCC_ID << 32 | HW_ID, start, end} with
  // start / end from the constant-rate wall clock.
  unsigned long long* trace;
  uint32_t traceCapacity;       // records the buffer can hold
};

// kind: KernelKind; order 3, 4 or 5; G = row bytes / 16 lanes per factor row (fp32: rank / 4 = 2, 4, 8, 16 or 32;
// fp64: rank / 2 = 8, 16 or 32, the launch functions named ...64...);
// steps = records a lane group keeps in flight (4 or 8); wide = some gathered factor matrix
// is 4 GiB or larger (64-bit row addressing).  One launch function per (G, order) pair, each
// compiled in its own object file.  For the CSL and B-CSF kernels `blocks` is the number of compute
// units and the launcher sizes the grid (one wavefront per span, or persistent).
#define HBCSF_DECLARE_LAUNCH(G, N)                                                                  \
  hipError_t launch_group_g##G##_n##N(int kind, int steps, bool wide, const GroupArgs& a,          \
                                      uint32_t blocks, uint32_t threads, size_t ldsBytes, hipStream_t s); \
  hipError_t launch_define_coo_g##G##_n##N(bool wide, const GroupArgs& a, const uint32_t* ownedBits,   \
                                           const uint32_t* cooBits, const uint32_t* cooPtr, uint64_t rows, \
                                           uint32_t blocks, hipStream_t s);
HBCSF_DECLARE_LAUNCH(2, 3)
HBCSF_DECLARE_LAUNCH(4, 3)
HBCSF_DECLARE_LAUNCH(8, 3)
HBCSF_DECLARE_LAUNCH(16, 3)
HBCSF_DECLARE_LAUNCH(32, 3)
HBCSF_DECLARE_LAUNCH(2, 4)
HBCSF_DECLARE_LAUNCH(4, 4)
HBCSF_DECLARE_LAUNCH(8, 4)
HBCSF_DECLARE_LAUNCH(16, 4)
HBCSF_DECLARE_LAUNCH(32, 4)
HBCSF_DECLARE_LAUNCH(2, 5)
HBCSF_DECLARE_LAUNCH(4, 5)
HBCSF_DECLARE_LAUNCH(8, 5)
HBCSF_DECLARE_LAUNCH(16, 5)
HBCSF_DECLARE_LAUNCH(32, 5)
#undef HBCSF_DECLARE_LAUNCH
#define HBCSF_DECLARE_LAUNCH64(G, N)                                                                  \
  hipError_t launch_group64_g##G##_n##N(int kind, int steps, bool wide, const GroupArgs& a,          \
                                        uint32_t blocks, uint32_t threads, size_t ldsBytes, hipStream_t s); \
  hipError_t launch_define_coo64_g##G##_n##N(bool wide, const GroupArgs& a, const uint32_t* ownedBits,   \
                                             const uint32_t* cooBits, const uint32_t* cooPtr, uint64_t rows, \
                                             uint32_t blocks, hipStream_t s);
HBCSF_DECLARE_LAUNCH64(8, 3)
HBCSF_DECLARE_LAUNCH64(16, 3)
HBCSF_DECLARE_LAUNCH64(32, 3)
HBCSF_DECLARE_LAUNCH64(8, 4)
HBCSF_DECLARE_LAUNCH64(16, 4)
HBCSF_DECLARE_LAUNCH64(32, 4)
HBCSF_DECLARE_LAUNCH64(8, 5)
HBCSF_DECLARE_LAUNCH64(16, 5)
HBCSF_DECLARE_LAUNCH64(32, 5)
#undef HBCSF_DECLARE_LAUNCH64

// f64: the factor matrices and the output hold doubles (GroupArgs' float pointers then address doubles).
inline hipError_t launch_group(bool f64, int kind, int order, int G, int steps, bool wide, const GroupArgs& a,
                               uint32_t blocks, uint32_t threads, size_t ldsBytes, hipStream_t s) {
#define HBCSF_CASE64(GV)                                                                              \
  case GV:                                                                                            \
    return order == 3   ? launch_group64_g##GV##_n3(kind, steps, wide, a, blocks, threads, ldsBytes, s) \
           : order == 4 ? launch_group64_g##GV##_n4(kind, steps, wide, a, blocks, threads, ldsBytes, s) \
                        : launch_group64_g##GV##_n5(kind, steps, wide, a, blocks, threads, ldsBytes, s);
  if (f64) {
    switch (G) {
      HBCSF_CASE64(8)
      HBCSF_CASE64(16)
      HBCSF_CASE64(32)
      default:
        return hipErrorInvalidValue;
    }
  }
#undef HBCSF_CASE64
#define HBCSF_CASE(GV)                                                                              \
  case GV:                                                                                          \
    return order == 3   ? launch_group_g##GV##_n3(kind, steps, wide, a, blocks, threads, ldsBytes, s) \
           : order == 4 ? launch_group_g##GV##_n4(kind, steps, wide, a, blocks, threads, ldsBytes, s) \
                        : launch_group_g##GV##_n5(kind, steps, wide, a, blocks, threads, ldsBytes, s);
  switch (G) {
    HBCSF_CASE(2)
    HBCSF_CASE(4)
    HBCSF_CASE(8)
    HBCSF_CASE(16)
    HBCSF_CASE(32)
    default:
      return hipErrorInvalidValue;
  }
#undef HBCSF_CASE
}

// Output definition fused with the COO group (a: the COO group's arguments).
inline hipError_t launch_define_coo(bool f64, int order, int G, bool wide, const GroupArgs& a,
                                    const uint32_t* ownedBits, const uint32_t* cooBits, const uint32_t* cooPtr,
                                    uint64_t rows, uint32_t blocks, hipStream_t s) {
#define HBCSF_CASE64(GV)                                                                                     \
  case GV:                                                                                                   \
    return order == 3   ? launch_define_coo64_g##GV##_n3(wide, a, ownedBits, cooBits, cooPtr, rows, blocks, s) \
           : order == 4 ? launch_define_coo64_g##GV##_n4(wide, a, ownedBits, cooBits, cooPtr, rows, blocks, s) \
                        : launch_define_coo64_g##GV##_n5(wide, a, ownedBits, cooBits, cooPtr, rows, blocks, s);
  if (f64) {
    switch (G) {
      HBCSF_CASE64(8)
      HBCSF_CASE64(16)
      HBCSF_CASE64(32)
      default:
        return hipErrorInvalidValue;
    }
  }
#undef HBCSF_CASE64
#define HBCSF_CASE(GV)                                                                                     \
  case GV:                                                                                                 \
    return order == 3   ? launch_define_coo_g##GV##_n3(wide, a, ownedBits, cooBits, cooPtr, rows, blocks, s) \
           : order == 4 ? launch_define_coo_g##GV##_n4(wide, a, ownedBits, cooBits, cooPtr, rows, blocks, s) \
                        : launch_define_coo_g##GV##_n5(wide, a, ownedBits, cooBits, cooPtr, rows, blocks, s);
  switch (G) {
    HBCSF_CASE(2)
    HBCSF_CASE(4)
    HBCSF_CASE(8)
    HBCSF_CASE(16)
    HBCSF_CASE(32)
    default:
      return hipErrorInvalidValue;
  }
#undef HBCSF_CASE
}

// Zero fill of the rows whose bit in ownedBits is clear; a row is G 16-byte pieces (fp32 or fp64 alike).
hipError_t launch_define(float* out, const uint32_t* ownedBits, uint64_t rows, int G,
                         uint32_t blocks, hipStream_t s);

// Zero fill of nvec float4s (an output that is then only reached by atomic adds).
hipError_t launch_zero_rows(float* out, uint64_t nvec, uint32_t blocks, hipStream_t s);

// Single-representation kernels (rank 32): the target mode is at tree level `level` >= 1 of the representation
// whose B-CSF group `a` describes (fac[l] set for every level but `level`, fac[0] included).
hipError_t launch_nonroot_n3(int level, bool wide, const GroupArgs& a, uint32_t threads, size_t ldsBytes, hipStream_t s);
hipError_t launch_nonroot_n4(int level, bool wide, const GroupArgs& a, uint32_t threads, size_t ldsBytes, hipStream_t s);
hipError_t launch_nonroot_n5(int level, bool wide, const GroupArgs& a, uint32_t threads, size_t ldsBytes, hipStream_t s);

// Diagnostic row-gather probe: `waves` (a multiple of 4) wavefronts, each walking `perWave`
// (a multiple of 64) entries of idx (row numbers of a table of 32-float rows); `active` (1..8) of a
// wavefront's 8 lane groups take part in each load instruction.
hipError_t launch_probe_gather(const uint32_t* idx, uint64_t n, const float* table, float* sink,
                               uint32_t waves, uint32_t perWave, int active, hipStream_t s);

}  // namespace hbcsf

#endif  // HBCSF_DEVICE_H_
