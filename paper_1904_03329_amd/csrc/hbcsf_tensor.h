// The tensor handle behind the C ABI, shared by the translation units that implement its entry points.
#pragma once

#include <hip/hip_runtime.h>

#include <memory>
#include <string>
#include <vector>

#include "hbcsf.h"
#include "hbcsf_internal.h"

struct hbcsf_tensor {
  int order = 0;
  uint64_t dims[HBCSF_MAX_ORDER] = {};
  uint64_t nnz = 0;
  double normSq = 0.0;  // sum of the squared values (for the CPD fit)
  hbcsf_opts opts{};
  std::unique_ptr<hbcsf::ModeFormat> modes[HBCSF_MAX_ORDER];
  uint64_t arenaBytes = 0;
  uint8_t* arena = nullptr;  // caller's device memory
  bool uploaded = false;
  bool single = false;       // only modes[0] exists; the other modes are computed from it (single representation)
  int numCU = 256;
  uint64_t sliceThreshold = 0;
  uint64_t wavesPerCU = 0;   // launch sizing override, 0 = default
  int steps = 8;             // records in flight per lane group
  uint32_t kernelMask = 15;  // bit0 define, bit1 COO, bit2 CSL, bit3 CSF
  bool persistent = false;   // resident wavefronts walk the spans round-robin
  int denseMid = 0;          // B-CSF fiber-row gather through an LDS row cache (tuning variant): 0 off, 1 on
  int fuseCoo = 2;           // COO-group rows written by the output-definition pass: 0 never, 1 always, 2 small outputs
  uint64_t streamBytes = 1ull << 30;  // fiber-level factors at least this large are gathered with streaming loads
  unsigned long long* trace = nullptr;  // caller's device buffer for wavefront traces
  uint64_t traceCapacity = 0;
  // profiling: a ring of event sets, one per hbcsf_mttkrp call
  struct EventSet {
    hipEvent_t ev[5];
    bool launched[4] = {false, false, false, false};
    bool valid = false;
  };
  // hbcsf_mttkrp takes a const handle; recording a profiled call is bookkeeping, not state of the tensor
  mutable std::vector<EventSet> ring;
  mutable uint64_t calls = 0;  // profiled calls so far
};

namespace hbcsf {

// Records the message hbcsf_last_error returns on this thread and passes the code through.
int fail(int code, const std::string& msg);
int fail_hip(hipError_t e, const char* what);
// For the handler of an entry point's function-try-block: turns the exception in flight into an error code
// (std::bad_alloc -> HBCSF_ENOMEM, anything else -> HBCSF_EINVAL with its text) and never throws itself.
int fail_exception() noexcept;

}  // namespace hbcsf

// Every entry point that returns an error code is a function-try-block closed by this handler, so that no C++
// exception (a failed allocation in a container, above all) crosses the C boundary.
#define HBCSF_CATCH_ALL catch (...) { return hbcsf::fail_exception(); }
