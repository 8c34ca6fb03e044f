// Internal layout shared by the host format builder and the device launch code.
#ifndef HBCSF_INTERNAL_H_
#define HBCSF_INTERNAL_H_

#include <cstdint>
#include <cstdlib>
#include <string>
#include <vector>

#include "hbcsf.h"

namespace hbcsf {

enum Group { kCoo = 0, kCsl = 1, kCsf = 2 };

constexpr uint32_t kOwnedBit = 0x80000000u;  // in a slice index: the slice lies inside one run
constexpr uint64_t kAlign = 256;             // every device array starts on a 256-byte boundary

struct ArrayRef {
  uint64_t off = 0;    // byte offset inside the mode's blob
  uint64_t count = 0;  // elements (4 bytes each)
  bool present = false;
};

// One slice group of one mode.  Levels: 0 = root (slices) .. order-1 = leaf (nonzeros).
//   COO : ind[0..order-1] per nonzero, val.
//   CSL : ind[0] per slice (+ owned bit), ptr[0] -> nonzeros, ind[1..order-1] per nonzero, val,
//         runFirst[0].
//   CSF : ind[l] / ptr[l] / runFirst[l] per slice (l = 0) or fiber segment (0 < l < order-1),
//         every ptr indexes the group's nonzero stream; ind[order-1] per nonzero, val.
struct GroupFormat {
  uint64_t nnz = 0;
  uint64_t n[HBCSF_MAX_ORDER] = {0, 0, 0, 0};  // entries per level above the leaf
  uint64_t runs = 0;                           // ceil(nnz / L)
  ArrayRef ind[HBCSF_MAX_ORDER];
  ArrayRef ptr[HBCSF_MAX_ORDER];
  ArrayRef runFirst[HBCSF_MAX_ORDER];
  ArrayRef val;
};

struct ModeFormat {
  int order = 0;
  int mode = 0;
  uint32_t L = 64;                 // run length = fiber threshold T_f
  int levelMode[HBCSF_MAX_ORDER] = {0, 0, 0, 0};
  uint64_t rows = 0;               // dims[mode]
  GroupFormat g[3];
  ArrayRef ownedBits;
  ArrayRef cooBits;                // bitmap over output rows: 1 = the row belongs to a COO-group slice
  ArrayRef cooPtr;                 // COO-group nonzeros before each 32-row word (words + 1 entries)
  uint8_t* blob = nullptr;         // host copy of all arrays, kAlign-aligned
  uint64_t blobBytes = 0;
  uint64_t devOffset = 0;          // where the blob sits in the device arena
  hbcsf_stats stats{};

  ModeFormat() = default;
  ModeFormat(const ModeFormat&) = delete;
  ModeFormat& operator=(const ModeFormat&) = delete;
  ~ModeFormat() { std::free(blob); }
};

// Builds one mode's representation.  Returns HBCSF_OK or an error code and fills `err`.
int build_mode(int order, const uint64_t* dims, uint64_t nnz, const uint32_t* const* inds,
               const float* vals, const hbcsf_opts& opts, int mode, ModeFormat* out,
               std::string* err);

}  // namespace hbcsf

#endif  // HBCSF_INTERNAL_H_
