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
  uint64_t n[HBCSF_MAX_ORDER] = {};            // entries per level above the leaf
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
  bool cooRowFlags = false;        // the COO group has no root index array (rows come from cooBits / cooPtr)
  int blockBits = 0;               // level-1 blocking: a slice is stored as one piece per block, none owns its row
  int levelMode[HBCSF_MAX_ORDER] = {};
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

// Places every array of one mode in its blob, given the group sizes; both format builders (host and
// device) call this, so the two produce the same byte layout.  gS / gM: slices and nonzeros per group;
// nSeg: fiber segments of the CSF group per fiber level.  Sets out->blobBytes.
inline void layout_mode(ModeFormat* out, int N, const uint64_t gS[3], const uint64_t gM[3],
                        const uint64_t nSeg[HBCSF_MAX_FIBER_LEVELS]) {
  uint64_t bytes = 0;
  auto add = [&bytes](uint64_t count) {
    ArrayRef r;
    r.off = bytes;
    r.count = count;
    r.present = true;
    bytes += ((count * 4 + kAlign - 1) / kAlign) * kAlign;
    if (count == 0) bytes += kAlign;
    return r;
  };
  const uint32_t L = out->L;
  for (int g = 0; g < 3; ++g) {
    out->g[g].nnz = gM[g];
    out->g[g].runs = (gM[g] + L - 1) / L;
  }
  {
    GroupFormat& G = out->g[kCoo];
    for (int l = 0; l < N; ++l) G.ind[l] = add(l == 0 && out->cooRowFlags ? 0 : G.nnz);
    G.val = add(G.nnz);
  }
  {
    GroupFormat& G = out->g[kCsl];
    G.n[0] = gS[kCsl];
    G.ind[0] = add(G.n[0] + 1);
    G.ptr[0] = add(G.n[0] + 1);
    G.runFirst[0] = add(G.runs + 1);
    for (int l = 1; l < N; ++l) G.ind[l] = add(G.nnz);
    G.val = add(G.nnz);
  }
  {
    GroupFormat& G = out->g[kCsf];
    G.n[0] = gS[kCsf];
    for (int f = 0; f < N - 2; ++f) G.n[1 + f] = nSeg[f];
    for (int l = 0; l < N - 1; ++l) {
      G.ind[l] = add(G.n[l] + 1);
      G.ptr[l] = add(G.n[l] + 1);
      G.runFirst[l] = add(G.runs + 1);
    }
    G.ind[N - 1] = add(G.nnz);
    G.val = add(G.nnz);
  }
  const uint64_t ownedWords = (out->rows + 31) / 32;
  out->ownedBits = add(ownedWords);
  out->cooBits = add(ownedWords);
  out->cooPtr = add(ownedWords + 1);
  out->blobBytes = bytes;
}

// The statistics that follow from counts alone (call after layout_mode).
inline void fill_count_stats(ModeFormat* out, int N, uint64_t M, uint64_t S,
                             const uint64_t fibNat[HBCSF_MAX_FIBER_LEVELS],
                             const uint64_t fibNatCsf[HBCSF_MAX_FIBER_LEVELS],
                             const uint64_t nSeg[HBCSF_MAX_FIBER_LEVELS], const uint64_t gS[3],
                             const uint64_t gM[3], uint64_t sharedSlices) {
  hbcsf_stats& st = out->stats;
  st = hbcsf_stats{};
  st.nnz = M;
  st.slices = S;
  for (int f = 0; f < N - 2; ++f) {
    st.fibers[f] = fibNat[f];
    st.segments[f] = nSeg[f];
  }
  for (int g = 0; g < 3; ++g) {
    st.group_nnz[g] = gM[g];
    st.group_slices[g] = gS[g];
    st.runs[g] = out->g[g].runs;
  }
  st.shared_slices = sharedSlices;
  st.words_coo = (uint64_t)N * M;
  st.words_csf = 2 * S + M;
  st.words_hbcsf = (uint64_t)N * gM[kCoo] + 2 * gS[kCsl] + (uint64_t)(N - 1) * gM[kCsl] + 2 * gS[kCsf] + gM[kCsf];
  for (int f = 0; f < N - 2; ++f) {
    st.words_csf += 2 * fibNat[f];
    st.words_hbcsf += 2 * fibNatCsf[f];
  }
  for (int g = 0; g < 3; ++g) {
    const GroupFormat& G = out->g[g];
    uint64_t words = G.val.count;
    for (int l = 0; l < N; ++l) {
      if (G.ind[l].present) words += G.ind[l].count;
      if (G.ptr[l].present) words += G.ptr[l].count;
      if (G.runFirst[l].present) words += G.runFirst[l].count;
    }
    st.stream_bytes[g] = G.nnz ? words * 4 : 0;
    st.distinct_rows[g][0] = gS[g];
  }
  uint64_t csf = gM[kCsf];
  for (int f = 0; f < N - 2; ++f) csf += nSeg[f];
  st.flops_real = (uint64_t)(N - 1) * gM[kCoo] + (uint64_t)N * gM[kCsl] + 2 * csf;
  for (int l = 0; l < N; ++l) st.level_mode[l] = (uint32_t)out->levelMode[l];
  st.fiber_threshold = out->L;
}

// Defaults measured on MI355X.  Order 3: runs of 64 nonzeros, 8 gathers in flight per lane group (132 / 128
// vector registers, 8 KB of LDS records per wavefront).  Order 4 records are twice as large and the kernel holds
// two fiber-level rows per step, so the same choice leaves 8 wavefronts per CU; runs of 32 and 4 gathers in
// flight give 16 and were 25 % faster on a 50 M-nonzero order-4 tensor.
inline uint32_t default_fiber_threshold(int order) { return order >= 4 ? 32u : 64u; }
inline int default_steps(int order) { return order >= 4 ? 4 : 8; }

// Tree levels of a mode's representation: the root is the mode itself, the others follow the policy
// (0: shortest mode first, 1: longest first, 2: natural order).
inline void level_order(int N, const uint64_t* dims, int mode, uint32_t policy, int lv[HBCSF_MAX_ORDER]) {
  lv[0] = mode;
  int rest[HBCSF_MAX_ORDER], n = 0;
  for (int m = 0; m < N; ++m)
    if (m != mode) rest[n++] = m;
  if (policy == 0 || policy == 1) {  // stable insertion sort
    for (int i = 1; i < n; ++i)
      for (int j = i; j > 0; --j) {
        const bool swap = policy == 0 ? dims[rest[j]] < dims[rest[j - 1]] : dims[rest[j]] > dims[rest[j - 1]];
        if (!swap) break;
        const int t = rest[j]; rest[j] = rest[j - 1]; rest[j - 1] = t;
      }
  }
  for (int l = 1; l < N; ++l) lv[l] = rest[l - 1];
}

inline int bits_for(uint64_t dim) {
  int b = 1;
  while (b < 63 && (1ull << b) < dim) ++b;
  return b;
}

// Blocking of the first fiber level (Section VIII names blocking as complementary future work).  A mode with
// few, huge slices whose level-1 factor matrix is far larger than an L2 gathers every level-1 row once per slice,
// each time after the whole slice has streamed through the cache.  With 2^bits blocks the level-1 index range is
// cut into equal parts and the nonzeros are ordered by (block, root, level 1, ..., leaf): a slice is stored as
// one piece per block, all pieces merged with atomic adds, and the pieces of consecutive slices that share a
// block -- hence the same level-1 rows -- are neighbours in the stream, so those rows are reused from the L2.
// Returns the number of block bits for this mode (0 = no blocking).  opts.mid_blocking: 0 or 1 = off (the
// default: on the benchmark's one qualifying mode, 1000 slices over two 40 M-row modes, 20 / 153 / 1221 blocks
// measured 4 / 10 / 19 % slower than none), 2..13 = that many bits wherever level 1 has more index bits than that.
inline int mid_block_bits(int N, const uint64_t* dims, const hbcsf_opts& opts, int mode) {
  int lv[HBCSF_MAX_ORDER];
  level_order(N, dims, mode, opts.mode_order_policy, lv);
  const int b1 = bits_for(dims[lv[1]]);
  if (opts.mid_blocking >= 2) return (int)opts.mid_blocking < b1 ? (int)opts.mid_blocking : 0;
  return 0;
}

// Builds one mode's representation.  Returns HBCSF_OK or an error code and fills `err`.
int build_mode(int order, const uint64_t* dims, uint64_t nnz, const uint32_t* const* inds,
               const float* vals, const hbcsf_opts& opts, int mode, ModeFormat* out,
               std::string* err);

}  // namespace hbcsf

#endif  // HBCSF_INTERNAL_H_
