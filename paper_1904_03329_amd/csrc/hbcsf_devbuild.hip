// Device-side format builder: COO in device memory -> per-mode HB-CSF in the caller's device arena
// (Sections III-B, IV, V; the pre-processing whose cost Section VI-E discusses).  It produces, array for
// array, what the host builder produces: sort by the packed (root, ..., leaf) key, find slices and fibers,
// put each slice into the COO / CSL / CSF group, cut fibers on the run grid (fbr-split), record which
// slices span several runs (slc-split), and write the run tables and row bitmaps.
//
// Sorting, scans and reductions are rocPRIM device primitives; everything specific to the format is in
// the kernels below.  Every per-nonzero quantity is a function of the nonzero's place p in the sorted
// order: its slice (scan of "root index changes here"), the slice's group and start inside the group's
// stream (scan over slices), hence its position in that stream, hence whether a fiber segment starts
// there (fiber index changes, or the position lies on the run grid).

#include <hip/hip_runtime.h>

#include <cstring>  // before rocPRIM, whose texture iterator calls memset without including it

#include <rocprim/rocprim.hpp>

#include <chrono>
#include <memory>
#include <new>
#include <string>

#include "hbcsf.h"
#include "hbcsf_tensor.h"

using namespace hbcsf;

namespace {

typedef unsigned __int128 u128;

struct Spec {
  int N, NF;
  int shift[HBCSF_MAX_ORDER];
  uint64_t mask[HBCSF_MAX_ORDER];
  uint32_t L, cooOn, cslOn, cooRowFlags;
  uint32_t perFiber;  // hybrid_granularity = 1: heavy slices are split into a CSL piece and a CSF piece
  int blockBits, blockShift, blockDrop;  // level-1 blocking: (index of level 1 >> blockDrop) << blockShift tops the key
};

struct C6 {  // running slice and nonzero counts of the three groups
  uint32_t s[3], m[3];
};
struct C6Plus {
  __host__ __device__ C6 operator()(const C6& a, const C6& b) const {
    C6 r;
    for (int g = 0; g < 3; ++g) {
      r.s[g] = a.s[g] + b.s[g];
      r.m[g] = a.m[g] + b.m[g];
    }
    return r;
  }
};

constexpr uint8_t kSplit = 3;  // a slice stored as a CSL piece (its singleton-fiber nonzeros) and a CSF piece

struct Tables {
  const uint32_t* sidp;    // [M] 1 + slice number of every sorted nonzero
  const uint32_t* sStart;  // [S + 1] first nonzero of every slice
  const uint8_t* grp;      // [S] group of every slice (kSplit: both)
  const C6* c6;            // [S + 1] slices / nonzeros of each group before every slice
  // per-fiber group choice only (else nullptr):
  const uint32_t* sgScan;        // [M] singleton-fiber nonzeros at or before every sorted nonzero
  const uint32_t* nat[2];        // [M] natural fiber number (inclusive scan) at fiber levels 1 and 2, where such a
                                 // level lies above the deepest one
  const uint32_t* firstKept[2];  // by natural fiber of that level: its first nonzero that stays in the CSF group
};

// Is nonzero p the only one of its deepest-level fiber?  (shiftDeep: key shift of that level)
template <typename Key>
__device__ __forceinline__ bool single_at(const Key* K, size_t p, size_t M, int shiftDeep) {
  const bool freshHere = p == 0 || (K[p] >> shiftDeep) != (K[p - 1] >> shiftDeep);
  const bool freshNext = p + 1 == M || (K[p + 1] >> shiftDeep) != (K[p] >> shiftDeep);
  return freshHere && freshNext;
}

// Group and position of sorted nonzero p.  In a split slice the singleton-fiber nonzeros go, in order, to the
// slice's CSL piece and the others to its CSF piece; sgScan counts the former.
__device__ __forceinline__ void locate(const Tables& t, size_t p, uint32_t& s, int& g, uint32_t& pos) {
  s = t.sidp[p] - 1;
  g = t.grp[s];
  const uint32_t b = t.sStart[s];
  if (g != kSplit) {
    pos = t.c6[s].m[g] + (uint32_t)(p - b);
    return;
  }
  const uint32_t before = b ? t.sgScan[b - 1] : 0u;
  const uint32_t upTo = t.sgScan[p] - before;                 // singles of the slice at or before p
  const bool single = upTo != (p > b ? t.sgScan[p - 1] - before : 0u);
  if (single) {
    g = kCsl;
    pos = t.c6[s].m[kCsl] + upTo - 1u;
  } else {
    g = kCsf;
    pos = t.c6[s].m[kCsf] + (uint32_t)(p - b) - upTo;
  }
}

template <typename Key>
struct FreshFlag {  // 1 where the index at some tree level (and everything above it) changes
  const Key* K;
  int shift;
  __device__ uint32_t operator()(size_t p) const {
    return (p == 0 || (K[p] >> shift) != (K[p - 1] >> shift)) ? 1u : 0u;
  }
};

// Does a fiber of the CSF group start at nonzero p (of that group) at the level whose key shift is `shift`?  Without
// the per-fiber choice: where the index at that level or above changes.  With it, nonzeros may have left the slice
// for the CSL piece, so: where p is the first nonzero of its natural fiber that stayed (`upper` = 0 / 1 selects the
// tables of fiber level 1 / 2; the deepest level needs none: a nonzero that left was a fiber of its own).
template <typename Key>
__device__ __forceinline__ bool fiber_starts(const Key* K, size_t p, int shift, const Tables& t, int upper) {
  if (upper >= 0 && t.firstKept[upper]) return t.firstKept[upper][t.nat[upper][p] - 1u] == (uint32_t)p;
  return p == 0 || (K[p] >> shift) != (K[p - 1] >> shift);
}

template <typename Key>
struct SegFlag {  // 1 where a fiber segment of the CSF group starts
  const Key* K;
  int shift;
  Tables t;
  uint32_t L;
  size_t M;
  int upper;  // 0 / 1: fiber level 1 / 2 lies above the deepest level (per-fiber tables apply); -1: deepest level
  __device__ uint32_t operator()(size_t p) const {
    if (p >= M) return 0u;
    uint32_t s, pos;
    int g;
    locate(t, p, s, g, pos);
    if (g != kCsf) return 0u;
    return ((pos % L) == 0 || fiber_starts(K, p, shift, t, upper)) ? 1u : 0u;
  }
};

template <typename Key>
struct SingleFlag {  // 1 where a nonzero is the only one of its deepest-level fiber
  const Key* K;
  int shiftDeep;
  size_t M;
  __device__ uint32_t operator()(size_t p) const { return p < M && single_at(K, p, M, shiftDeep) ? 1u : 0u; }
};

struct SliceIn {  // what a slice adds to the running group counts
  const uint8_t* grp;
  const uint32_t* sStart;
  size_t S;
  const uint32_t* sgScan;  // per-fiber choice only
  __device__ C6 operator()(size_t s) const {
    C6 r{{0, 0, 0}, {0, 0, 0}};
    if (s < S) {
      const int g = grp[s];
      const uint32_t b = sStart[s], e = sStart[s + 1];
      if (g == kSplit) {
        const uint32_t ns = sgScan[e - 1] - (b ? sgScan[b - 1] : 0u);
        r.s[kCsl] = 1;
        r.m[kCsl] = ns;
        r.s[kCsf] = 1;
        r.m[kCsf] = (e - b) - ns;
      } else {
        r.s[g] = 1;
        r.m[g] = e - b;
      }
    }
    return r;
  }
};

struct PopcIn {
  const uint32_t* bits;
  size_t words;
  __device__ uint32_t operator()(size_t w) const { return w < words ? (uint32_t)__popc(bits[w]) : 0u; }
};

struct SquareIn {
  const float* v;
  __device__ double operator()(size_t z) const { return (double)v[z] * (double)v[z]; }
};

__device__ __forceinline__ void wave_add(unsigned long long* dst, unsigned long long v) {
  for (int d = 32; d > 0; d >>= 1) v += __shfl_down(v, d, 64);
  if ((threadIdx.x & 63) == 0 && v) atomicAdd(dst, v);
}

struct IndPtrs {
  const uint32_t* p[HBCSF_MAX_ORDER];
};

struct Carried {  // what rides along while one 64-bit half of a wide key is being sorted
  uint64_t other;  // the half that is not the sort key of this pass
  uint32_t v, pad;
};

// Key = uint64_t: K / V receive the packed key and the value bits.  Key = u128: the key is sorted in two
// stable 64-bit passes, so the low half goes to K (as uint64_t) and the high half rides in C.
template <typename Key>
__global__ void pack_kernel(IndPtrs inds, const float* vals, size_t M, Spec sp, uint64_t dim0, uint64_t dim1,
                            uint64_t dim2, uint64_t dim3, uint64_t dim4, uint64_t* K, uint32_t* V, Carried* C,
                            unsigned long long* cnt) {
  const size_t z = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (z >= M) return;
  const uint64_t dims[HBCSF_MAX_ORDER] = {dim0, dim1, dim2, dim3, dim4};
  Key key = 0;
  bool bad = false;
  for (int l = 0; l < sp.N; ++l) {
    const uint32_t i = inds.p[l][z];
    bad = bad || (uint64_t)i >= dims[l];
    key |= (Key)i << sp.shift[l];
    if (l == 1 && sp.blockBits) key |= (Key)(i >> sp.blockDrop) << sp.blockShift;
  }
  if (sizeof(Key) == 8) {
    K[z] = (uint64_t)key;
    V[z] = __float_as_uint(vals[z]);
  } else {
    K[z] = (uint64_t)key;
    C[z] = Carried{(uint64_t)((u128)key >> 64), __float_as_uint(vals[z]), 0u};
  }
  if (bad) atomicOr(cnt, 1ull);
}

// between the two passes of a wide sort: the high half becomes the key, the low half rides along
__global__ void swap_halves_kernel(const uint64_t* keyIn, const Carried* carIn, size_t M, uint64_t* keyOut,
                                   Carried* carOut) {
  const size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= M) return;
  const Carried c = carIn[p];
  keyOut[p] = c.other;
  carOut[p] = Carried{keyIn[p], c.v, 0u};
}

__global__ void join_halves_kernel(const uint64_t* hi, const Carried* car, size_t M, u128* K, uint32_t* V) {
  const size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= M) return;
  const Carried c = car[p];
  K[p] = ((u128)hi[p] << 64) | (u128)c.other;
  V[p] = c.v;
}

// first nonzero of every slice, from the scanned slice numbers
template <typename Key>
__global__ void slice_start_kernel(const Key* K, const uint32_t* sidp, size_t M, int shift0, uint32_t* sStart) {
  const size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= M) return;
  if (p == 0 || (K[p] >> shift0) != (K[p - 1] >> shift0)) sStart[sidp[p] - 1] = (uint32_t)p;
  if (p == M - 1) sStart[sidp[p]] = (uint32_t)M;
}

// Section V / VI-D: one nonzero -> COO; every fiber a single nonzero -> CSL; otherwise CSF
__global__ void classify_kernel(const uint32_t* sStart, const uint32_t* F0, const uint32_t* F1, const uint32_t* F2,
                                size_t S, Spec sp, const uint32_t* sgScan, uint8_t* grp, unsigned long long* cnt) {
  unsigned long long c0 = 0, c1 = 0, c2 = 0;
  for (size_t s = (size_t)blockIdx.x * blockDim.x + threadIdx.x; s < S; s += (size_t)gridDim.x * blockDim.x) {
    const uint32_t b = sStart[s], e = sStart[s + 1];
    const uint32_t n = e - b;
    const uint32_t nf0 = F0[e - 1] - (b ? F0[b - 1] : 0u);
    const uint32_t nf1 = sp.NF >= 2 ? F1[e - 1] - (b ? F1[b - 1] : 0u) : 0u;
    const uint32_t nf2 = sp.NF >= 3 ? F2[e - 1] - (b ? F2[b - 1] : 0u) : 0u;
    const uint32_t deep = sp.NF == 3 ? nf2 : sp.NF == 2 ? nf1 : nf0;
    uint8_t g;
    if (n == 1 && sp.cooOn) g = kCoo;
    else if (deep == n && sp.cslOn) g = kCsl;
    else g = kCsf;
    if (sp.perFiber && g == kCsf && n >= 2u * sp.L) {
      // heavy enough to be merged with atomic adds anyway, and at least an eighth of it in singleton fibers
      const uint32_t ns = sgScan[e - 1] - (b ? sgScan[b - 1] : 0u);
      if ((unsigned long long)ns * 8ull >= (unsigned long long)n) g = kSplit;
    }
    grp[s] = g;
    if (g == kCsf && !sp.perFiber) {  // with the per-fiber choice the fibers that stay are counted after the split
      c0 += nf0;
      c1 += nf1;
      c2 += nf2;
    }
  }
  wave_add(cnt + 2, c0);
  wave_add(cnt + 3, c1);
  wave_add(cnt + 5, c2);
}

// per-fiber choice: for every natural fiber of an upper fiber level, the first of its nonzeros that stays in the
// CSF group (atomic minimum over the nonzeros of CSF and split slices)
__global__ void first_kept_kernel(size_t M, Tables t, uint32_t* first0, uint32_t* first1) {
  const size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= M) return;
  uint32_t s, pos;
  int g;
  locate(t, p, s, g, pos);
  if (g != kCsf) return;
  if (first0) atomicMin(&first0[t.nat[0][p] - 1u], (uint32_t)p);
  if (first1) atomicMin(&first1[t.nat[1][p] - 1u], (uint32_t)p);
}

__global__ void fill_words_kernel(uint32_t* p, size_t n, uint32_t v) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// per-fiber choice: fibers per level among the nonzeros that stay in the CSF group (statistics)
template <typename Key>
__global__ void count_kept_fibers_kernel(const Key* K, size_t M, Spec sp, Tables t, unsigned long long* cnt) {
  unsigned long long c[3] = {0, 0, 0};
  for (size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x; p < M; p += (size_t)gridDim.x * blockDim.x) {
    uint32_t s, pos;
    int g;
    locate(t, p, s, g, pos);
    if (g != kCsf) continue;
    for (int l = 1; l <= sp.NF; ++l) c[l - 1] += fiber_starts(K, p, sp.shift[l], t, l < sp.NF ? l - 1 : -1) ? 1u : 0u;
  }
  wave_add(cnt + 2, c[0]);
  wave_add(cnt + 3, c[1]);
  wave_add(cnt + 5, c[2]);
}

struct OutArrays {
  uint32_t* cooInd[HBCSF_MAX_ORDER];
  uint32_t* cooVal;
  uint32_t* cslInd[HBCSF_MAX_ORDER];
  uint32_t* cslPtr;
  uint32_t* cslRun;
  uint32_t* cslVal;
  uint32_t* csfInd[HBCSF_MAX_ORDER];
  uint32_t* csfPtr[HBCSF_MAX_ORDER];
  uint32_t* csfRun[HBCSF_MAX_ORDER];
  uint32_t* csfVal;
  uint32_t* owned;
  uint32_t* cooBits;
  uint32_t* seen[3][HBCSF_MAX_ORDER];  // statistics: bitmap of the factor rows each group gathers, per level
};

__device__ __forceinline__ void mark_row(uint32_t* bitmap, uint32_t r) {
  const uint32_t bit = 1u << (r & 31);
  if (!(bitmap[r >> 5] & bit)) atomicOr(&bitmap[r >> 5], bit);
}

// every nonzero writes itself into its group's stream; segment starts write the fiber-level entries
template <typename Key>
__global__ void fill_nonzeros_kernel(const Key* K, const uint32_t* V, size_t M, Spec sp, Tables t,
                                     const uint32_t* seg0, const uint32_t* seg1, const uint32_t* seg2, OutArrays o) {
  const size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= M) return;
  uint32_t s, pos;
  int g;
  locate(t, p, s, g, pos);
  const Key key = K[p];
  uint32_t idx[HBCSF_MAX_ORDER];
  for (int l = 0; l < sp.N; ++l) idx[l] = (uint32_t)((uint64_t)(key >> sp.shift[l]) & sp.mask[l]);
  const uint32_t v = V[p];
  if (g == kCoo) {
    for (int l = sp.cooRowFlags ? 1 : 0; l < sp.N; ++l) o.cooInd[l][pos] = idx[l];
    for (int l = 1; l < sp.N; ++l) mark_row(o.seen[kCoo][l], idx[l]);
    o.cooVal[pos] = v;
    atomicOr(&o.cooBits[idx[0] >> 5], 1u << (idx[0] & 31));
    atomicOr(&o.owned[idx[0] >> 5], 1u << (idx[0] & 31));
    return;
  }
  const bool cut = (pos % sp.L) == 0;
  const uint32_t ord = t.c6[s].s[g];
  if (g == kCsl) {
    for (int l = 1; l < sp.N; ++l) o.cslInd[l][pos] = idx[l];
    for (int l = 1; l < sp.N; ++l) mark_row(o.seen[kCsl][l], idx[l]);
    o.cslVal[pos] = v;
    if (cut) o.cslRun[pos / sp.L] = ord;
    return;
  }
  o.csfInd[sp.N - 1][pos] = idx[sp.N - 1];
  mark_row(o.seen[kCsf][sp.N - 1], idx[sp.N - 1]);
  o.csfVal[pos] = v;
  if (cut) o.csfRun[0][pos / sp.L] = ord;
  for (int l = 1; l <= sp.NF; ++l) {
    const bool fresh = fiber_starts(K, p, sp.shift[l], t, l < sp.NF ? l - 1 : -1);
    if (cut || fresh) {
      const uint32_t id = (l == 1 ? seg0 : l == 2 ? seg1 : seg2)[p];
      o.csfInd[l][id] = idx[l];
      o.csfPtr[l][id] = pos;
      mark_row(o.seen[kCsf][l], idx[l]);
      if (cut) o.csfRun[l][pos / sp.L] = id;
    }
  }
}

// per-slice entries of the CSL and CSF groups; a slice inside one run owns its output row
template <typename Key>
__global__ void fill_slices_kernel(const Key* K, size_t S, Spec sp, Tables t, OutArrays o,
                                   unsigned long long* cnt) {
  unsigned long long shared = 0;
  for (size_t s = (size_t)blockIdx.x * blockDim.x + threadIdx.x; s < S; s += (size_t)gridDim.x * blockDim.x) {
    const int g = t.grp[s];
    if (g == kSplit) {  // two pieces with the same root index, neither owns the row
      const uint32_t root = (uint32_t)((uint64_t)(K[t.sStart[s]] >> sp.shift[0]) & sp.mask[0]);
      o.cslInd[0][t.c6[s].s[kCsl]] = root;
      o.cslPtr[t.c6[s].s[kCsl]] = t.c6[s].m[kCsl];
      o.csfInd[0][t.c6[s].s[kCsf]] = root;
      o.csfPtr[0][t.c6[s].s[kCsf]] = t.c6[s].m[kCsf];
      ++shared;
    } else if (g != kCoo) {
      const uint32_t b = t.sStart[s], n = t.sStart[s + 1] - b;
      const uint32_t a = t.c6[s].m[g], ord = t.c6[s].s[g];
      const uint32_t root = (uint32_t)((uint64_t)(K[b] >> sp.shift[0]) & sp.mask[0]);
      const bool own = sp.blockBits == 0 && (a / sp.L) == ((a + n - 1) / sp.L);
      if (g == kCsl) {
        o.cslInd[0][ord] = root | (own ? kOwnedBit : 0u);
        o.cslPtr[ord] = a;
      } else {
        o.csfInd[0][ord] = root | (own ? kOwnedBit : 0u);
        o.csfPtr[0][ord] = a;
      }
      if (own) atomicOr(&o.owned[root >> 5], 1u << (root & 31));
      else ++shared;
    }
  }
  wave_add(cnt + 1, shared);
}

struct Sentinels {
  uint64_t cslN0, cslNnz, cslRuns, csfN[HBCSF_MAX_ORDER], csfNnz, csfRuns;
};

__global__ void sentinel_kernel(Spec sp, OutArrays o, Sentinels z) {
  if (blockIdx.x != 0 || threadIdx.x != 0) return;
  o.cslInd[0][z.cslN0] = 0;
  o.cslPtr[z.cslN0] = (uint32_t)z.cslNnz;
  o.cslRun[z.cslRuns] = (uint32_t)z.cslN0;
  for (int l = 0; l < sp.N - 1; ++l) {
    o.csfInd[l][z.csfN[l]] = 0;
    o.csfPtr[l][z.csfN[l]] = (uint32_t)z.csfNnz;
    o.csfRun[l][z.csfRuns] = (uint32_t)z.csfN[l];
  }
}

__global__ void zero_words_kernel(uint32_t* p, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

__global__ void count_bits_kernel(const uint32_t* bitmap, size_t words, unsigned long long* dst) {
  unsigned long long c = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += (size_t)gridDim.x * blockDim.x)
    c += (unsigned long long)__popc(bitmap[i]);
  wave_add(dst, c);
}

// for kernels that loop over their items and end in a few same-address atomics per wavefront
inline unsigned grid_capped(size_t n) { const size_t b = (n + 255) / 256; return (unsigned)(b < 1 ? 1 : (b > 2048 ? 2048 : b)); }
inline unsigned grid_for(size_t n) { return (unsigned)((n + 255) / 256 > 0 ? (n + 255) / 256 : 1); }
inline uint64_t up256(uint64_t v) { return (v + 255) / 256 * 256; }

// Workspace carve-up for M nonzeros; `temp` is the rocPRIM scratch, sized by temp_bytes().
struct Workspace {
  uint64_t* K[2];        // 64-bit sort keys (the packed key, or one half of a wide key), double buffered
  uint32_t* V[2];        // values riding along a 64-bit key sort, double buffered
  Carried* C[2];         // wide keys only: the other half + value, double buffered
  u128* K128;            // wide keys only: the sorted keys put together again
  uint32_t* seg2;        // order 5 only: the third fiber level's scan
  uint32_t* sgScan;      // per-fiber choice only: scan of the singleton-fiber flags
  uint32_t* nat[2];      // per-fiber choice, orders 4 / 5: natural fiber numbers of the upper fiber levels
  uint32_t* firstKept[2];  // ... and the first nonzero of each such fiber that stays in the CSF group
  uint32_t* sStart;
  uint8_t* grp;
  C6* c6;
  unsigned long long* cnt;  // 32 counters
  double* normSq;
  uint32_t* bitmap;      // 3 groups x (order - 1) levels of row bitmaps (statistics)
  size_t bitmapWords;    // words of one of them
  void* temp;
  size_t tempBytes;
  uint64_t total;
};

constexpr int kCounters = 32;

hipError_t temp_bytes(size_t M, size_t maxWords, int totalBits, size_t* out) {
  const bool wide = totalBits > 64;
  // the largest scratch any rocPRIM call below asks for
  size_t need = 0, b = 0;
  hipError_t e;
  rocprim::double_buffer<uint64_t> kb((uint64_t*)nullptr, (uint64_t*)nullptr);
  rocprim::double_buffer<uint32_t> vb((uint32_t*)nullptr, (uint32_t*)nullptr);
  e = rocprim::radix_sort_pairs(nullptr, b, kb, vb, M, 0u, (unsigned)(wide ? 64 : totalBits));
  if (e != hipSuccess) return e;
  need = b > need ? b : need;
  if (wide) {
    rocprim::double_buffer<Carried> cb((Carried*)nullptr, (Carried*)nullptr);
    e = rocprim::radix_sort_pairs(nullptr, b, kb, cb, M, 0u, 64u);
    if (e != hipSuccess) return e;
    need = b > need ? b : need;
  }
  auto cnt = rocprim::counting_iterator<size_t>(0);
  e = rocprim::inclusive_scan(nullptr, b, rocprim::make_transform_iterator(cnt, FreshFlag<u128>{nullptr, 0}),
                              (uint32_t*)nullptr, M + 1, rocprim::plus<uint32_t>());
  if (e != hipSuccess) return e;
  need = b > need ? b : need;
  e = rocprim::inclusive_scan(nullptr, b, rocprim::make_transform_iterator(cnt, SingleFlag<u128>{nullptr, 0, 0}),
                              (uint32_t*)nullptr, M + 1, rocprim::plus<uint32_t>());
  if (e != hipSuccess) return e;
  need = b > need ? b : need;
  e = rocprim::exclusive_scan(nullptr, b, rocprim::make_transform_iterator(cnt, SegFlag<u128>{nullptr, 0, Tables{}, 1, 0, -1}),
                              (uint32_t*)nullptr, 0u, M + 1, rocprim::plus<uint32_t>());
  if (e != hipSuccess) return e;
  need = b > need ? b : need;
  e = rocprim::exclusive_scan(nullptr, b, rocprim::make_transform_iterator(cnt, SliceIn{nullptr, nullptr, 0, nullptr}),
                              (C6*)nullptr, C6{{0, 0, 0}, {0, 0, 0}}, M + 1, C6Plus());
  if (e != hipSuccess) return e;
  need = b > need ? b : need;
  e = rocprim::exclusive_scan(nullptr, b, rocprim::make_transform_iterator(cnt, PopcIn{nullptr, 0}),
                              (uint32_t*)nullptr, 0u, maxWords + 1, rocprim::plus<uint32_t>());
  if (e != hipSuccess) return e;
  need = b > need ? b : need;
  e = rocprim::reduce(nullptr, b, rocprim::make_transform_iterator(cnt, SquareIn{nullptr}), (double*)nullptr, 0.0,
                      M, rocprim::plus<double>());
  if (e != hipSuccess) return e;
  need = b > need ? b : need;
  *out = need + 256;
  return hipSuccess;
}

void carve(Workspace& w, uint8_t* base, int order, size_t M, uint64_t maxDim, size_t tempBytes, bool wide,
           bool perFiber) {
  uint64_t off = 0;
  auto take = [&](uint64_t bytes) {
    uint8_t* p = base ? base + off : nullptr;
    off += up256(bytes);
    return p;
  };
  for (int i = 0; i < 2; ++i) w.K[i] = (uint64_t*)take((M + 1) * 8);
  for (int i = 0; i < 2; ++i) w.V[i] = (uint32_t*)take((M + 1) * 4);
  for (int i = 0; i < 2; ++i) w.C[i] = wide ? (Carried*)take((M + 1) * sizeof(Carried)) : nullptr;
  w.K128 = wide ? (u128*)take((M + 1) * 16) : nullptr;
  w.seg2 = order >= 5 ? (uint32_t*)take((M + 2) * 4) : nullptr;
  w.sgScan = perFiber ? (uint32_t*)take((M + 2) * 4) : nullptr;
  for (int f = 0; f < 2; ++f) {
    const bool upper = perFiber && f < order - 3;   // fiber level f + 1 lies above the deepest one
    w.nat[f] = upper ? (uint32_t*)take((M + 2) * 4) : nullptr;
    w.firstKept[f] = upper ? (uint32_t*)take((M + 2) * 4) : nullptr;
  }
  w.sStart = (uint32_t*)take((M + 2) * 4);
  w.grp = (uint8_t*)take(M + 1);
  w.c6 = (C6*)take((M + 2) * sizeof(C6));
  w.cnt = (unsigned long long*)take(kCounters * 8);
  w.normSq = (double*)take(8);
  w.bitmap = (uint32_t*)take(3 * (HBCSF_MAX_ORDER - 1) * ((maxDim + 31) / 32 + 1) * 4);
  w.bitmapWords = (maxDim + 31) / 32 + 1;
  w.temp = take(tempBytes);
  w.tempBytes = tempBytes;
  w.total = off;
}

uint64_t arena_bound(int N, const uint64_t* dims, uint64_t M, uint32_t L) {
  uint64_t bytes = 0;
  for (int m = 0; m < N; ++m) {
    const uint64_t words = (uint64_t)(2 * N + 1) * M + (uint64_t)3 * N * (M / L + 2) + 3 * (dims[m] / 32 + 2) + 64;
    bytes += words * 4 + 40 * kAlign;
  }
  return bytes;
}

// totalBits: bits of the packed (root, .., leaf) key; maxBits: the widest key of any mode, block bits included
int check_args(int order, const uint64_t* dims, uint64_t nnz, const hbcsf_opts* opts, hbcsf_opts* o, int* totalBits,
               int* maxBits) {
  if (order < 3 || order > HBCSF_MAX_ORDER) return fail(HBCSF_EINVAL, "order must be 3, 4 or 5");
  if (!dims) return fail(HBCSF_EINVAL, "dims is null");
  if (nnz >= 0xffff0000ull) return fail(HBCSF_ERANGE, "nnz must be below 2^32 - 2^16");
  int total = 0;
  for (int m = 0; m < order; ++m) {
    if (dims[m] == 0 || dims[m] > 0x7ffffffeull) return fail(HBCSF_ERANGE, "each dimension must be in 1 .. 2^31-2");
    total += bits_for(dims[m]);
  }
  *o = hbcsf_opts{};
  if (opts) *o = *opts;
  if (o->fiber_threshold == 0) o->fiber_threshold = default_fiber_threshold(order);
  const uint32_t ft = o->fiber_threshold;
  if (!(ft == 8 || ft == 16 || ft == 32 || ft == 64)) return fail(HBCSF_EINVAL, "fiber_threshold must be 8, 16, 32 or 64");
  if (o->mode_order_policy > 2) return fail(HBCSF_EINVAL, "mode_order_policy must be 0, 1 or 2");
  if (o->group_mask > 4) return fail(HBCSF_EINVAL, "group_mask must be 0..4");
  if (o->coo_row_flags > 1) return fail(HBCSF_EINVAL, "coo_row_flags must be 0 or 1");
  if (o->mid_blocking > 13) return fail(HBCSF_EINVAL, "mid_blocking must be 0 or 1 (off) or 2..13 bits");
  if (o->hybrid_granularity > 1) return fail(HBCSF_EINVAL, "hybrid_granularity must be 0 or 1");
  if (o->single_representation > 1) return fail(HBCSF_EINVAL, "single_representation must be 0 or 1");
  if (o->single_representation) {
    if ((opts->fiber_threshold && opts->fiber_threshold != default_fiber_threshold(order)) || o->group_mask ||
        o->hybrid_granularity || o->coo_row_flags || o->mid_blocking > 1)
      return fail(HBCSF_EINVAL, "single_representation goes with default options only");
    o->group_mask = 4;  // plain B-CSF: the kernel for the other modes walks one group
  }
  if (total > 128)
    return fail(HBCSF_ERANGE, "the packed coordinates exceed 128 bits: build this tensor with hbcsf_build_format");
  *totalBits = total;
  int bbMax = 0;
  for (int m = 0; m < order; ++m) {
    const int bb = mid_block_bits(order, dims, *o, m);
    bbMax = bb > bbMax ? bb : bbMax;
  }
  *maxBits = total + bbMax;
  return HBCSF_OK;
}

#define HIP_TRY(expr, what)                         \
  do {                                              \
    const hipError_t e_ = (expr);                   \
    if (e_ != hipSuccess) return fail_hip(e_, what); \
  } while (0)

template <typename Key>
int build_mode_device(int N, const uint64_t* dims, size_t M, const uint32_t* const* inds, const float* vals,
                      const hbcsf_opts& opts, int mode, int totalBits, Workspace& w, uint8_t* arena,
                      uint64_t arenaBytes, uint64_t* arenaUsed, ModeFormat* out, hipStream_t st) {
  const auto t_begin = std::chrono::steady_clock::now();
  Spec sp{};
  sp.N = N;
  sp.NF = N - 2;
  sp.L = opts.fiber_threshold;
  const uint32_t gmask = opts.group_mask == 0 ? 3u : (opts.group_mask & 3u);
  sp.blockBits = mid_block_bits(N, dims, opts, mode);
  sp.cooOn = (gmask & 1u) && sp.blockBits == 0 ? 1u : 0u;   // with blocking no piece owns its row
  sp.cslOn = (gmask & 2u) ? 1u : 0u;
  sp.cooRowFlags = opts.coo_row_flags == 1 ? 1u : 0u;
  sp.perFiber = opts.hybrid_granularity == 1 && sp.cslOn ? 1u : 0u;
  int lv[HBCSF_MAX_ORDER];
  level_order(N, dims, mode, opts.mode_order_policy, lv);
  int total = 0;
  for (int l = N - 1; l >= 0; --l) {
    const int b = bits_for(dims[lv[l]]);
    sp.shift[l] = total;
    sp.mask[l] = (1ull << b) - 1;
    total += b;
  }
  out->order = N;
  out->mode = mode;
  sp.blockShift = total;
  sp.blockDrop = sp.blockBits ? bits_for(dims[lv[1]]) - sp.blockBits : 0;
  out->L = sp.L;
  out->blockBits = sp.blockBits;
  out->cooRowFlags = sp.cooRowFlags != 0;
  out->rows = dims[mode];
  for (int l = 0; l < N; ++l) out->levelMode[l] = lv[l];

  uint64_t S = 0, gS[3] = {0, 0, 0}, gM[3] = {0, 0, 0}, nSeg[HBCSF_MAX_FIBER_LEVELS] = {0, 0, 0}, fibNat[HBCSF_MAX_FIBER_LEVELS] = {0, 0, 0};
  unsigned long long hostCnt[kCounters];
  std::memset(hostCnt, 0, sizeof(hostCnt));
  HIP_TRY(hipMemsetAsync(w.cnt, 0, kCounters * 8, st), "hipMemsetAsync");
  const Key* K = nullptr;
  const uint32_t* V = w.V[0];
  uint32_t* sidp = nullptr;
  uint32_t* seg[3] = {nullptr, nullptr, w.seg2};
  Tables tb{};
  auto cit = rocprim::counting_iterator<size_t>(0);

  if (M > 0) {
    // ---- packed keys, sorted; the value rides along ----
    IndPtrs ip{};
    uint64_t dl[HBCSF_MAX_ORDER] = {1, 1, 1, 1, 1};
    for (int l = 0; l < N; ++l) {
      ip.p[l] = inds[lv[l]];
      dl[l] = dims[lv[l]];
    }
    constexpr bool kWide = sizeof(Key) == 16;
    hipLaunchKernelGGL(pack_kernel<Key>, dim3(grid_for(M)), dim3(256), 0, st, ip, vals, M, sp, dl[0], dl[1], dl[2],
                       dl[3], dl[4], w.K[0], w.V[0], w.C[0], w.cnt);
    rocprim::double_buffer<uint64_t> kb(w.K[0], w.K[1]);
    size_t tb_ = w.tempBytes;
    if (!kWide) {
      rocprim::double_buffer<uint32_t> vb(w.V[0], w.V[1]);
      HIP_TRY(rocprim::radix_sort_pairs(w.temp, tb_, kb, vb, M, 0u, (unsigned)totalBits, st), "radix sort");
      K = (const Key*)kb.current();
      V = vb.current();
      // the buffers the sort no longer needs hold the per-nonzero scans from here on
      sidp = (uint32_t*)kb.alternate();
      seg[0] = sidp + (M + 1);
      seg[1] = vb.alternate();
    } else {
      // two stable passes: by the low 64 bits with the high half riding along, then by the high bits
      rocprim::double_buffer<Carried> cb(w.C[0], w.C[1]);
      HIP_TRY(rocprim::radix_sort_pairs(w.temp, tb_, kb, cb, M, 0u, 64u, st), "radix sort");
      hipLaunchKernelGGL(swap_halves_kernel, dim3(grid_for(M)), dim3(256), 0, st, kb.current(), cb.current(), M,
                         kb.alternate(), cb.alternate());
      rocprim::double_buffer<uint64_t> kb2(kb.alternate(), kb.current());
      rocprim::double_buffer<Carried> cb2(cb.alternate(), cb.current());
      tb_ = w.tempBytes;
      HIP_TRY(rocprim::radix_sort_pairs(w.temp, tb_, kb2, cb2, M, 0u, (unsigned)(totalBits - 64), st), "radix sort");
      hipLaunchKernelGGL(join_halves_kernel, dim3(grid_for(M)), dim3(256), 0, st, kb2.current(), cb2.current(), M,
                         w.K128, w.V[1]);
      K = (const Key*)w.K128;
      V = w.V[1];
      sidp = (uint32_t*)w.K[0];      // 8 (M + 1) bytes: slice numbers and the first fiber level's scan
      seg[0] = sidp + (M + 1);
      seg[1] = w.V[0];
    }

    // ---- slices: scan of "root index changes" ----
    tb_ = w.tempBytes;
    HIP_TRY(rocprim::inclusive_scan(w.temp, tb_, rocprim::make_transform_iterator(cit, FreshFlag<Key>{K, sp.shift[0]}),
                                    sidp, M, rocprim::plus<uint32_t>(), st), "scan");
    hipLaunchKernelGGL(slice_start_kernel<Key>, dim3(grid_for(M)), dim3(256), 0, st, K, sidp, M, sp.shift[0], w.sStart);
    // natural fibers per level (the deepest level decides CSL membership)
    for (int f = 0; f < sp.NF; ++f) {
      tb_ = w.tempBytes;
      HIP_TRY(rocprim::inclusive_scan(w.temp, tb_, rocprim::make_transform_iterator(cit, FreshFlag<Key>{K, sp.shift[1 + f]}),
                                      seg[f], M, rocprim::plus<uint32_t>(), st), "scan");
    }
    uint32_t tail[4] = {0, 0, 0, 0};
    HIP_TRY(hipMemcpyAsync(&tail[0], sidp + (M - 1), 4, hipMemcpyDeviceToHost, st), "hipMemcpyAsync");
    for (int f = 0; f < sp.NF; ++f)
      HIP_TRY(hipMemcpyAsync(&tail[1 + f], seg[f] + (M - 1), 4, hipMemcpyDeviceToHost, st), "hipMemcpyAsync");
    HIP_TRY(hipMemcpyAsync(hostCnt, w.cnt, 8, hipMemcpyDeviceToHost, st), "hipMemcpyAsync");
    HIP_TRY(hipStreamSynchronize(st), "hipStreamSynchronize");
    if (hostCnt[0]) return fail(HBCSF_ERANGE, "an index is not below its dimension");
    S = tail[0];
    fibNat[0] = tail[1];
    fibNat[1] = tail[2];
    fibNat[2] = tail[3];

    // ---- per-fiber group choice: which nonzeros are whole fibers of their own; the natural fiber numbers of the
    //      upper fiber levels are kept (the segment scans below overwrite seg[]) ----
    if (sp.perFiber) {
      tb_ = w.tempBytes;
      HIP_TRY(rocprim::inclusive_scan(w.temp, tb_,
                                      rocprim::make_transform_iterator(cit, SingleFlag<Key>{K, sp.shift[sp.NF], M}),
                                      w.sgScan, M, rocprim::plus<uint32_t>(), st), "scan");
      for (int f = 0; f + 1 < sp.NF; ++f)
        HIP_TRY(hipMemcpyAsync(w.nat[f], seg[f], M * 4, hipMemcpyDeviceToDevice, st), "hipMemcpyAsync");
    }
    // ---- groups, and where every slice starts inside its group ----
    hipLaunchKernelGGL(classify_kernel, dim3(grid_capped(S)), dim3(256), 0, st, w.sStart, seg[0], seg[1], seg[2], S, sp,
                       sp.perFiber ? w.sgScan : nullptr, w.grp, w.cnt);
    tb_ = w.tempBytes;
    HIP_TRY(rocprim::exclusive_scan(w.temp, tb_,
                                    rocprim::make_transform_iterator(cit, SliceIn{w.grp, w.sStart, S, w.sgScan}),
                                    w.c6, C6{{0, 0, 0}, {0, 0, 0}}, S + 1, C6Plus(), st), "scan");
    tb = Tables{sidp, w.sStart, w.grp, w.c6, sp.perFiber ? w.sgScan : nullptr, {nullptr, nullptr}, {nullptr, nullptr}};
    if (sp.perFiber) {
      // the first nonzero of every upper-level fiber that stays in the CSF group, then the fibers that stay
      for (int f = 0; f + 1 < sp.NF; ++f) {
        tb.nat[f] = w.nat[f];
        hipLaunchKernelGGL(fill_words_kernel, dim3(grid_for(M + 1)), dim3(256), 0, st, w.firstKept[f], M + 1, 0xffffffffu);
      }
      if (sp.NF >= 2)
        hipLaunchKernelGGL(first_kept_kernel, dim3(grid_for(M)), dim3(256), 0, st, M, tb, w.firstKept[0],
                           sp.NF >= 3 ? w.firstKept[1] : nullptr);
      for (int f = 0; f + 1 < sp.NF; ++f) tb.firstKept[f] = w.firstKept[f];
      hipLaunchKernelGGL(count_kept_fibers_kernel<Key>, dim3(grid_capped(M)), dim3(256), 0, st, K, M, sp, tb, w.cnt);
    }
    // ---- fiber segments of the CSF group: numbered by a scan over the sorted order ----
    for (int f = 0; f < sp.NF; ++f) {
      tb_ = w.tempBytes;
      HIP_TRY(rocprim::exclusive_scan(w.temp, tb_,
                                      rocprim::make_transform_iterator(
                                          cit, SegFlag<Key>{K, sp.shift[1 + f], tb, sp.L, M, f + 1 < sp.NF ? f : -1}),
                                      seg[f], 0u, M + 1, rocprim::plus<uint32_t>(), st), "scan");
    }
    C6 totals{};
    uint32_t segTotal[3] = {0, 0, 0};
    HIP_TRY(hipMemcpyAsync(&totals, w.c6 + S, sizeof(C6), hipMemcpyDeviceToHost, st), "hipMemcpyAsync");
    for (int f = 0; f < sp.NF; ++f)
      HIP_TRY(hipMemcpyAsync(&segTotal[f], seg[f] + M, 4, hipMemcpyDeviceToHost, st), "hipMemcpyAsync");
    HIP_TRY(hipStreamSynchronize(st), "hipStreamSynchronize");
    for (int g = 0; g < 3; ++g) {
      gS[g] = totals.s[g];
      gM[g] = totals.m[g];
    }
    nSeg[0] = segTotal[0];
    nSeg[1] = segTotal[1];
    nSeg[2] = segTotal[2];
  }

  // ---- layout, then fill ----
  layout_mode(out, N, gS, gM, nSeg);
  if (*arenaUsed + out->blobBytes > arenaBytes) return fail(HBCSF_ENOMEM, "device arena is too small for the format");
  out->devOffset = *arenaUsed;
  uint8_t* base = arena + out->devOffset;
  *arenaUsed += out->blobBytes;
  auto U32 = [&](const ArrayRef& r) { return (uint32_t*)(base + r.off); };
  OutArrays o{};
  for (int l = 0; l < N; ++l) {
    o.cooInd[l] = U32(out->g[kCoo].ind[l]);
    o.cslInd[l] = U32(out->g[kCsl].ind[l]);
    o.csfInd[l] = U32(out->g[kCsf].ind[l]);
    o.csfPtr[l] = l < N - 1 ? U32(out->g[kCsf].ptr[l]) : nullptr;
    o.csfRun[l] = l < N - 1 ? U32(out->g[kCsf].runFirst[l]) : nullptr;
  }
  o.cooVal = U32(out->g[kCoo].val);
  o.cslVal = U32(out->g[kCsl].val);
  o.csfVal = U32(out->g[kCsf].val);
  o.cslPtr = U32(out->g[kCsl].ptr[0]);
  o.cslRun = U32(out->g[kCsl].runFirst[0]);
  o.owned = U32(out->ownedBits);
  o.cooBits = U32(out->cooBits);
  const size_t ownedWords = (out->rows + 31) / 32;
  hipLaunchKernelGGL(zero_words_kernel, dim3(grid_for(ownedWords)), dim3(256), 0, st, o.owned, ownedWords);
  hipLaunchKernelGGL(zero_words_kernel, dim3(grid_for(ownedWords)), dim3(256), 0, st, o.cooBits, ownedWords);
  for (int g = 0; g < 3; ++g)
    for (int l = 1; l < N; ++l) o.seen[g][l] = w.bitmap + (size_t)(g * (HBCSF_MAX_ORDER - 1) + (l - 1)) * w.bitmapWords;
  {
    const size_t all = (size_t)3 * (HBCSF_MAX_ORDER - 1) * w.bitmapWords;
    hipLaunchKernelGGL(zero_words_kernel, dim3(grid_for(all)), dim3(256), 0, st, w.bitmap, all);
  }
  if (M > 0) {
    hipLaunchKernelGGL(fill_nonzeros_kernel<Key>, dim3(grid_for(M)), dim3(256), 0, st, K, V, M, sp, tb, seg[0], seg[1],
                       seg[2], o);
    hipLaunchKernelGGL(fill_slices_kernel<Key>, dim3(grid_capped(S)), dim3(256), 0, st, K, S, sp, tb, o, w.cnt);
  }
  Sentinels z{};
  z.cslN0 = out->g[kCsl].n[0];
  z.cslNnz = out->g[kCsl].nnz;
  z.cslRuns = out->g[kCsl].runs;
  for (int l = 0; l < N - 1; ++l) z.csfN[l] = out->g[kCsf].n[l];
  z.csfNnz = out->g[kCsf].nnz;
  z.csfRuns = out->g[kCsf].runs;
  hipLaunchKernelGGL(sentinel_kernel, dim3(1), dim3(64), 0, st, sp, o, z);
  {
    size_t tb_ = w.tempBytes;
    HIP_TRY(rocprim::exclusive_scan(w.temp, tb_, rocprim::make_transform_iterator(cit, PopcIn{o.cooBits, ownedWords}),
                                    U32(out->cooPtr), 0u, ownedWords + 1, rocprim::plus<uint32_t>(), st), "scan");
  }

  // ---- statistics that need a pass: rows owned by a plain store, distinct factor rows per group and level ----
  hipLaunchKernelGGL(count_bits_kernel, dim3(grid_capped(ownedWords)), dim3(256), 0, st, o.owned, ownedWords, w.cnt + 4);
  for (int g = 0; g < 3; ++g)
    for (int l = 1; l < N; ++l) {
      if (out->g[g].nnz == 0) continue;
      const size_t words = (dims[lv[l]] + 31) / 32;
      hipLaunchKernelGGL(count_bits_kernel, dim3(grid_capped(words)), dim3(256), 0, st, o.seen[g][l], words,
                         w.cnt + 8 + g * HBCSF_MAX_ORDER + l);
    }
  HIP_TRY(hipGetLastError(), "format kernels");
  HIP_TRY(hipMemcpyAsync(hostCnt, w.cnt, kCounters * 8, hipMemcpyDeviceToHost, st), "hipMemcpyAsync");
  HIP_TRY(hipStreamSynchronize(st), "hipStreamSynchronize");
  const uint64_t fibNatCsf[HBCSF_MAX_FIBER_LEVELS] = {hostCnt[2], hostCnt[3], hostCnt[5]};
  fill_count_stats(out, N, M, S, fibNat, fibNatCsf, nSeg, gS, gM, hostCnt[1]);
  out->stats.owned_rows = hostCnt[4];
  for (int g = 0; g < 3; ++g)
    for (int l = 1; l < N; ++l) out->stats.distinct_rows[g][l] = hostCnt[8 + g * HBCSF_MAX_ORDER + l];
  out->stats.build_seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t_begin).count();
  return HBCSF_OK;
}

}  // namespace

extern "C" {

int hbcsf_device_build_bytes(int order, const uint64_t* dims, uint64_t nnz, const hbcsf_opts* opts,
                             uint64_t* arena_bytes, uint64_t* workspace_bytes) try {
  hbcsf_opts o;
  int totalBits = 0, maxBits = 0;
  const int rc = check_args(order, dims, nnz, opts, &o, &totalBits, &maxBits);
  if (rc != HBCSF_OK) return rc;
  if (!arena_bytes || !workspace_bytes) return fail(HBCSF_EINVAL, "null argument");
  uint64_t maxDim = 0;
  for (int m = 0; m < order; ++m) maxDim = dims[m] > maxDim ? dims[m] : maxDim;
  size_t tbytes = 0;
  HIP_TRY(temp_bytes((size_t)nnz, (size_t)((maxDim + 31) / 32), maxBits, &tbytes), "rocPRIM scratch query");
  Workspace w{};
  carve(w, nullptr, order, (size_t)nnz, maxDim, tbytes, maxBits > 64, o.hybrid_granularity == 1);
  *workspace_bytes = w.total;
  *arena_bytes = arena_bound(order, dims, nnz, o.fiber_threshold);
  return HBCSF_OK;
} HBCSF_CATCH_ALL

int hbcsf_build_format_device(int order, const uint64_t* dims, uint64_t nnz, const uint32_t* const* inds,
                              const float* vals, const hbcsf_opts* opts, void* device_arena, uint64_t arena_bytes,
                              void* workspace, uint64_t workspace_bytes, void* hip_stream, hbcsf_tensor** out) try {
  if (!out) return fail(HBCSF_EINVAL, "out is null");
  *out = nullptr;
  hbcsf_opts o;
  int totalBits = 0, maxBits = 0;
  const int rc = check_args(order, dims, nnz, opts, &o, &totalBits, &maxBits);
  if (rc != HBCSF_OK) return rc;
  if (nnz > 0 && (!inds || !vals)) return fail(HBCSF_EINVAL, "inds or vals is null");
  for (int m = 0; m < order; ++m)
    if (nnz > 0 && !inds[m]) return fail(HBCSF_EINVAL, "an index array is null");
  if (!device_arena || !workspace) return fail(HBCSF_EINVAL, "null argument");
  if ((((uintptr_t)device_arena | (uintptr_t)workspace) & (kAlign - 1)) != 0)
    return fail(HBCSF_EINVAL, "device arena and workspace must be 256-byte aligned");
  hipStream_t st = (hipStream_t)hip_stream;
  uint64_t maxDim = 0;
  for (int m = 0; m < order; ++m) maxDim = dims[m] > maxDim ? dims[m] : maxDim;
  size_t tbytes = 0;
  HIP_TRY(temp_bytes((size_t)nnz, (size_t)((maxDim + 31) / 32), maxBits, &tbytes), "rocPRIM scratch query");
  Workspace w{};
  carve(w, (uint8_t*)workspace, order, (size_t)nnz, maxDim, tbytes, maxBits > 64, o.hybrid_granularity == 1);
  if (workspace_bytes < w.total) return fail(HBCSF_ENOMEM, "workspace is smaller than hbcsf_device_build_bytes");

  std::unique_ptr<hbcsf_tensor> t(new (std::nothrow) hbcsf_tensor);
  if (!t) return fail(HBCSF_ENOMEM, "out of host memory");
  t->order = order;
  t->nnz = nnz;
  t->opts = o;
  t->sliceThreshold = o.slice_threshold;
  t->steps = default_steps(order);
  for (int m = 0; m < order; ++m) t->dims[m] = dims[m];
  int dev = 0, cu = 0;
  HIP_TRY(hipGetDevice(&dev), "hipGetDevice");
  HIP_TRY(hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev), "hipDeviceGetAttribute");
  t->numCU = cu > 0 ? cu : 256;
  uint64_t used = 0;
  t->single = o.single_representation == 1;
  for (int m = 0; m < (t->single ? 1 : order); ++m) {  // single representation: only mode 0's tree is stored
    t->modes[m].reset(new (std::nothrow) ModeFormat);
    if (!t->modes[m]) return fail(HBCSF_ENOMEM, "out of host memory");
    const int modeBits = totalBits + mid_block_bits(order, dims, o, m);   // this mode's key width
    const int rb = modeBits > 64
                       ? build_mode_device<u128>(order, dims, (size_t)nnz, inds, vals, o, m, modeBits, w,
                                                 (uint8_t*)device_arena, arena_bytes, &used, t->modes[m].get(), st)
                       : build_mode_device<uint64_t>(order, dims, (size_t)nnz, inds, vals, o, m, modeBits, w,
                                                     (uint8_t*)device_arena, arena_bytes, &used, t->modes[m].get(), st);
    if (rb != HBCSF_OK) return rb;
  }
  double sq = 0.0;
  if (nnz > 0) {
    size_t tb_ = w.tempBytes;
    auto cit = rocprim::counting_iterator<size_t>(0);
    HIP_TRY(rocprim::reduce(w.temp, tb_, rocprim::make_transform_iterator(cit, SquareIn{vals}), w.normSq, 0.0,
                            (size_t)nnz, rocprim::plus<double>(), st), "reduce");
    HIP_TRY(hipMemcpyAsync(&sq, w.normSq, 8, hipMemcpyDeviceToHost, st), "hipMemcpyAsync");
    HIP_TRY(hipStreamSynchronize(st), "hipStreamSynchronize");
  }
  t->normSq = sq;
  t->arenaBytes = used;
  t->arena = (uint8_t*)device_arena;
  t->uploaded = true;
  *out = t.release();
  return HBCSF_OK;
} HBCSF_CATCH_ALL

int hbcsf_relocate(hbcsf_tensor* t, void* new_arena, uint64_t bytes, void* hip_stream) try {
  if (!t || !new_arena) return fail(HBCSF_EINVAL, "null argument");
  if (!t->uploaded || !t->arena) return fail(HBCSF_ESTATE, "the tensor has no device copy");
  if (bytes < t->arenaBytes) return fail(HBCSF_ENOMEM, "the new arena is smaller than hbcsf_device_bytes");
  if (((uintptr_t)new_arena & (kAlign - 1)) != 0) return fail(HBCSF_EINVAL, "device arena must be 256-byte aligned");
  hipStream_t st = (hipStream_t)hip_stream;
  HIP_TRY(hipMemcpyAsync(new_arena, t->arena, t->arenaBytes, hipMemcpyDeviceToDevice, st), "hipMemcpyAsync");
  HIP_TRY(hipStreamSynchronize(st), "hipStreamSynchronize");
  t->arena = (uint8_t*)new_arena;
  return HBCSF_OK;
} HBCSF_CATCH_ALL

int hbcsf_download(hbcsf_tensor* t, void* hip_stream) try {
  if (!t) return fail(HBCSF_EINVAL, "null argument");
  if (!t->uploaded || !t->arena) return fail(HBCSF_ESTATE, "the tensor has no device copy");
  hipStream_t st = (hipStream_t)hip_stream;
  for (int m = 0; m < t->order; ++m) {
    if (!t->modes[m]) continue;   // single representation: only mode 0 exists
    ModeFormat& f = *t->modes[m];
    if (f.blob) continue;
    void* mem = nullptr;
    if (posix_memalign(&mem, kAlign, (size_t)f.blobBytes) != 0 || !mem) return fail(HBCSF_ENOMEM, "out of host memory");
    f.blob = (uint8_t*)mem;
    HIP_TRY(hipMemcpyAsync(f.blob, t->arena + f.devOffset, f.blobBytes, hipMemcpyDeviceToHost, st), "hipMemcpyAsync");
  }
  HIP_TRY(hipStreamSynchronize(st), "hipStreamSynchronize");
  return HBCSF_OK;
} HBCSF_CATCH_ALL

}  // extern "C"
