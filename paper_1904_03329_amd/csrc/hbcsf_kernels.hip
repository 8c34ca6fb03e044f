// HIP kernels for gfx950 (MI355X): one per HB-CSF slice group plus the output definition.
//
// Mapping (wave64).  One factor row of R = 4G floats is held by G adjacent lanes, a float4
// each, so a wavefront has NG = 64/G lane groups and a row gather is one 16-byte load per
// lane.  (Built with HBCSF_F64 the factor matrices, the partial sums and the output are fp64: a lane
// then holds two doubles, R = 2G, and every address computation stays the same; the tensor's
// values are stored as fp32 either way and widened where they are multiplied.)  The nonzero stream of a group is cut into runs of L nonzeros (L = fiber threshold);
// a lane group walks one run sequentially with its partial sums in registers, so every lane
// group has exactly the same amount of work whatever the slice and fiber lengths are.  A
// unit is NG consecutive runs (one per lane group); a wavefront works through a contiguous
// span of units.
//
// B-CSF kernel (Algorithm "CSF-MTTKRP" with fbr-split / slc-split, Sections III-B and IV):
// per unit the wavefront loads the leaf indices and values coalesced into LDS records and
// turns the compressed pointer arrays into per-nonzero end marks in the same records (lane
// = fiber segment / slice, one LDS write each).  The inner loop then reads one 16-byte
// record per nonzero: tmp += v*C(k,:); at a segment end acc += tmp*B(j,:) (Eq. 8's factored
// form); at a slice end the row goes out with one plain 128-byte store if the slice lies in
// one run, else with atomic adds (Section IV-A's merge of split slices).  A partial row left
// at the end of a run stays in registers while the following units still belong to the same
// slice, so a heavy slice costs one atomic row per wavefront span, not one per run.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hbcsf_device.h"

namespace hbcsf {

namespace {

constexpr int kDenseCache = kDenseCacheRows;  // rows of the dense variant's per-wavefront row cache


// A lane's 16 bytes of a row: four floats, or two doubles.
#ifdef HBCSF_F64
typedef double real;
struct __attribute__((aligned(16))) rowvec {
  double x, y;
};
typedef double vec16 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ rowvec rv_zero() { return rowvec{0.0, 0.0}; }
__device__ __forceinline__ rowvec rv_ones() { return rowvec{1.0, 1.0}; }
__device__ __forceinline__ vec16 to_vec16(const rowvec& a) { return vec16{a.x, a.y}; }
__device__ __forceinline__ rowvec from_vec16(const vec16& v) { return rowvec{v.x, v.y}; }
#else
typedef float real;
typedef float4 rowvec;
typedef float vec16 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ rowvec rv_zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
__device__ __forceinline__ rowvec rv_ones() { return make_float4(1.f, 1.f, 1.f, 1.f); }
__device__ __forceinline__ vec16 to_vec16(const rowvec& a) { return vec16{a.x, a.y, a.z, a.w}; }
__device__ __forceinline__ rowvec from_vec16(const vec16& v) { return make_float4(v.x, v.y, v.z, v.w); }
#endif

// Streaming 16-byte store: the data is not read again by the kernel that writes it.
__device__ __forceinline__ void store_streaming(rowvec* p, const rowvec& a) {
  __builtin_nontemporal_store(to_vec16(a), reinterpret_cast<vec16*>(p));
}

// Rows are addressed in bytes (16 G per row, 16 per lane) from a base typed `const float*` whatever the
// element type.  WIDE = false: the factor matrix is smaller than 4 GiB, so a 32-bit byte offset from a
// scalar base is enough (one VALU instruction per gather); WIDE = true: 64-bit arithmetic.
template <int G, bool WIDE>
__device__ __forceinline__ rowvec row_load(const float* __restrict__ base, uint32_t row, int c) {
  if (WIDE) {
    return *reinterpret_cast<const rowvec*>(base + ((size_t)row * (size_t)(4 * G) + (size_t)(4 * c)));
  } else {
    const uint32_t off = row * (uint32_t)(16 * G) + (uint32_t)(16 * c);
    return *reinterpret_cast<const rowvec*>(reinterpret_cast<const char*>(base) + off);
  }
}

// Streaming variant: the row is not expected to be used again while it could still be cached, so
// it should not push reusable rows out of the L2.
template <int G, bool WIDE>
__device__ __forceinline__ rowvec row_load_streaming(const float* __restrict__ base, uint32_t row, int c) {
  const vec16* p;
  if (WIDE) {
    p = reinterpret_cast<const vec16*>(base + ((size_t)row * (size_t)(4 * G) + (size_t)(4 * c)));
  } else {
    const uint32_t off = row * (uint32_t)(16 * G) + (uint32_t)(16 * c);
    p = reinterpret_cast<const vec16*>(reinterpret_cast<const char*>(base) + off);
  }
  return from_vec16(__builtin_nontemporal_load(p));
}

template <int G>
__device__ __forceinline__ void row_store(float* __restrict__ out, uint32_t row, int c, rowvec a) {
  store_streaming(reinterpret_cast<rowvec*>(out + ((size_t)row * (size_t)(4 * G) + (size_t)(4 * c))), a);
}

template <int G>
__device__ __forceinline__ void row_atomic(float* __restrict__ out, uint32_t row, int c, rowvec a) {
  real* p = reinterpret_cast<real*>(out + ((size_t)row * (size_t)(4 * G) + (size_t)(4 * c)));
  unsafeAtomicAdd(p + 0, a.x);
  unsafeAtomicAdd(p + 1, a.y);
#ifndef HBCSF_F64
  unsafeAtomicAdd(p + 2, a.z);
  unsafeAtomicAdd(p + 3, a.w);
#endif
}

#ifdef HBCSF_F64
__device__ __forceinline__ void fma4(rowvec& d, float s, const rowvec& x) {
  d.x = fma((double)s, x.x, d.x);
  d.y = fma((double)s, x.y, d.y);
}

__device__ __forceinline__ void fma4(rowvec& d, const rowvec& a, const rowvec& x) {
  d.x = fma(a.x, x.x, d.x);
  d.y = fma(a.y, x.y, d.y);
}

__device__ __forceinline__ rowvec mul4(const rowvec& a, const rowvec& x) { return rowvec{a.x * x.x, a.y * x.y}; }

__device__ __forceinline__ rowvec scale4(float s, const rowvec& x) { return rowvec{(double)s * x.x, (double)s * x.y}; }

// Sum over the lanes 2^k * G apart (the same row position in every lane group).
template <int G>
__device__ __forceinline__ void sum_lane_groups(rowvec& a) {
#pragma unroll
  for (int o = G; o < 64; o <<= 1) {
    a.x += __shfl_xor(a.x, o);
    a.y += __shfl_xor(a.y, o);
  }
}
#else
__device__ __forceinline__ void fma4(rowvec& d, float s, const rowvec& x) {
  d.x = fmaf(s, x.x, d.x);
  d.y = fmaf(s, x.y, d.y);
  d.z = fmaf(s, x.z, d.z);
  d.w = fmaf(s, x.w, d.w);
}

__device__ __forceinline__ void fma4(rowvec& d, const rowvec& a, const rowvec& x) {
  d.x = fmaf(a.x, x.x, d.x);
  d.y = fmaf(a.y, x.y, d.y);
  d.z = fmaf(a.z, x.z, d.z);
  d.w = fmaf(a.w, x.w, d.w);
}

__device__ __forceinline__ rowvec mul4(const rowvec& a, const rowvec& x) {
  return make_float4(a.x * x.x, a.y * x.y, a.z * x.z, a.w * x.w);
}

__device__ __forceinline__ rowvec scale4(float s, const rowvec& x) {
  return make_float4(s * x.x, s * x.y, s * x.z, s * x.w);
}

// Sum over the lanes 2^k * G apart (the same row position in every lane group).
template <int G>
__device__ __forceinline__ void sum_lane_groups(rowvec& a) {
#pragma unroll
  for (int o = G; o < 64; o <<= 1) {
    a.x += __shfl_xor(a.x, o);
    a.y += __shfl_xor(a.y, o);
    a.z += __shfl_xor(a.z, o);
    a.w += __shfl_xor(a.w, o);
  }
}
#endif

// Which spans a wavefront works through.  Blocks are dealt round-robin to the 8 XCDs and the
// grid is a multiple of 8, so XCD x = blockIdx % 8 is given the x-th eighth of the stream: one
// slice's partial rows and its factor rows then stay within one L2 where possible.
//   default      one wavefront per span (the grid has as many wavefronts as spans);
//   persistent   a grid of resident blocks only; an XCD's wavefronts take the spans of its
//                eighth round-robin, so each gets the same number of spans from all over it.
struct SpanWalk {
  uint32_t first, end, stride;
};

__device__ __forceinline__ SpanWalk span_walk(const GroupArgs& a, int wib, int wpb) {
  const uint32_t xcd = blockIdx.x & 7u;
  const uint32_t local = (blockIdx.x >> 3) * (uint32_t)wpb + (uint32_t)wib;  // wavefront within its XCD
  const uint32_t wavesPerXcd = (gridDim.x >> 3) * (uint32_t)wpb;
  SpanWalk w;
  if (a.persistent) {
    const uint32_t perXcd = (a.nSpans + 7u) >> 3;
    w.stride = wavesPerXcd;
    w.first = __builtin_amdgcn_readfirstlane(xcd * perXcd + local);
    w.end = min((xcd + 1u) * perXcd, a.nSpans);
  } else {
    w.stride = 1;
    w.first = __builtin_amdgcn_readfirstlane(xcd * wavesPerXcd + local);
    w.end = min(w.first + 1u, a.nSpans);
  }
  return w;
}

// Pending partial row of a lane group, merged at the end of the wavefront's span.
template <int G>
__device__ __forceinline__ void final_merge(float* __restrict__ out, bool pend, uint32_t pendRow,
                                            rowvec acc, int g, int c) {
  const uint32_t first = __builtin_amdgcn_readfirstlane(pendRow);
  const bool uniform = __all(pend ? 1 : 0) && __all(pendRow == first ? 1 : 0);
  if (uniform) {
    sum_lane_groups<G>(acc);
    if (g == 0) row_atomic<G>(out, pendRow, c, acc);
  } else if (pend) {
    row_atomic<G>(out, pendRow, c, acc);
  }
}

// One trace record per wavefront: which compute unit it ran on and when (profiling only).
__device__ __forceinline__ void trace_wave(const GroupArgs& a, int kind, unsigned long long t0, int lane) {
  if (a.trace == nullptr || lane != 0) return;
  const unsigned long long t1 = wall_clock64();
  // s_getreg_b32: HW_ID (register 4, 32 bits) = wave / SIMD / CU / SH / SE ids; XCC_ID (register 20, 4 bits)
  const uint32_t hw = __builtin_amdgcn_s_getreg((31 << 11) | (0 << 6) | 4);
  const uint32_t xcc = __builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 20);
  const unsigned long long slot = atomicAdd(a.trace, 1ull);
  if (slot < a.traceCapacity) {
    unsigned long long* r = a.trace + 4 + 4 * slot;
    r[0] = (unsigned long long)kind;
    r[1] = ((unsigned long long)xcc << 32) | hw;
    r[2] = t0;
    r[3] = t1;
  }
}

__device__ __forceinline__ uint32_t mark_of_slice(uint32_t si) {
  return ((si & 0x7fffffffu) + 1u) | (si & 0x80000000u);
}


// ---------------------------------------------------------------------------------------
// Unit staging shared by the B-CSF and CSL kernels.
//
// All global loads a unit needs before its inner loop (stream data, fiber-segment and slice
// arrays, the rows at the ends of the runs) are issued back to back and awaited once, then the
// LDS records are written and the end marks scattered into them.  The run-table entries of
// the next unit are fetched one unit ahead (UnitBounds), so nothing here waits on a chain of
// dependent loads.
// ---------------------------------------------------------------------------------------
struct UnitBounds {
  uint32_t rf;      // lane t <= NG: slice holding the first nonzero of run r0 + t (clipped to runs)
  uint32_t fHi[3];  // fiber levels 1..3: first segment of the next unit (wave-uniform)
};

template <int G, int N, bool CSF>
__device__ __forceinline__ UnitBounds load_bounds(const GroupArgs& a, uint32_t u, int lane) {
  constexpr int NG = 64 / G;
  UnitBounds b;
  const uint32_t r0 = u * NG;
  b.rf = a.runFirst[0][min(r0 + (uint32_t)min(lane, NG), a.runs)];
  b.fHi[0] = b.fHi[1] = b.fHi[2] = 0;
  if (CSF) {
    const uint32_t rN = min(r0 + NG, a.runs);
#pragma unroll
    for (int l = 1; l <= N - 2; ++l) b.fHi[l - 1] = a.runFirst[l][rN];
  }
  return b;
}

struct UnitEnds {
  uint32_t headRow;  // output row of the slice holding this lane group's first nonzero
  uint32_t tailRow;  // output row of the slice holding the first nonzero of the next run
  uint32_t ng;       // nonzeros in this lane group's run (0 beyond the end of the stream)
  uint32_t sideAt;   // PACK: where the slices that end in this lane group's run start in the unit's slice list
};

// fLo: first segment of this unit per fiber level (wave-uniform; = previous unit's fHi).
// START = false: end marks (index + 1 at the LAST nonzero of a segment / slice; slice marks carry the owned bit).
// START = true : start marks (index + 1 at the FIRST nonzero), for the kernel that needs a level's index while
//                its segment is still open; a slice that began before the unit has no mark in it (headRow tells).
// PACK (B-CSF, order 4, end marks): 16-byte records {leaf, value, level-2 mark, level-1 mark | slice-end flag in bit
//                31} instead of 32-byte ones; the marks of slices (row | owned bit, as stored) go to `side`, one
//                word per slice that ends in the unit, in slice order (`side` holds NG * L words).
template <int G, int N, int LS, bool CSF, bool START = false, bool PACK = false>
__device__ __forceinline__ UnitEnds stage_unit(const GroupArgs& a, uint32_t* __restrict__ rec, uint32_t u,
                                               const UnitBounds& b, const uint32_t (&fLo)[3], int lane,
                                               uint32_t* __restrict__ side = nullptr) {
  static_assert(!PACK || (CSF && N == 4 && !START), "packed records: the order-4 B-CSF kernel");
  constexpr int NG = 64 / G;
  constexpr int NF = N - 2;
  constexpr int RW = (N == 3 || PACK) ? 4 : 8;
  constexpr int KV = 8;  // stream loads per lane issued together (covers 512 nonzeros)
  constexpr int KF = 4;  // segment loads per lane and level issued together (256 segments)
  constexpr int KS = 2;  // slice loads per lane issued together (128 slices)
  constexpr int markWord = (N == 3) ? 3 : N;  // slice mark: after the N-2 segment marks (B-CSF) / the value (CSL)
  constexpr uint32_t ls = LS, L = 1u << LS;
  constexpr uint32_t slots = (uint32_t)NG << LS;
  const uint32_t r0 = u * NG;
  const uint32_t z0 = r0 << ls;
  const int g = lane / G;
  const uint32_t* __restrict__ valb = reinterpret_cast<const uint32_t*>(a.val);

  // -- issue: rows at the ends of this lane group's run
  const uint32_t hs = __shfl(b.rf, g), ts = __shfl(b.rf, g + 1);
  const uint32_t headRaw = a.ind[0][hs], tailRaw = a.ind[0][ts];
  // -- issue: stream data
  // B-CSF: w0 = leaf index, w1 = value.  CSL: w0..w(N-2) = the N-1 non-root indices, w(N-1) = value.
  uint32_t w0[KV], w1[KV], w2[KV], w3[KV], w4[KV];
  if (z0 + slots <= a.nnz) {  // wave-uniform: every slot of the unit holds a nonzero
#pragma unroll
    for (int t = 0; t < KV; ++t) {
      const uint32_t p = (uint32_t)t * 64u + lane;
      w0[t] = w1[t] = w2[t] = w3[t] = w4[t] = 0;
      if ((uint32_t)t * 64u < slots) {
        if (CSF) {
          w0[t] = __builtin_nontemporal_load(a.ind[N - 1] + z0 + p);
          w1[t] = __builtin_nontemporal_load(valb + z0 + p);
        } else {
          w0[t] = __builtin_nontemporal_load(a.ind[1] + z0 + p);
          w1[t] = __builtin_nontemporal_load(a.ind[2] + z0 + p);
          if (N >= 4) w2[t] = __builtin_nontemporal_load(a.ind[3] + z0 + p);
          if (N >= 5) w3[t] = __builtin_nontemporal_load(a.ind[4] + z0 + p);
          (N == 3 ? w2[t] : N == 4 ? w3[t] : w4[t]) = __builtin_nontemporal_load(valb + z0 + p);
        }
      }
    }
  } else {
#pragma unroll
    for (int t = 0; t < KV; ++t) {
      const uint32_t p = (uint32_t)t * 64u + lane;
      const uint32_t z = z0 + p;
      w0[t] = w1[t] = w2[t] = w3[t] = w4[t] = 0;
      if (p < slots && z < a.nnz) {
        if (CSF) {
          w0[t] = __builtin_nontemporal_load(a.ind[N - 1] + z);
          w1[t] = __builtin_nontemporal_load(valb + z);
        } else {
          w0[t] = __builtin_nontemporal_load(a.ind[1] + z);
          w1[t] = __builtin_nontemporal_load(a.ind[2] + z);
          if (N >= 4) w2[t] = __builtin_nontemporal_load(a.ind[3] + z);
          if (N >= 5) w3[t] = __builtin_nontemporal_load(a.ind[4] + z);
          (N == 3 ? w2[t] : N == 4 ? w3[t] : w4[t]) = __builtin_nontemporal_load(valb + z);
        }
      }
    }
  }
  // -- issue: fiber-segment ends and indices
  uint32_t fe[3][KF], fi[3][KF];
  if (CSF) {
#pragma unroll
    for (int l = 1; l <= NF; ++l) {
#pragma unroll
      for (int t = 0; t < KF; ++t) {
        const uint32_t f = fLo[l - 1] + (uint32_t)t * 64u + lane;
        fe[l - 1][t] = 0;
        fi[l - 1][t] = 0;
        if (f < b.fHi[l - 1]) {
          fe[l - 1][t] = __builtin_nontemporal_load(a.ptr[l] + f + (START ? 0 : 1));
          fi[l - 1][t] = __builtin_nontemporal_load(a.ind[l] + f);
        }
      }
    }
  }
  // -- issue: slice ends and indices
  // END marks: the slices that end in this unit are those before the one holding the next unit's first nonzero.
  // START marks: that slice may itself begin in this unit, so it is looked at too (a position test decides).
  const uint32_t s0 = __builtin_amdgcn_readfirstlane(b.rf);
  const uint32_t s1 = __shfl(b.rf, NG) + (START ? 1u : 0u);
  uint32_t se[KS], si[KS];
#pragma unroll
  for (int t = 0; t < KS; ++t) {
    const uint32_t sl = s0 + (uint32_t)t * 64u + lane;
    se[t] = 0;
    si[t] = 0;
    if (sl < s1) {
      se[t] = a.ptr[0][sl + (START ? 0 : 1)];
      si[t] = a.ind[0][sl];
    }
  }

  // -- records: stream data in, marks cleared
#pragma unroll
  for (int t = 0; t < KV; ++t) {
    const uint32_t p = (uint32_t)t * 64u + lane;
    if (p < slots) {
      uint4* dst = reinterpret_cast<uint4*>(rec + (size_t)(p + (p >> ls)) * RW);
      if (CSF) {
        dst[0] = make_uint4(w0[t], w1[t], 0u, 0u);
        if (N >= 4 && !PACK) dst[1] = make_uint4(0u, 0u, 0u, 0u);
      } else if (N == 3) {
        dst[0] = make_uint4(w0[t], w1[t], w2[t], 0u);
      } else {
        dst[0] = make_uint4(w0[t], w1[t], w2[t], w3[t]);
        dst[1] = make_uint4(N == 5 ? w4[t] : 0u, 0u, 0u, 0u);
      }
    }
  }
  for (uint32_t p = (uint32_t)KV * 64u + lane; p < slots; p += 64) {  // units above 512 nonzeros
    const uint32_t z = z0 + p;
    uint32_t x0 = 0, x1 = 0, x2 = 0, x3 = 0, x4 = 0;
    if (z < a.nnz) {
      if (CSF) {
        x0 = a.ind[N - 1][z];
        x1 = valb[z];
      } else {
        x0 = a.ind[1][z];
        x1 = a.ind[2][z];
        if (N >= 4) x2 = a.ind[3][z];
        if (N >= 5) x3 = a.ind[4][z];
        (N == 3 ? x2 : N == 4 ? x3 : x4) = valb[z];
      }
    }
    uint4* dst = reinterpret_cast<uint4*>(rec + (size_t)(p + (p >> ls)) * RW);
    if (CSF) {
      dst[0] = make_uint4(x0, x1, 0u, 0u);
      if (N >= 4 && !PACK) dst[1] = make_uint4(0u, 0u, 0u, 0u);
    } else if (N == 3) {
      dst[0] = make_uint4(x0, x1, x2, 0u);
    } else {
      dst[0] = make_uint4(x0, x1, x2, x3);
      dst[1] = make_uint4(N == 5 ? x4 : 0u, 0u, 0u, 0u);
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");

  // -- segment end marks
  if (CSF) {
#pragma unroll
    for (int l = 1; l <= NF; ++l) {
      const int word = 2 + (NF - l);
#pragma unroll
      for (int t = 0; t < KF; ++t) {
        const uint32_t f = fLo[l - 1] + (uint32_t)t * 64u + lane;
        if (f < b.fHi[l - 1]) {
          const uint32_t p = fe[l - 1][t] - (START ? 0u : 1u) - z0;
          uint32_t* at = rec + (size_t)(p + (p >> ls)) * RW + word;
          if (PACK && l == 1) atomicOr(at, fi[l - 1][t] + 1u);   // the slice-end flag may land in the same word
          else *at = fi[l - 1][t] + 1u;
        }
      }
      for (uint32_t f = fLo[l - 1] + (uint32_t)KF * 64u + lane; f < b.fHi[l - 1]; f += 64) {
        const uint32_t p = a.ptr[l][f + (START ? 0 : 1)] - (START ? 0u : 1u) - z0;
        uint32_t* at = rec + (size_t)(p + (p >> ls)) * RW + word;
        if (PACK && l == 1) atomicOr(at, a.ind[l][f] + 1u);
        else *at = a.ind[l][f] + 1u;
      }
    }
  }
  // -- slice end marks
#pragma unroll
  for (int t = 0; t < KS; ++t) {
    const uint32_t sl = s0 + (uint32_t)t * 64u + lane;
    if (sl < s1 && (!START || (se[t] >= z0 && se[t] < z0 + slots && se[t] < a.nnz))) {
      const uint32_t p = se[t] - (START ? 0u : 1u) - z0;
      if (PACK) {
        atomicOr(rec + (size_t)(p + (p >> ls)) * RW + 3, 0x80000000u);
        side[sl - s0] = si[t];
      } else {
        rec[(size_t)(p + (p >> ls)) * RW + markWord] = START ? (si[t] & 0x7fffffffu) + 1u : mark_of_slice(si[t]);
      }
    }
  }
  for (uint32_t sl = s0 + (uint32_t)KS * 64u + lane; sl < s1; sl += 64) {
    const uint32_t at = a.ptr[0][sl + (START ? 0 : 1)];
    if (START && (at < z0 || at >= z0 + slots || at >= a.nnz)) continue;
    const uint32_t p = at - (START ? 0u : 1u) - z0;
    const uint32_t sv = a.ind[0][sl];
    if (PACK) {
      atomicOr(rec + (size_t)(p + (p >> ls)) * RW + 3, 0x80000000u);
      side[sl - s0] = sv;
    } else {
      rec[(size_t)(p + (p >> ls)) * RW + markWord] = START ? (sv & 0x7fffffffu) + 1u : mark_of_slice(sv);
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

  UnitEnds e;
  const uint32_t r = r0 + g;
  e.headRow = headRaw & 0x7fffffffu;
  e.tailRow = tailRaw & 0x7fffffffu;
  e.ng = r < a.runs ? min(L, a.nnz - (r << ls)) : 0u;
  e.sideAt = hs - s0;
  return e;
}

}  // namespace

// The fp64 objects instantiate the same kernel templates with the same arguments as the fp32 ones: a namespace of
// their own keeps the two sets of kernels apart at link time.
#ifdef HBCSF_F64
namespace f64 {
#endif

// ---------------------------------------------------------------------------------------
// Output definition: rows that no plain store will write (empty slices and rows merged with
// atomic adds) are set to zero; the others are left to their single store.
// ---------------------------------------------------------------------------------------
#ifdef HBCSF_WITH_DEFINE
// One wavefront takes one bitmap word (32 rows) at a time: the word is read once through the
// scalar path and each lane then stores its share of the 32 rows' float4s.
__global__ __launch_bounds__(256) void define_rows_kernel(rowvec* __restrict__ out,
                                                          const uint32_t* __restrict__ ownedBits,
                                                          uint64_t nvec, int gshift) {
  const int lane = threadIdx.x & 63;
  const uint32_t waves = (gridDim.x * blockDim.x) >> 6;
  const uint32_t wave = __builtin_amdgcn_readfirstlane((blockIdx.x * blockDim.x + threadIdx.x) >> 6);
  const uint64_t perWord = (uint64_t)32 << gshift;      // float4s covered by one bitmap word
  const uint64_t words = (nvec + perWord - 1) / perWord;
  const int reps = (int)(perWord >> 6);                  // stores per lane per word (G / 2)
  // a wavefront fills kChunk consecutive words (kChunk x 32 rows) before it strides on
  constexpr uint64_t kChunk = 8;
  for (uint64_t w0 = (uint64_t)wave * kChunk; w0 < words; w0 += (uint64_t)waves * kChunk) {
    const uint64_t w1 = min(w0 + kChunk, words);
    for (uint64_t wd = w0; wd < w1; ++wd) {
      const uint32_t w = ownedBits[wd];
      const uint64_t base = wd * perWord;
      for (int q = 0; q < reps; ++q) {
        const uint32_t f = (uint32_t)q * 64u + lane;        // rowvec within the word's 32 rows
        const uint64_t t = base + f;
        if (t < nvec && !((w >> (f >> gshift)) & 1u)) store_streaming(out + t, rv_zero());
      }
    }
  }
}
#endif  // HBCSF_WITH_DEFINE

// ---------------------------------------------------------------------------------------
// B-CSF group.  N = tensor order (3, 4 or 5); G = lanes per factor row.
// LDS record per nonzero: N = 3: {leaf, val, seg1 mark, slice mark};
//                         N = 4: {leaf, val, seg2 mark, seg1 mark | slice-end flag} (16 bytes; the marks of the
//                                slices that end in the unit sit in a list beside the records, in slice order,
//                                and a lane group takes them one after the other as it meets the flags);
//                                the dense-gather variant keeps {leaf, val, seg2, seg1, slice mark, -, -, -};
//                         N = 5: {leaf, val, seg3 mark, seg2 mark, seg1 mark, slice mark, -, -}.
// A segment mark is index+1 at the segment's last nonzero, else 0.  A slice mark is
// (row+1) | owned bit at the slice's last nonzero, else 0.
// ---------------------------------------------------------------------------------------
//
// DENSE (orders 3 and 4): the rows of the fiber levels are not gathered at the step where a segment ends (one
// load instruction per step in which ANY lane group ends a segment, most of its lanes idle) but once per block of
// kSteps steps for the whole wavefront: every lane group counts the marks in its kSteps records, a prefix sum over
// the lane groups gives each mark a slot, the row numbers go to a list in LDS, and ceil(marks / NG) load
// instructions with all lanes busy bring the rows into an LDS row cache, from which the steps then read them.
// Every vector-memory instruction keeps the CU's address unit busy for the same 16 cycles however many lanes
// are active, and that unit is what bounds this kernel when the factor matrices are cache-resident.  The cache
// holds kDenseCache rows; marks beyond it (rare when segments average a few nonzeros) load their row directly.
template <int G, int N, int LS, int kSteps, bool WIDE, bool DENSE>
__device__ __forceinline__ void csf_group_body(const GroupArgs& a) {
  constexpr int NG = 64 / G;
  constexpr int NF = N - 2;
  // order 4 (the plain variant): 16-byte records, the level-1 mark and the slice-end flag in one word, the slices'
  // rows in a per-unit list beside the records
  constexpr bool PACK = N == 4 && !DENSE;
  constexpr int RW = (N == 3 || PACK) ? 4 : 8;
  static_assert(!DENSE || N <= 4, "the dense fiber-row gather handles orders 3 and 4");
  extern __shared__ uint32_t lds[];
  const int lane = threadIdx.x & 63;
  const int wib = threadIdx.x >> 6;
  const int wpb = blockDim.x >> 6;
  const int g = lane / G, c = lane % G;
  constexpr uint32_t L = 1u << LS;
  constexpr uint32_t recWords = NG * (L + 1) * RW;
  constexpr uint32_t waveWords = recWords + (DENSE ? 64u + (uint32_t)kDenseCache * G * 4u : 0u) + (PACK ? NG * L : 0u);
  uint32_t* rec = lds + (size_t)wib * waveWords;
  uint32_t* side = rec + recWords;                                   // PACK: marks of the slices that end in the unit
  uint32_t* list = rec + recWords;                                   // DENSE: row numbers by slot
  rowvec* cache = reinterpret_cast<rowvec*>(rec + recWords + 64);    // DENSE: rows by slot, G rowvec each


  const float* __restrict__ facLeaf = a.fac[N - 1];
  const float* __restrict__ facDeep = a.fac[N - 2];   // deepest fiber level
  const float* __restrict__ facNext = a.fac[N >= 4 ? N - 3 : 1];  // the fiber level above it (N >= 4)
  const float* __restrict__ facTop = a.fac[1];        // level 1 (N = 5: the third fiber level from the leaf)

  const unsigned long long traceStart = a.trace ? wall_clock64() : 0ull;
  const SpanWalk walk = span_walk(a, wib, wpb);
  for (uint32_t span = walk.first; span < walk.end; span += walk.stride) {
  uint32_t u = span * a.unitsPerWave;
  const uint32_t uEnd = min(u + a.unitsPerWave, a.nUnits);
  rowvec acc = rv_zero();
  bool pend = false;
  uint32_t pendRow = 0;

  UnitBounds cur = load_bounds<G, N, true>(a, u, lane);
  uint32_t fLo[3] = {0, 0, 0};
#pragma unroll
  for (int l = 1; l <= NF; ++l) fLo[l - 1] = a.runFirst[l][u * NG];

  for (; u < uEnd; ++u) {
    // run-table entries of the next unit: in flight while this unit is staged and processed
    const UnitBounds nxt = load_bounds<G, N, true>(a, min(u + 1, a.nUnits - 1), lane);
    const UnitEnds ends = stage_unit<G, N, LS, true, false, PACK>(a, rec, u, cur, fLo, lane, side);
    const uint32_t headRow = ends.headRow, tailRow = ends.tailRow, ng = ends.ng;
    uint32_t sideAt = ends.sideAt;   // PACK: the next slice of this lane group's run in the unit's slice list
    fLo[0] = cur.fHi[0];
    fLo[1] = cur.fHi[1];
    fLo[2] = cur.fHi[2];
    cur = nxt;

    // A lane group whose run lies beyond the end of the stream (ng = 0, last unit only) has all-zero records.  The
    // dense variant's block loop is collective (prefix sum over the lane groups, shared list and row cache), so
    // every lane group runs it, live or not; zero records hold no marks and so change nothing.
    {
      if (ng > 0 && pend && pendRow != headRow) {
        row_atomic<G>(a.out, pendRow, c, acc);
        acc = rv_zero();
      }
      // tmp: sum over the leaves of the open deepest-level segment; tmp1 / tmp2: sums over the closed segments
      // of the next levels up (N >= 4 / N = 5); acc: the slice's row.  Marks are nested: a segment of a level
      // can only end where one of every deeper level ends.
      rowvec tmp = rv_zero();
      rowvec tmp1 = rv_zero();
      rowvec tmp2 = rv_zero();
      const uint32_t* myrec = rec + (size_t)g * (L + 1) * RW;
      if constexpr (DENSE) {
      for (uint32_t sb = 0; sb < L; sb += kSteps) {
        uint4 rr[kSteps];
        uint32_t mi[kSteps];   // slice mark
        uint32_t sl[kSteps];   // slot (within this lane group) of the deepest level's mark, then of the next level's
        rowvec cr[kSteps];
#pragma unroll
        for (int t = 0; t < kSteps; ++t) {
          const uint4* src = reinterpret_cast<const uint4*>(myrec + (size_t)(sb + t) * RW);
          rr[t] = src[0];
          mi[t] = (N == 3) ? rr[t].w : reinterpret_cast<const uint32_t*>(src)[4];
        }
        // marks of this block per lane group, and where its slots start
        uint32_t cnt = 0;
#pragma unroll
        for (int t = 0; t < kSteps; ++t) {
          sl[t] = cnt;
          cnt += rr[t].z ? 1u : 0u;
          if (N == 4) cnt += rr[t].w ? 1u : 0u;   // its slot is sl[t] + 1 (a level-1 mark implies a level-2 mark)
        }
        uint32_t incl = cnt;
#pragma unroll
        for (int o = G; o < 64; o <<= 1) {
          const uint32_t up = __shfl_up(incl, o);
          if (lane >= o) incl += up;
        }
        const uint32_t base = incl - cnt;
        const uint32_t total = __builtin_amdgcn_readlane(incl, 63);
#pragma unroll
        for (int t = 0; t < kSteps; ++t) {
          sl[t] += base;
          if (rr[t].z && sl[t] < (uint32_t)kDenseCache) list[sl[t]] = rr[t].z - 1u;
          if (N == 4 && rr[t].w && sl[t] + 1u < (uint32_t)kDenseCache) list[sl[t] + 1u] = (rr[t].w - 1u) | 0x80000000u;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        // the rows, NG per load instruction
        const uint32_t nq = min(total, (uint32_t)kDenseCache);
        constexpr int kRounds = kDenseCache / NG;
        rowvec mr[kRounds];
#pragma unroll
        for (int u2 = 0; u2 < kRounds; ++u2) {
          const uint32_t q = (uint32_t)u2 * NG + g;
          if ((uint32_t)u2 * NG < nq) {        // wave-uniform: rounds past the last slot issue nothing
            if (q < nq) {
              const uint32_t e = list[q];
              const uint32_t row = e & 0x7fffffffu;
              if (N == 4 && (e >> 31)) {
                mr[u2] = (a.streamLevel & 2u) ? row_load_streaming<G, WIDE>(facNext, row, c)
                                              : row_load<G, WIDE>(facNext, row, c);
              } else {
                mr[u2] = (a.streamLevel & (1u << (N - 2))) ? row_load_streaming<G, WIDE>(facDeep, row, c)
                                                           : row_load<G, WIDE>(facDeep, row, c);
              }
            }
          }
        }
#pragma unroll
        for (int t = 0; t < kSteps; ++t) cr[t] = row_load<G, WIDE>(facLeaf, rr[t].x, c);
#pragma unroll
        for (int u2 = 0; u2 < kRounds; ++u2) {
          const uint32_t q = (uint32_t)u2 * NG + g;
          if ((uint32_t)u2 * NG < nq && q < nq) cache[(size_t)q * G + c] = mr[u2];
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
        for (int t = 0; t < kSteps; ++t) {
          fma4(tmp, __uint_as_float(rr[t].y), cr[t]);
          if (rr[t].z) {
            const rowvec br = sl[t] < (uint32_t)kDenseCache ? cache[(size_t)sl[t] * G + c]
                                                             : row_load<G, WIDE>(facDeep, rr[t].z - 1u, c);
            if (N == 3) {
              fma4(acc, tmp, br);
            } else {
              fma4(tmp1, tmp, br);
              if (rr[t].w) {
                const rowvec nr = sl[t] + 1u < (uint32_t)kDenseCache ? cache[(size_t)(sl[t] + 1u) * G + c]
                                                                      : row_load<G, WIDE>(facNext, rr[t].w - 1u, c);
                fma4(acc, tmp1, nr);
                tmp1 = rv_zero();
              }
            }
            tmp = rv_zero();
            if (mi[t]) {  // a slice can only end where a segment ends
              const uint32_t row = (mi[t] & 0x7fffffffu) - 1u;
              if (mi[t] & 0x80000000u) row_store<G>(a.out, row, c, acc);
              else row_atomic<G>(a.out, row, c, acc);
              acc = rv_zero();
            }
          }
        }
        // the next block rewrites the list and the cache
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      }
      } else if (ng > 0) {
      for (uint32_t sb = 0; sb < L; sb += kSteps) {
        uint4 rr[kSteps];
        uint32_t m1[kSteps];   // N = 5: mark of fiber level 1
        uint32_t mi[kSteps];   // slice mark
        rowvec cr[kSteps], br[kSteps], nr[kSteps], ar[kSteps];
#pragma unroll
        for (int t = 0; t < kSteps; ++t) {
          const uint4* src = reinterpret_cast<const uint4*>(myrec + (size_t)(sb + t) * RW);
          rr[t] = src[0];
          if (N == 3) {
            mi[t] = rr[t].w;
            m1[t] = 0;
          } else if (PACK) {
            mi[t] = rr[t].w & 0x80000000u;   // slice-end flag; the slice's mark is next in the unit's slice list
            rr[t].w &= 0x7fffffffu;
            m1[t] = 0;
          } else if (N == 4) {
            mi[t] = reinterpret_cast<const uint32_t*>(src)[4];
            m1[t] = 0;
          } else {
            const uint2 hi = reinterpret_cast<const uint2*>(src)[2];
            m1[t] = hi.x;
            mi[t] = hi.y;
          }
        }
        // Conditional loads first: loads return in order, so once a leaf row has arrived every
        // load issued before it has arrived too, and the leaf rows can be awaited one by one.
#pragma unroll
        for (int t = 0; t < kSteps; ++t) {
          if (rr[t].z) {
            br[t] = (a.streamLevel & (1u << (N - 2))) ? row_load_streaming<G, WIDE>(facDeep, rr[t].z - 1u, c)
                                                       : row_load<G, WIDE>(facDeep, rr[t].z - 1u, c);
          }
          if (N >= 4 && rr[t].w) {
            nr[t] = (a.streamLevel & (1u << (N - 3))) ? row_load_streaming<G, WIDE>(facNext, rr[t].w - 1u, c)
                                                       : row_load<G, WIDE>(facNext, rr[t].w - 1u, c);
          }
          if (N == 5 && m1[t]) {
            ar[t] = (a.streamLevel & 2u) ? row_load_streaming<G, WIDE>(facTop, m1[t] - 1u, c)
                                         : row_load<G, WIDE>(facTop, m1[t] - 1u, c);
          }
        }
#pragma unroll
        for (int t = 0; t < kSteps; ++t) cr[t] = row_load<G, WIDE>(facLeaf, rr[t].x, c);
#pragma unroll
        for (int t = 0; t < kSteps; ++t) {
          fma4(tmp, __uint_as_float(rr[t].y), cr[t]);
          if (rr[t].z) {
            if (N == 3) {
              fma4(acc, tmp, br[t]);
            } else {
              fma4(tmp1, tmp, br[t]);
              if (rr[t].w) {
                if (N == 4) {
                  fma4(acc, tmp1, nr[t]);
                } else {
                  fma4(tmp2, tmp1, nr[t]);
                  if (m1[t]) {
                    fma4(acc, tmp2, ar[t]);
                    tmp2 = rv_zero();
                  }
                }
                tmp1 = rv_zero();
              }
            }
            tmp = rv_zero();
            if (mi[t]) {  // a slice can only end where a segment ends
              // PACK: the stored root entry (row | owned bit) of the next slice of this run; else the mark itself
              const uint32_t sm = PACK ? side[sideAt++] : mi[t];
              const uint32_t row = (sm & 0x7fffffffu) - (PACK ? 0u : 1u);
              if (sm & 0x80000000u) row_store<G>(a.out, row, c, acc);
              else row_atomic<G>(a.out, row, c, acc);
              acc = rv_zero();
            }
          }
        }
      }
      }  // classic / dense
      // the run leaves a partial row behind unless its last nonzero ends a slice
      if (ng > 0) {
        pend = PACK ? (myrec[(size_t)(ng - 1) * RW + 3] & 0x80000000u) == 0u
                    : myrec[(size_t)(ng - 1) * RW + (N == 3 ? 3 : N)] == 0u;
        pendRow = tailRow;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  }
  final_merge<G>(a.out, pend, pendRow, acc, g, c);
  }  // spans
  trace_wave(a, kCsfKernel, traceStart, lane);
}

template <int G, int N, int LS, int kSteps, bool WIDE>
__global__ __launch_bounds__(256) void csf_group_kernel(const GroupArgs a) {
  csf_group_body<G, N, LS, kSteps, WIDE, false>(a);
}

template <int G, int N, int LS, int kSteps, bool WIDE>
__global__ __launch_bounds__(256) void csf_group_dense_kernel(const GroupArgs a) {
  csf_group_body<G, N, LS, kSteps, WIDE, true>(a);
}

// The order-3, R = 32, 32-bit-offset instantiation needs 132 vector registers, four more than fit four
// wavefronts per SIMD; held to 128 it spills three registers and gains a wavefront per SIMD, which pays on
// the cache-resident workloads (measured -4.5 % on a 100 M-nonzero tensor whose factors fit the L2).  The
// 64-bit-offset instantiation spills more and loses; order 4 (176 registers, held to 168 for a third wavefront
// per SIMD) measured no gain; both keep the plain kernel.
template <int G, int N, int LS, int kSteps>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4))) void csf_group_kernel_occ4(const GroupArgs a) {
  csf_group_body<G, N, LS, kSteps, false, false>(a);
}

// ---------------------------------------------------------------------------------------
// Single-representation variant (Section VI-A's other setting: one representation serves every mode, at 1 / N of
// the storage).  The target mode sits at tree level T >= 1 of another mode's B-CSF representation (all slices in
// the CSF group).  A lane group walks its run with START marks and keeps the current row of every level above the
// leaf; writing i_l for the index at level l,
//     out(i_T, :) += prod_{l < T} A_l(i_l, :)  *  sum over the level-T segment of  v * prod_{l > T} A_l(i_l, :)
// is added with atomic adds at the end of each level-T segment (T = leaf: per nonzero; then no leaf row is
// gathered).  The rows of the levels above the leaf are loaded where they change; leaf rows kSteps at a time.
// Rank 32 only (G = 8).  Every output row is reached by atomics, so the caller zero-fills the output first.
// ---------------------------------------------------------------------------------------
template <int N, int LS, int T, bool WIDE>
__global__ __launch_bounds__(256) void csf_nonroot_kernel(const GroupArgs a) {
  constexpr int G = 8;
  constexpr int NG = 64 / G;
  constexpr int NF = N - 2;
  constexpr int RW = (N == 3) ? 4 : 8;
  constexpr int LEAF = N - 1;
  constexpr int kSteps = 4;
  static_assert(T >= 1 && T <= LEAF, "the target is below the root");
  extern __shared__ uint32_t lds[];
  const int lane = threadIdx.x & 63;
  const int wib = threadIdx.x >> 6;
  const int wpb = blockDim.x >> 6;
  const int g = lane / G, c = lane % G;
  constexpr uint32_t L = 1u << LS;
  uint32_t* rec = lds + (size_t)wib * (NG * (L + 1) * RW);

  const SpanWalk walk = span_walk(a, wib, wpb);
  for (uint32_t span = walk.first; span < walk.end; span += walk.stride) {
    uint32_t u = span * a.unitsPerWave;
    const uint32_t uEnd = min(u + a.unitsPerWave, a.nUnits);
    UnitBounds cur = load_bounds<G, N, true>(a, u, lane);
    uint32_t fLo[3] = {0, 0, 0};
#pragma unroll
    for (int l = 1; l <= NF; ++l) fLo[l - 1] = a.runFirst[l][u * NG];

    for (; u < uEnd; ++u) {
      const UnitBounds nxt = load_bounds<G, N, true>(a, min(u + 1, a.nUnits - 1), lane);
      const UnitEnds ends = stage_unit<G, N, LS, true, true>(a, rec, u, cur, fLo, lane);
      fLo[0] = cur.fHi[0];
      fLo[1] = cur.fHi[1];
      fLo[2] = cur.fHi[2];
      cur = nxt;
      const uint32_t ng = ends.ng;
      if (ng > 0) {
        // rows of the levels above the leaf (lr[T] unused), their products above / below the target level
        rowvec lr[LEAF];
#pragma unroll
        for (int l = 0; l < LEAF; ++l) lr[l] = rv_ones();
        lr[0] = row_load<G, WIDE>(a.fac[0], ends.headRow, c);   // the slice may have begun in an earlier run
        rowvec up = rv_ones(), dn = rv_ones();
        rowvec acc = rv_zero();
        uint32_t curT = 0;
        bool open = false;
        const uint32_t* myrec = rec + (size_t)g * (L + 1) * RW;
        for (uint32_t sb = 0; sb < ng; sb += kSteps) {
          uint4 rr[kSteps];
          uint32_t hi0[kSteps], hi1[kSteps];   // record words 4 and 5 (N >= 4)
          rowvec cr[kSteps];
#pragma unroll
          for (int t = 0; t < kSteps; ++t) {
            const uint4* src = reinterpret_cast<const uint4*>(myrec + (size_t)(sb + t) * RW);
            rr[t] = src[0];
            hi0[t] = hi1[t] = 0;
            if (N >= 4) {
              const uint2 h2 = reinterpret_cast<const uint2*>(src)[2];
              hi0[t] = h2.x;
              hi1[t] = h2.y;
            }
          }
          if (T < LEAF) {
#pragma unroll
            for (int t = 0; t < kSteps; ++t) cr[t] = row_load<G, WIDE>(a.fac[LEAF], rr[t].x, c);
          }
#pragma unroll
          for (int t = 0; t < kSteps; ++t) {
            if (sb + (uint32_t)t < ng) {
              // start marks by level: fiber level l at record word 2 + (NF - l), the slice after them
              uint32_t mk[LEAF];
              mk[0] = (N == 3) ? rr[t].w : (N == 4 ? hi0[t] : hi1[t]);
              mk[LEAF - 1] = rr[t].z;                           // deepest fiber level
              if constexpr (N >= 4) mk[LEAF - 2] = rr[t].w;
              if constexpr (N == 5) mk[1] = hi0[t];
              bool any = false;
#pragma unroll
              for (int l = 0; l < LEAF; ++l) any = any || mk[l] != 0u;
              if (any) {
                if (T < LEAF && mk[T < LEAF ? T : 0] != 0u) {
                  if (open) {
                    row_atomic<G>(a.out, curT, c, mul4(acc, up));
                    acc = rv_zero();
                  }
                  curT = mk[T < LEAF ? T : 0] - 1u;
                  open = true;
                }
#pragma unroll
                for (int l = 0; l < LEAF; ++l)
                  if (l != T && mk[l] != 0u) lr[l] = row_load<G, WIDE>(a.fac[l], mk[l] - 1u, c);
                up = lr[0];
#pragma unroll
                for (int l = 1; l < T && l < LEAF; ++l) up = mul4(up, lr[l]);
                dn = rv_ones();
#pragma unroll
                for (int l = T + 1; l < LEAF; ++l) dn = mul4(dn, lr[l]);
              }
              const float v = __uint_as_float(rr[t].y);
              if (T == LEAF) {
                row_atomic<G>(a.out, rr[t].x, c, scale4(v, up));
              } else {
                fma4(acc, v, mul4(cr[t], dn));
              }
            }
          }
        }
        if (T < LEAF && open) row_atomic<G>(a.out, curT, c, mul4(acc, up));
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
  }
}

// ---------------------------------------------------------------------------------------
// CSL group (Algorithm "CSL-MTTKRP"): every nonzero carries all its non-root indices; the
// slice pointer goes straight to the nonzeros.
// LDS record: N = 3: {j, k, val, slice mark}; N = 4: {a, b, l, val, slice mark, -, -, -};
//             N = 5: {a, b, c, l, val, slice mark, -, -}.
// ---------------------------------------------------------------------------------------
template <int G, int N, int LS, int kSteps, bool WIDE>
__global__ __launch_bounds__(256) void csl_group_kernel(const GroupArgs a) {
  constexpr int NG = 64 / G;
  constexpr int RW = (N == 3) ? 4 : 8;
  extern __shared__ uint32_t lds[];
  const int lane = threadIdx.x & 63;
  const int wib = threadIdx.x >> 6;
  const int wpb = blockDim.x >> 6;
  const int g = lane / G, c = lane % G;
  constexpr uint32_t L = 1u << LS;
  uint32_t* rec = lds + (size_t)wib * (NG * (L + 1) * RW);


  const unsigned long long traceStart = a.trace ? wall_clock64() : 0ull;
  const SpanWalk walk = span_walk(a, wib, wpb);
  for (uint32_t span = walk.first; span < walk.end; span += walk.stride) {
  uint32_t u = span * a.unitsPerWave;
  const uint32_t uEnd = min(u + a.unitsPerWave, a.nUnits);
  rowvec acc = rv_zero();
  bool pend = false;
  uint32_t pendRow = 0;

  UnitBounds cur = load_bounds<G, N, false>(a, u, lane);
  const uint32_t fLo[3] = {0, 0, 0};

  for (; u < uEnd; ++u) {
    const UnitBounds nxt = load_bounds<G, N, false>(a, min(u + 1, a.nUnits - 1), lane);
    const UnitEnds ends = stage_unit<G, N, LS, false>(a, rec, u, cur, fLo, lane);
    const uint32_t headRow = ends.headRow, tailRow = ends.tailRow, ng = ends.ng;
    cur = nxt;

    if (ng > 0) {
      if (pend && pendRow != headRow) {
        row_atomic<G>(a.out, pendRow, c, acc);
        acc = rv_zero();
      }
      const uint32_t* myrec = rec + (size_t)g * (L + 1) * RW;
      for (uint32_t sb = 0; sb < L; sb += kSteps) {
        uint4 rr[kSteps];
        uint32_t vv[kSteps];   // value bits
        uint32_t mi[kSteps];   // slice mark
        rowvec x1[kSteps], x2[kSteps], x3[kSteps], x4[kSteps];
#pragma unroll
        for (int t = 0; t < kSteps; ++t) {
          const uint4* src = reinterpret_cast<const uint4*>(myrec + (size_t)(sb + t) * RW);
          rr[t] = src[0];
          if (N == 3) {
            vv[t] = rr[t].z;
            mi[t] = rr[t].w;
          } else if (N == 4) {
            vv[t] = rr[t].w;
            mi[t] = reinterpret_cast<const uint32_t*>(src)[4];
          } else {
            const uint2 hi = reinterpret_cast<const uint2*>(src)[2];
            vv[t] = hi.x;
            mi[t] = hi.y;
          }
        }
#pragma unroll
        for (int t = 0; t < kSteps; ++t) {
          x1[t] = row_load<G, WIDE>(a.fac[1], rr[t].x, c);
          x2[t] = row_load<G, WIDE>(a.fac[2], rr[t].y, c);
          if (N >= 4) x3[t] = row_load<G, WIDE>(a.fac[3], rr[t].z, c);
          if (N >= 5) x4[t] = row_load<G, WIDE>(a.fac[4], rr[t].w, c);
        }
#pragma unroll
        for (int t = 0; t < kSteps; ++t) {
          rowvec pr = mul4(x1[t], x2[t]);
          if (N >= 4) pr = mul4(pr, x3[t]);
          if (N >= 5) pr = mul4(pr, x4[t]);
          fma4(acc, __uint_as_float(vv[t]), pr);
          if (mi[t]) {
            const uint32_t row = (mi[t] & 0x7fffffffu) - 1u;
            if (mi[t] & 0x80000000u) row_store<G>(a.out, row, c, acc);
            else row_atomic<G>(a.out, row, c, acc);
            acc = rv_zero();
          }
        }
      }
      // the run leaves a partial row behind unless its last nonzero ends a slice
      pend = myrec[(size_t)(ng - 1) * RW + (N == 3 ? 3 : N)] == 0u;
      pendRow = tailRow;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  }
  final_merge<G>(a.out, pend, pendRow, acc, g, c);
  }  // spans
  trace_wave(a, kCslKernel, traceStart, lane);
}

// ---------------------------------------------------------------------------------------
// COO group (Algorithm "COO-MTTKRP" restricted to slices with one nonzero): each nonzero owns
// its output row, so the row is written with a plain store and no atomic is needed.
// Lane group g of a wavefront takes nonzero z = base + step*NG + g.
// ---------------------------------------------------------------------------------------
template <int G, int N, bool WIDE>
__global__ __launch_bounds__(256) void coo_group_kernel(const GroupArgs a) {
  constexpr int NG = 64 / G;
  constexpr int kU = G < 8 ? G : 8;  // nonzeros per lane group in flight
  const int lane = threadIdx.x & 63;
  const int g = lane / G, c = lane % G;
  const uint32_t waves = (gridDim.x * blockDim.x) >> 6;
  const uint32_t wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const uint32_t* __restrict__ valb = reinterpret_cast<const uint32_t*>(a.val);
  // 64 nonzeros per wavefront and iteration: lane l loads the coordinates of nonzero base + l
  // (coalesced), then lane group g takes nonzero base + step*NG + g from lane step*NG + g.
  for (uint64_t base = (uint64_t)wave * 64u; base < a.nnz; base += (uint64_t)waves * 64u) {
    const uint64_t z = base + lane;
    uint32_t m0 = 0, m1 = 0, m2 = 0, m3 = 0, m4 = 0, mv = 0;
    if (z < a.nnz) {
      m0 = __builtin_nontemporal_load(a.ind[0] + z);
      m1 = __builtin_nontemporal_load(a.ind[1] + z);
      m2 = __builtin_nontemporal_load(a.ind[2] + z);
      if (N >= 4) m3 = __builtin_nontemporal_load(a.ind[3] + z);
      if (N >= 5) m4 = __builtin_nontemporal_load(a.ind[4] + z);
      mv = __builtin_nontemporal_load(valb + z);
    }
    const uint32_t left = (uint32_t)min((uint64_t)64, a.nnz - base);
#pragma unroll
    for (int sb = 0; sb < G; sb += kU) {
      uint32_t i0[kU], v[kU];
      rowvec x1[kU], x2[kU], x3[kU], x4[kU];
      bool ok[kU];
#pragma unroll
      for (int t = 0; t < kU; ++t) {
        const int src = (sb + t) * NG + g;
        ok[t] = (uint32_t)src < left;
        i0[t] = __shfl(m0, src);
        v[t] = __shfl(mv, src);
        const uint32_t i1 = __shfl(m1, src), i2 = __shfl(m2, src);
        const uint32_t i3 = N >= 4 ? __shfl(m3, src) : 0u;
        const uint32_t i4 = N >= 5 ? __shfl(m4, src) : 0u;
        if (ok[t]) {
          x1[t] = row_load<G, WIDE>(a.fac[1], i1, c);
          x2[t] = row_load<G, WIDE>(a.fac[2], i2, c);
          if (N >= 4) x3[t] = row_load<G, WIDE>(a.fac[3], i3, c);
          if (N >= 5) x4[t] = row_load<G, WIDE>(a.fac[4], i4, c);
        }
      }
#pragma unroll
      for (int t = 0; t < kU; ++t) {
        if (ok[t]) {
          rowvec pr = mul4(x1[t], x2[t]);
          if (N >= 4) pr = mul4(pr, x3[t]);
          if (N >= 5) pr = mul4(pr, x4[t]);
          row_store<G>(a.out, i0[t], c, scale4(__uint_as_float(v[t]), pr));
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// Output definition fused with the COO group.  The rows of single-nonzero slices are scattered
// thinly over the output (about one row in five on the hypersparse workloads), and writing them
// in a pass of their own costs far more DRAM time per byte than writing them together with the
// zero fill of their neighbours.  One wavefront takes one 32-row word at a time: rows of the
// COO group get v * hadamard(factor rows), rows that nothing else stores get zeros, rows owned
// by a CSL / CSF slice are left alone.  COO nonzeros are stored in row order, so the nonzero of
// a row is cooPtr[word] + (number of COO rows before it in the word).
// ---------------------------------------------------------------------------------------
template <int G, int N, bool WIDE>
__global__ __launch_bounds__(256) void define_coo_kernel(const GroupArgs a, const uint32_t* __restrict__ ownedBits,
                                                         const uint32_t* __restrict__ cooBits,
                                                         const uint32_t* __restrict__ cooPtr, uint64_t rows) {
  constexpr int NG = 64 / G;
  constexpr int RPG = 32 / NG;              // rows of a word per lane group (NG <= 32)
  constexpr int CH = RPG < 4 ? RPG : 4;     // rows per lane group handled together
  const int lane = threadIdx.x & 63;
  const int g = lane / G, c = lane % G;
  const uint32_t waves = (gridDim.x * blockDim.x) >> 6;
  const uint32_t wave = __builtin_amdgcn_readfirstlane((blockIdx.x * blockDim.x + threadIdx.x) >> 6);
  const uint64_t words = (rows + 31) >> 5;
  const uint32_t* __restrict__ valb = reinterpret_cast<const uint32_t*>(a.val);
  for (uint64_t wd = wave; wd < words; wd += waves) {
    const uint32_t wo = ownedBits[wd];
    const uint32_t wc = cooBits[wd];
    const uint32_t zBase = cooPtr[wd];
#pragma unroll
    for (int qb = 0; qb < RPG; qb += CH) {
      uint32_t i1[CH], i2[CH], i3[CH], i4[CH], v[CH];
      bool isCoo[CH], fill[CH];
#pragma unroll
      for (int q = 0; q < CH; ++q) {
        const uint32_t bit = (uint32_t)(g * RPG + qb + q);
        const uint64_t row = (wd << 5) + bit;
        isCoo[q] = ((wc >> bit) & 1u) != 0u;
        fill[q] = row < rows && !isCoo[q] && ((wo >> bit) & 1u) == 0u;
        i1[q] = i2[q] = i3[q] = i4[q] = v[q] = 0;
        if (isCoo[q]) {
          const uint32_t z = zBase + (uint32_t)__builtin_popcount(wc & ((1u << bit) - 1u));
          i1[q] = a.ind[1][z];
          i2[q] = a.ind[2][z];
          if (N >= 4) i3[q] = a.ind[3][z];
          if (N >= 5) i4[q] = a.ind[4][z];
          v[q] = valb[z];
        }
      }
      rowvec x1[CH], x2[CH], x3[CH], x4[CH];
#pragma unroll
      for (int q = 0; q < CH; ++q) {
        if (isCoo[q]) {
          x1[q] = row_load<G, WIDE>(a.fac[1], i1[q], c);
          x2[q] = row_load<G, WIDE>(a.fac[2], i2[q], c);
          if (N >= 4) x3[q] = row_load<G, WIDE>(a.fac[3], i3[q], c);
          if (N >= 5) x4[q] = row_load<G, WIDE>(a.fac[4], i4[q], c);
        }
      }
#pragma unroll
      for (int q = 0; q < CH; ++q) {
        const uint32_t bit = (uint32_t)(g * RPG + qb + q);
        rowvec* dst = reinterpret_cast<rowvec*>(a.out + (((wd << 5) + bit) * (uint64_t)(4 * G) + (uint64_t)(4 * c)));
        if (isCoo[q]) {
          rowvec pr = mul4(x1[q], x2[q]);
          if (N >= 4) pr = mul4(pr, x3[q]);
          if (N >= 5) pr = mul4(pr, x4[q]);
          store_streaming(dst, scale4(__uint_as_float(v[q]), pr));
        } else if (fill[q]) {
          store_streaming(dst, rv_zero());
        }
      }
    }
  }
}

#ifdef HBCSF_F64
}  // namespace f64
using namespace f64;
#endif

// ---------------------------------------------------------------------------------------
// Launch helpers (host)
// ---------------------------------------------------------------------------------------
namespace {

// `grid` carries the number of compute units.  Default launch: one wavefront per span.  Persistent
// launch: (resident blocks per CU) x CUs blocks, capped by the spans.  Both rounded to a multiple of 8.
template <int G, int N, int LS, int S, bool WIDE>
hipError_t launch_one(int kind, const GroupArgs& a, dim3 grid, dim3 block, size_t lds, hipStream_t s) {
  auto csf = (G == 8 && N == 3 && S == 8 && !WIDE) ? csf_group_kernel_occ4<G, N, LS, S> : csf_group_kernel<G, N, LS, S, WIDE>;
  if constexpr (G == 8 && N <= 4 && (LS == 5 || LS == 6)) {
    if (a.denseMid) csf = csf_group_dense_kernel<G, N, LS, S, WIDE>;
  }
  auto csl = csl_group_kernel<G, N, LS, S, WIDE>;
  const int which = kind == kCsfKernel ? 1 : 0;
  const uint32_t wpb = block.x >> 6;
  const uint64_t need = ((uint64_t)a.nSpans + wpb - 1) / wpb;
  uint64_t blocks = need;
  if (a.persistent) {
    // resident blocks per CU of this kernel on the current device (asked per launch: the persistent launch is a
    // tuning variant, and a cached answer would be wrong for another device of the process)
    int n = 0;
    const hipError_t e = which ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, csf, (int)block.x, lds)
                               : hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, csl, (int)block.x, lds);
    if (e != hipSuccess) return e;
    blocks = (uint64_t)grid.x * (uint64_t)(n > 0 ? n : 1);
    if (blocks > need) blocks = need;
  }
  blocks = (blocks + 7) / 8 * 8;
  if (which) hipLaunchKernelGGL(csf, dim3((uint32_t)blocks), block, lds, s, a);
  else hipLaunchKernelGGL(csl, dim3((uint32_t)blocks), block, lds, s, a);
  return hipGetLastError();
}

template <int G, int N, int LS>
hipError_t launch_ls(int kind, int steps, bool wide, const GroupArgs& a, dim3 grid, dim3 block, size_t lds,
                     hipStream_t s) {
  if (G == 8 && steps == 4)
    return wide ? launch_one<G, N, LS, 4, true>(kind, a, grid, block, lds, s)
                : launch_one<G, N, LS, 4, false>(kind, a, grid, block, lds, s);
  return wide ? launch_one<G, N, LS, 8, true>(kind, a, grid, block, lds, s)
              : launch_one<G, N, LS, 8, false>(kind, a, grid, block, lds, s);
}

template <int G, int N>
hipError_t launch_g(int kind, int steps, bool wide, const GroupArgs& a, dim3 grid, dim3 block, size_t lds,
                    hipStream_t s) {
  if (kind == kCooKernel) {
    if (wide) hipLaunchKernelGGL((coo_group_kernel<G, N, true>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((coo_group_kernel<G, N, false>), grid, block, 0, s, a);
    return hipGetLastError();
  }
  switch (a.lshift) {
    case 3: return launch_ls<G, N, 3>(kind, steps, wide, a, grid, block, lds, s);
    case 4: return launch_ls<G, N, 4>(kind, steps, wide, a, grid, block, lds, s);
    case 5: return launch_ls<G, N, 5>(kind, steps, wide, a, grid, block, lds, s);
    case 6: return launch_ls<G, N, 6>(kind, steps, wide, a, grid, block, lds, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

// This file is compiled once per (HBCSF_G, HBCSF_N) pair so that the instantiations build in
// parallel; each object exports one launch function, and the object built with
// HBCSF_WITH_DEFINE also holds the output-definition kernel's launcher.
#ifndef HBCSF_G
#error "compile with -DHBCSF_G=<lanes per row> -DHBCSF_N=<order>"
#endif
#define HBCSF_CAT2(a, b, c, d) a##b##c##d
#define HBCSF_CAT(a, b, c, d) HBCSF_CAT2(a, b, c, d)
#ifdef HBCSF_F64
#define HBCSF_LAUNCH_DEFINE_COO launch_define_coo64_g
#define HBCSF_LAUNCH_GROUP launch_group64_g
#else
#define HBCSF_LAUNCH_DEFINE_COO launch_define_coo_g
#define HBCSF_LAUNCH_GROUP launch_group_g
#endif

hipError_t HBCSF_CAT(HBCSF_LAUNCH_DEFINE_COO, HBCSF_G, _n, HBCSF_N)(bool wide, const GroupArgs& a,
                                                               const uint32_t* ownedBits, const uint32_t* cooBits,
                                                               const uint32_t* cooPtr, uint64_t rows, uint32_t blocks,
                                                               hipStream_t s) {
  if (wide)
    hipLaunchKernelGGL((define_coo_kernel<HBCSF_G, HBCSF_N, true>), dim3(blocks), dim3(256), 0, s, a, ownedBits,
                       cooBits, cooPtr, rows);
  else
    hipLaunchKernelGGL((define_coo_kernel<HBCSF_G, HBCSF_N, false>), dim3(blocks), dim3(256), 0, s, a, ownedBits,
                       cooBits, cooPtr, rows);
  return hipGetLastError();
}

hipError_t HBCSF_CAT(HBCSF_LAUNCH_GROUP, HBCSF_G, _n, HBCSF_N)(int kind, int steps, bool wide, const GroupArgs& a,
                                                          uint32_t blocks, uint32_t threads, size_t ldsBytes,
                                                          hipStream_t s) {
  return launch_g<HBCSF_G, HBCSF_N>(kind, steps, wide, a, dim3(blocks), dim3(threads), ldsBytes, s);
}

#if HBCSF_G == 8 && !defined(HBCSF_F64)
namespace {
template <int N, int LS, int T>
hipError_t launch_nonroot_t(bool wide, const GroupArgs& a, uint32_t threads, size_t lds, hipStream_t s) {
  const uint32_t wpb = threads >> 6;
  const uint64_t blocks = (((uint64_t)a.nSpans + wpb - 1) / wpb + 7) / 8 * 8;
  if (wide) hipLaunchKernelGGL((csf_nonroot_kernel<N, LS, T, true>), dim3((uint32_t)blocks), dim3(threads), lds, s, a);
  else hipLaunchKernelGGL((csf_nonroot_kernel<N, LS, T, false>), dim3((uint32_t)blocks), dim3(threads), lds, s, a);
  return hipGetLastError();
}
}  // namespace

// Single-representation kernel for this object's order: target at tree level `level` (1 .. order-1) of the
// representation in `a` (B-CSF group only, runs of the order's default length), rank 32.
hipError_t HBCSF_CAT(launch_nonroot_n, HBCSF_N, , )(int level, bool wide, const GroupArgs& a, uint32_t threads,
                                                     size_t ldsBytes, hipStream_t s) {
  constexpr int LS = HBCSF_N == 3 ? 6 : 5;
  if (a.lshift != (uint32_t)LS || a.persistent) return hipErrorInvalidValue;
  switch (level) {
    case 1: return launch_nonroot_t<HBCSF_N, LS, 1>(wide, a, threads, ldsBytes, s);
    case 2: return launch_nonroot_t<HBCSF_N, LS, 2>(wide, a, threads, ldsBytes, s);
#if HBCSF_N >= 4
    case 3: return launch_nonroot_t<HBCSF_N, LS, 3>(wide, a, threads, ldsBytes, s);
#endif
#if HBCSF_N >= 5
    case 4: return launch_nonroot_t<HBCSF_N, LS, 4>(wide, a, threads, ldsBytes, s);
#endif
    default: return hipErrorInvalidValue;
  }
}
#endif  // HBCSF_G == 8, fp32

#ifdef HBCSF_WITH_DEFINE
// Plain zero fill of an output every row of which is then reached by atomic adds (the single-representation kernel).
__global__ __launch_bounds__(256) void zero_rows_kernel(rowvec* __restrict__ out, uint64_t nvec) {
  for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (uint64_t)gridDim.x * 256)
    store_streaming(out + i, rv_zero());
}

hipError_t launch_zero_rows(float* out, uint64_t nvec, uint32_t blocks, hipStream_t s) {
  hipLaunchKernelGGL(zero_rows_kernel, dim3(blocks), dim3(256), 0, s, reinterpret_cast<rowvec*>(out), nvec);
  return hipGetLastError();
}

hipError_t launch_define(float* out, const uint32_t* ownedBits, uint64_t rows, int G, uint32_t blocks,
                         hipStream_t s) {
  int gshift = 0;
  while ((1 << gshift) < G) ++gshift;
  hipLaunchKernelGGL(define_rows_kernel, dim3(blocks), dim3(256), 0, s, reinterpret_cast<rowvec*>(out),
                     ownedBits, rows * (uint64_t)G, gshift);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Diagnostic: the row-gather rate the memory system sustains for this access shape (128-byte
// rows, 8 lanes x rowvec, 8 gathers in flight per lane group), with none of the MTTKRP work
// around it.  Used to put a measured ceiling beside the kernels' achieved rates.
// `active` (1..8): load instruction t of a block of 8 is executed by the lane groups g with
// (g - t) mod 8 < active only, the others sit it out, as the lane groups without a segment end
// do in the B-CSF kernel's fiber-row loads; every instruction is still issued by the wavefront.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void probe_gather_kernel(const uint32_t* __restrict__ idx, uint64_t n,
                                                           const float* __restrict__ table,
                                                           float* __restrict__ sink, uint32_t perWave, int active) {
  constexpr int S = 8;
  const int lane = threadIdx.x & 63;
  const int g = lane >> 3, c = lane & 7;
  const uint64_t wave = (uint64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const uint32_t per = perWave / 8;
  uint64_t p = wave * perWave + (uint64_t)g * per;
  const uint64_t pEnd = p + per;
  rowvec acc = rv_zero();
  for (; p + S <= pEnd && p + S <= n; p += S) {
    // one index load per block: lane c of a lane group fetches the index of step c
    const uint32_t mine = idx[p + c];
    uint32_t k[S];
    rowvec r[S];
#pragma unroll
    for (int t = 0; t < S; ++t) k[t] = __shfl(mine, (g << 3) + t);
#pragma unroll
    for (int t = 0; t < S; ++t) {
      r[t] = rv_zero();
      if (((g - t) & 7) < active) r[t] = *reinterpret_cast<const rowvec*>(table + ((size_t)k[t] * 32 + (size_t)(4 * c)));
    }
#pragma unroll
    for (int t = 0; t < S; ++t) {
      acc.x += r[t].x;
      acc.y += r[t].y;
      acc.z += r[t].z;
      acc.w += r[t].w;
    }
  }
  if (acc.x == 123.456f) sink[0] = acc.x + acc.y + acc.z + acc.w;  // keeps the loads alive
}

hipError_t launch_probe_gather(const uint32_t* idx, uint64_t n, const float* table, float* sink,
                               uint32_t waves, uint32_t perWave, int active, hipStream_t s) {
  hipLaunchKernelGGL(probe_gather_kernel, dim3(waves / 4), dim3(256), 0, s, idx, n, table, sink, perWave, active);
  return hipGetLastError();
}
#endif  // HBCSF_WITH_DEFINE

}  // namespace hbcsf
