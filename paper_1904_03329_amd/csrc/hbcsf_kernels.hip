// HIP kernels for gfx950 (MI355X): one per HB-CSF slice group plus the output definition.
//
// Mapping (wave64).  One factor row of R = 4G floats is held by G adjacent lanes, a float4
// each, so a wavefront has NG = 64/G lane groups and a row gather is one 16-byte load per
// lane.  The nonzero stream of a group is cut into runs of L nonzeros (L = fiber threshold);
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

constexpr int kSteps = 8;  // records in flight per lane group

__device__ __forceinline__ float4 f4zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }

template <int G>
__device__ __forceinline__ float4 row_load(const float* __restrict__ base, uint32_t row, int c) {
  return *reinterpret_cast<const float4*>(base + ((size_t)row * (size_t)(4 * G) + (size_t)(4 * c)));
}

template <int G>
__device__ __forceinline__ void row_store(float* __restrict__ out, uint32_t row, int c, float4 a) {
  *reinterpret_cast<float4*>(out + ((size_t)row * (size_t)(4 * G) + (size_t)(4 * c))) = a;
}

template <int G>
__device__ __forceinline__ void row_atomic(float* __restrict__ out, uint32_t row, int c, float4 a) {
  float* p = out + ((size_t)row * (size_t)(4 * G) + (size_t)(4 * c));
  unsafeAtomicAdd(p + 0, a.x);
  unsafeAtomicAdd(p + 1, a.y);
  unsafeAtomicAdd(p + 2, a.z);
  unsafeAtomicAdd(p + 3, a.w);
}

__device__ __forceinline__ void fma4(float4& d, float s, const float4& x) {
  d.x = fmaf(s, x.x, d.x);
  d.y = fmaf(s, x.y, d.y);
  d.z = fmaf(s, x.z, d.z);
  d.w = fmaf(s, x.w, d.w);
}

__device__ __forceinline__ void fma4(float4& d, const float4& a, const float4& x) {
  d.x = fmaf(a.x, x.x, d.x);
  d.y = fmaf(a.y, x.y, d.y);
  d.z = fmaf(a.z, x.z, d.z);
  d.w = fmaf(a.w, x.w, d.w);
}

__device__ __forceinline__ float4 mul4(const float4& a, const float4& x) {
  return make_float4(a.x * x.x, a.y * x.y, a.z * x.z, a.w * x.w);
}

__device__ __forceinline__ float4 scale4(float s, const float4& x) {
  return make_float4(s * x.x, s * x.y, s * x.z, s * x.w);
}

// Blocks are dealt round-robin to the 8 XCDs; give each XCD a contiguous part of the stream
// so that one slice's partial rows and its factor rows stay within one L2 where possible.
__device__ __forceinline__ uint32_t logical_block() {
  const uint32_t nb = gridDim.x;  // a multiple of 8
  return (blockIdx.x & 7u) * (nb >> 3) + (blockIdx.x >> 3);
}

// Pending partial row of a lane group, merged at the end of the wavefront's span.
template <int G>
__device__ __forceinline__ void final_merge(float* __restrict__ out, bool pend, uint32_t pendRow,
                                            float4 acc, int g, int c) {
  const uint32_t first = __builtin_amdgcn_readfirstlane(pendRow);
  const bool uniform = __all(pend ? 1 : 0) && __all(pendRow == first ? 1 : 0);
  if (uniform) {
#pragma unroll
    for (int o = G; o < 64; o <<= 1) {
      acc.x += __shfl_xor(acc.x, o);
      acc.y += __shfl_xor(acc.y, o);
      acc.z += __shfl_xor(acc.z, o);
      acc.w += __shfl_xor(acc.w, o);
    }
    if (g == 0) row_atomic<G>(out, pendRow, c, acc);
  } else if (pend) {
    row_atomic<G>(out, pendRow, c, acc);
  }
}

__device__ __forceinline__ uint32_t mark_of_slice(uint32_t si) {
  return ((si & 0x7fffffffu) + 1u) | (si & 0x80000000u);
}

}  // namespace

// ---------------------------------------------------------------------------------------
// Output definition: rows that no plain store will write (empty slices and rows merged with
// atomic adds) are set to zero; the others are left to their single store.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void define_rows_kernel(float4* __restrict__ out,
                                                          const uint32_t* __restrict__ ownedBits,
                                                          uint64_t nvec, int gshift) {
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; t < nvec; t += stride) {
    const uint64_t row = t >> gshift;
    const uint32_t w = ownedBits[row >> 5];
    if (!((w >> (row & 31)) & 1u)) out[t] = f4zero();
  }
}

// ---------------------------------------------------------------------------------------
// B-CSF group.  N = tensor order (3 or 4); G = lanes per factor row.
// LDS record per nonzero: N = 3: {leaf, val, seg1 mark, slice mark};
//                         N = 4: {leaf, val, seg2 mark, seg1 mark, slice mark, -, -, -}.
// A segment mark is index+1 at the segment's last nonzero, else 0.  A slice mark is
// (row+1) | owned bit at the slice's last nonzero, else 0.
// ---------------------------------------------------------------------------------------
template <int G, int N>
__global__ __launch_bounds__(256) void csf_group_kernel(const GroupArgs a) {
  constexpr int NG = 64 / G;
  constexpr int NF = N - 2;
  constexpr int RW = (N == 3) ? 4 : 8;
  extern __shared__ uint32_t lds[];
  const int lane = threadIdx.x & 63;
  const int wib = threadIdx.x >> 6;
  const int wpb = blockDim.x >> 6;
  const int g = lane / G, c = lane % G;
  const uint32_t ls = a.lshift, L = 1u << ls;
  uint32_t* rec = lds + (size_t)wib * (NG * (L + 1) * RW);

  const uint32_t wave = logical_block() * wpb + wib;
  uint32_t u = wave * a.unitsPerWave;
  const uint32_t uEnd = min(u + a.unitsPerWave, a.nUnits);

  const uint32_t* __restrict__ leaf = a.ind[N - 1];
  const uint32_t* __restrict__ valb = reinterpret_cast<const uint32_t*>(a.val);
  const float* __restrict__ facLeaf = a.fac[N - 1];
  const float* __restrict__ facDeep = a.fac[N - 2];   // deepest fiber level
  const float* __restrict__ facTop = a.fac[1];        // level 1 (same as facDeep when N = 3)

  float4 acc = f4zero();
  bool pend = false;
  uint32_t pendRow = 0;

  for (; u < uEnd; ++u) {
    const uint32_t r0 = u * NG;
    const uint32_t z0 = r0 << ls;
    const uint32_t rN = min(r0 + NG, a.runs);

    // -- stage leaf indices and values (coalesced), marks cleared
    for (uint32_t p = lane; p < (uint32_t)NG << ls; p += 64) {
      const uint32_t z = z0 + p;
      uint32_t k = 0, v = 0;
      if (z < a.nnz) {
        k = __builtin_nontemporal_load(leaf + z);
        v = __builtin_nontemporal_load(valb + z);
      }
      uint4* dst = reinterpret_cast<uint4*>(rec + (size_t)(p + (p >> ls)) * RW);
      dst[0] = make_uint4(k, v, 0u, 0u);
      if (N == 4) dst[1] = make_uint4(0u, 0u, 0u, 0u);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    // -- segment end marks
#pragma unroll
    for (int l = 1; l <= NF; ++l) {
      const uint32_t f0 = a.runFirst[l][r0], f1 = a.runFirst[l][rN];
      const int word = 2 + (NF - l);
      for (uint32_t f = f0 + lane; f < f1; f += 64) {
        const uint32_t p = a.ptr[l][f + 1] - 1u - z0;
        rec[(size_t)(p + (p >> ls)) * RW + word] = a.ind[l][f] + 1u;
      }
    }
    // -- slice end marks
    {
      const uint32_t s0 = a.runFirst[0][r0], s1 = a.runFirst[0][rN];
      for (uint32_t s = s0 + lane; s < s1; s += 64) {
        const uint32_t p = a.ptr[0][s + 1] - 1u - z0;
        rec[(size_t)(p + (p >> ls)) * RW + (N == 3 ? 3 : 4)] = mark_of_slice(a.ind[0][s]);
      }
    }
    // -- rows at the two ends of this lane group's run
    const uint32_t r = r0 + g;
    uint32_t headRow = 0, tailRow = 0, ng = 0;
    if (r < a.runs) {
      headRow = a.ind[0][a.runFirst[0][r]] & 0x7fffffffu;
      tailRow = a.ind[0][a.runFirst[0][r + 1]] & 0x7fffffffu;
      ng = min(L, a.nnz - (r << ls));
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

    if (ng > 0) {
      if (pend && pendRow != headRow) {
        row_atomic<G>(a.out, pendRow, c, acc);
        acc = f4zero();
      }
      bool open = true;
      float4 tmp = f4zero();
      float4 tmp1 = f4zero();
      const uint32_t* myrec = rec + (size_t)g * (L + 1) * RW;
      for (uint32_t sb = 0; sb < L; sb += kSteps) {
        uint4 rr[kSteps];
        uint32_t mi[kSteps];
        float4 cr[kSteps], br[kSteps], ar[kSteps];
#pragma unroll
        for (int t = 0; t < kSteps; ++t) {
          const uint4* src = reinterpret_cast<const uint4*>(myrec + (size_t)(sb + t) * RW);
          rr[t] = src[0];
          mi[t] = (N == 3) ? rr[t].w : reinterpret_cast<const uint32_t*>(src)[4];
        }
#pragma unroll
        for (int t = 0; t < kSteps; ++t) cr[t] = row_load<G>(facLeaf, rr[t].x, c);
#pragma unroll
        for (int t = 0; t < kSteps; ++t) {
          if (rr[t].z) br[t] = row_load<G>(facDeep, rr[t].z - 1u, c);
          if (N == 4 && rr[t].w) ar[t] = row_load<G>(facTop, rr[t].w - 1u, c);
        }
#pragma unroll
        for (int t = 0; t < kSteps; ++t) {
          fma4(tmp, __uint_as_float(rr[t].y), cr[t]);
          if (rr[t].z) {
            if (N == 3) {
              fma4(acc, tmp, br[t]);
            } else {
              fma4(tmp1, tmp, br[t]);
              if (rr[t].w) {
                fma4(acc, tmp1, ar[t]);
                tmp1 = f4zero();
              }
            }
            tmp = f4zero();
          }
          if (mi[t]) {
            const uint32_t row = (mi[t] & 0x7fffffffu) - 1u;
            if (mi[t] & 0x80000000u) row_store<G>(a.out, row, c, acc);
            else row_atomic<G>(a.out, row, c, acc);
            acc = f4zero();
          }
          if (sb + t < ng) open = (mi[t] == 0u);
        }
      }
      pend = open;
      pendRow = tailRow;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  }
  final_merge<G>(a.out, pend, pendRow, acc, g, c);
}

// ---------------------------------------------------------------------------------------
// CSL group (Algorithm "CSL-MTTKRP"): every nonzero carries all its non-root indices; the
// slice pointer goes straight to the nonzeros.
// LDS record: N = 3: {j, k, val, slice mark}; N = 4: {a, b, l, val, slice mark, -, -, -}.
// ---------------------------------------------------------------------------------------
template <int G, int N>
__global__ __launch_bounds__(256) void csl_group_kernel(const GroupArgs a) {
  constexpr int NG = 64 / G;
  constexpr int RW = (N == 3) ? 4 : 8;
  extern __shared__ uint32_t lds[];
  const int lane = threadIdx.x & 63;
  const int wib = threadIdx.x >> 6;
  const int wpb = blockDim.x >> 6;
  const int g = lane / G, c = lane % G;
  const uint32_t ls = a.lshift, L = 1u << ls;
  uint32_t* rec = lds + (size_t)wib * (NG * (L + 1) * RW);

  const uint32_t wave = logical_block() * wpb + wib;
  uint32_t u = wave * a.unitsPerWave;
  const uint32_t uEnd = min(u + a.unitsPerWave, a.nUnits);
  const uint32_t* __restrict__ valb = reinterpret_cast<const uint32_t*>(a.val);

  float4 acc = f4zero();
  bool pend = false;
  uint32_t pendRow = 0;

  for (; u < uEnd; ++u) {
    const uint32_t r0 = u * NG;
    const uint32_t z0 = r0 << ls;
    const uint32_t rN = min(r0 + NG, a.runs);
    for (uint32_t p = lane; p < (uint32_t)NG << ls; p += 64) {
      const uint32_t z = z0 + p;
      uint32_t i1 = 0, i2 = 0, i3 = 0, v = 0;
      if (z < a.nnz) {
        i1 = __builtin_nontemporal_load(a.ind[1] + z);
        i2 = __builtin_nontemporal_load(a.ind[2] + z);
        if (N == 4) i3 = __builtin_nontemporal_load(a.ind[3] + z);
        v = __builtin_nontemporal_load(valb + z);
      }
      uint4* dst = reinterpret_cast<uint4*>(rec + (size_t)(p + (p >> ls)) * RW);
      if (N == 3) {
        dst[0] = make_uint4(i1, i2, v, 0u);
      } else {
        dst[0] = make_uint4(i1, i2, i3, v);
        dst[1] = make_uint4(0u, 0u, 0u, 0u);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    {
      const uint32_t s0 = a.runFirst[0][r0], s1 = a.runFirst[0][rN];
      for (uint32_t s = s0 + lane; s < s1; s += 64) {
        const uint32_t p = a.ptr[0][s + 1] - 1u - z0;
        rec[(size_t)(p + (p >> ls)) * RW + (N == 3 ? 3 : 4)] = mark_of_slice(a.ind[0][s]);
      }
    }
    const uint32_t r = r0 + g;
    uint32_t headRow = 0, tailRow = 0, ng = 0;
    if (r < a.runs) {
      headRow = a.ind[0][a.runFirst[0][r]] & 0x7fffffffu;
      tailRow = a.ind[0][a.runFirst[0][r + 1]] & 0x7fffffffu;
      ng = min(L, a.nnz - (r << ls));
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

    if (ng > 0) {
      if (pend && pendRow != headRow) {
        row_atomic<G>(a.out, pendRow, c, acc);
        acc = f4zero();
      }
      bool open = true;
      const uint32_t* myrec = rec + (size_t)g * (L + 1) * RW;
      for (uint32_t sb = 0; sb < L; sb += kSteps) {
        uint4 rr[kSteps];
        uint32_t mi[kSteps];
        float4 x1[kSteps], x2[kSteps], x3[kSteps];
#pragma unroll
        for (int t = 0; t < kSteps; ++t) {
          const uint4* src = reinterpret_cast<const uint4*>(myrec + (size_t)(sb + t) * RW);
          rr[t] = src[0];
          mi[t] = (N == 3) ? rr[t].w : reinterpret_cast<const uint32_t*>(src)[4];
        }
#pragma unroll
        for (int t = 0; t < kSteps; ++t) {
          x1[t] = row_load<G>(a.fac[1], rr[t].x, c);
          x2[t] = row_load<G>(a.fac[2], rr[t].y, c);
          if (N == 4) x3[t] = row_load<G>(a.fac[3], rr[t].z, c);
        }
#pragma unroll
        for (int t = 0; t < kSteps; ++t) {
          float4 pr = mul4(x1[t], x2[t]);
          if (N == 4) pr = mul4(pr, x3[t]);
          fma4(acc, __uint_as_float(N == 3 ? rr[t].z : rr[t].w), pr);
          if (mi[t]) {
            const uint32_t row = (mi[t] & 0x7fffffffu) - 1u;
            if (mi[t] & 0x80000000u) row_store<G>(a.out, row, c, acc);
            else row_atomic<G>(a.out, row, c, acc);
            acc = f4zero();
          }
          if (sb + t < ng) open = (mi[t] == 0u);
        }
      }
      pend = open;
      pendRow = tailRow;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  }
  final_merge<G>(a.out, pend, pendRow, acc, g, c);
}

// ---------------------------------------------------------------------------------------
// COO group (Algorithm "COO-MTTKRP" restricted to slices with one nonzero): each nonzero owns
// its output row, so the row is written with a plain store and no atomic is needed.
// Lane group g of a wavefront takes nonzero z = base + step*NG + g.
// ---------------------------------------------------------------------------------------
template <int G, int N>
__global__ __launch_bounds__(256) void coo_group_kernel(const GroupArgs a) {
  constexpr int NG = 64 / G;
  constexpr int kU = 4;
  const int lane = threadIdx.x & 63;
  const int g = lane / G, c = lane % G;
  const uint32_t waves = (gridDim.x * blockDim.x) >> 6;
  const uint32_t wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const uint32_t* __restrict__ valb = reinterpret_cast<const uint32_t*>(a.val);
  for (uint64_t base = (uint64_t)wave * (NG * kU); base < a.nnz; base += (uint64_t)waves * (NG * kU)) {
    uint32_t i0[kU], i1[kU], i2[kU], i3[kU], v[kU];
    bool ok[kU];
#pragma unroll
    for (int t = 0; t < kU; ++t) {
      const uint64_t z = base + (uint64_t)t * NG + g;
      ok[t] = z < a.nnz;
      i0[t] = i1[t] = i2[t] = i3[t] = v[t] = 0;
      if (ok[t]) {
        i0[t] = a.ind[0][z];
        i1[t] = a.ind[1][z];
        i2[t] = a.ind[2][z];
        if (N == 4) i3[t] = a.ind[3][z];
        v[t] = valb[z];
      }
    }
    float4 x1[kU], x2[kU], x3[kU];
#pragma unroll
    for (int t = 0; t < kU; ++t) {
      if (ok[t]) {
        x1[t] = row_load<G>(a.fac[1], i1[t], c);
        x2[t] = row_load<G>(a.fac[2], i2[t], c);
        if (N == 4) x3[t] = row_load<G>(a.fac[3], i3[t], c);
      }
    }
#pragma unroll
    for (int t = 0; t < kU; ++t) {
      if (ok[t]) {
        float4 pr = mul4(x1[t], x2[t]);
        if (N == 4) pr = mul4(pr, x3[t]);
        row_store<G>(a.out, i0[t], c, scale4(__uint_as_float(v[t]), pr));
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// Launch helpers (host)
// ---------------------------------------------------------------------------------------
namespace {

template <int N>
hipError_t launch_group_n(int kind, int G, const GroupArgs& a, dim3 grid, dim3 block, size_t lds,
                          hipStream_t s) {
#define HBCSF_CASE(GV)                                                                          \
  case GV:                                                                                      \
    if (kind == kCsfKernel) hipLaunchKernelGGL((csf_group_kernel<GV, N>), grid, block, lds, s, a); \
    else if (kind == kCslKernel) hipLaunchKernelGGL((csl_group_kernel<GV, N>), grid, block, lds, s, a); \
    else hipLaunchKernelGGL((coo_group_kernel<GV, N>), grid, block, 0, s, a);                    \
    break;
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
  return hipGetLastError();
}

}  // namespace

hipError_t launch_group(int kind, int order, int G, const GroupArgs& a, uint32_t blocks,
                        uint32_t threads, size_t ldsBytes, hipStream_t s) {
  if (order == 3) return launch_group_n<3>(kind, G, a, dim3(blocks), dim3(threads), ldsBytes, s);
  return launch_group_n<4>(kind, G, a, dim3(blocks), dim3(threads), ldsBytes, s);
}

hipError_t launch_define(float* out, const uint32_t* ownedBits, uint64_t rows, int G, uint32_t blocks,
                         hipStream_t s) {
  int gshift = 0;
  while ((1 << gshift) < G) ++gshift;
  hipLaunchKernelGGL(define_rows_kernel, dim3(blocks), dim3(256), 0, s, reinterpret_cast<float4*>(out),
                     ownedBits, rows * (uint64_t)G, gshift);
  return hipGetLastError();
}

}  // namespace hbcsf
