// CPD-ALS iteration around the MTTKRP kernels (Section II-B, Eq. 1-3, Algorithm "CPD-ALS"): the dense
// steps of a mode update -- Gram matrix of a tall factor, product with the R x R pseudo-inverse -- as gfx950
// kernels, the R x R algebra on the host in fp64, and the C entry points that tie them to hbcsf_mttkrp.
//
// Per mode n the device does three passes over [I_n][R] data: the MTTKRP writes M, gram reads M, apply
// reads M and writes the new factor.  Everything else is R x R work on the host:
//   S = M^T M (device, fp64 accumulators)          V = Hadamard of the other factors' Gram matrices
//   A_n = M V^+                                    hence A_n^T A_n = V^+ S V^+ without another pass.
// The column norms of A_n are the square roots of that matrix's diagonal, so A_n can be written
// normalised in the same pass that computes it.  The algorithm normalises after all modes are updated;
// writing a factor normalised early scales the next MTTKRP's columns by a known diagonal, which the host
// folds back into the R x R matrices (column scaling commutes with every step), so the result is that of
// the algorithm's order up to rounding.

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "hbcsf.h"
#include "hbcsf_tensor.h"

using namespace hbcsf;

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kGramFlush = 4;  // 32-row steps between two flushes of the fp32 partial sums into fp64

// ---------------------------------------------------------------------------------------------------
// Gram matrix S = A^T A of a tall matrix in two steps, without atomics and therefore with the same bits on
// every run: each block writes the partial sums of its rows (all R x R entries, zeros included) to its own
// slot of a scratch buffer, and a second kernel adds the slots in block order.
//
// R = 32: the 32x32x2 fp32 matrix instruction.  One instruction consumes two rows of A: lane
// (h = lane / 32, c = lane % 32) supplies A[row 2u + h][c] as both operands, since the left operand is the
// transpose of the right one.  A wavefront walks a contiguous chunk of rows, sixteen coalesced 256-byte
// loads in flight; partial sums leave fp32 every 128 rows.
// Accumulator register v of a lane holds entry (8 (v / 4) + 4 h + v % 4, c).
// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gram32_partial_kernel(const float* __restrict__ a, uint64_t rows,
                                                             uint64_t rowsPerWave, double* __restrict__ partial) {
  __shared__ double red[4][1024];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int h = lane >> 5, c = lane & 31;
  const uint64_t w = (uint64_t)blockIdx.x * 4 + wave;
  uint64_t r0 = w * rowsPerWave;
  const uint64_t r1 = (r0 + rowsPerWave < rows) ? r0 + rowsPerWave : rows;
  double acc64[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) acc64[v] = 0.0;
  while (r0 < r1) {
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    for (int it = 0; it < kGramFlush && r0 < r1; ++it, r0 += 32) {
      float x[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const uint64_t r = r0 + 2 * u + h;
        x[u] = (r < r1) ? __builtin_nontemporal_load(a + r * 32 + c) : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 16; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(x[u], x[u], acc, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) acc64[v] += (double)acc[v];
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) red[wave][(8 * (v / 4) + 4 * h + (v % 4)) * 32 + c] = acc64[v];
  __syncthreads();
  double* mine = partial + (size_t)blockIdx.x * 1024;
  for (int e = threadIdx.x; e < 1024; e += 256) mine[e] = (red[0][e] + red[1][e]) + (red[2][e] + red[3][e]);
}

// s[e] = sum over the blocks' slots, in block order.  64 entries x 16 interleaved block subsets per workgroup;
// the 16 subset sums are added in a fixed order.
__global__ __launch_bounds__(1024) void gram_reduce_kernel(const double* __restrict__ partial, uint32_t nSlots,
                                                           uint32_t rr, double* __restrict__ s) {
  __shared__ double part[16][64];
  const int el = threadIdx.x & 63, q = threadIdx.x >> 6;
  const uint32_t e = blockIdx.x * 64u + (uint32_t)el;
  double t = 0.0;
  if (e < rr)
    for (uint32_t b = (uint32_t)q; b < nSlots; b += 16) t += partial[(size_t)b * rr + e];
  part[q][el] = t;
  __syncthreads();
  if (q == 0 && e < rr) {
    double sum = 0.0;
#pragma unroll
    for (int k = 0; k < 16; ++k) sum += part[k][el];
    s[e] = sum;
  }
}

// R = 32: out = M P for blocks of 32 rows.  The contraction index is split as k = 16 h + t so that lane
// (h, c) reads the 64 contiguous bytes M[row c of the block][16 h .. 16 h + 15] as its sixteen left
// operands, and holds P[16 h + t][c] as the sixteen right operands for the whole kernel.
__global__ __launch_bounds__(256) void apply32_kernel(const float* __restrict__ m, uint64_t rows,
                                                      const float* __restrict__ p, float* __restrict__ out,
                                                      uint64_t blocksPerWave) {
  const int lane = threadIdx.x & 63;
  const int h = lane >> 5, c = lane & 31;
  float pb[16];
#pragma unroll
  for (int t = 0; t < 16; ++t) pb[t] = p[(16 * h + t) * 32 + c];
  const uint64_t w = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const uint64_t nBlocks = (rows + 31) / 32;
  uint64_t b = w * blocksPerWave;
  const uint64_t bEnd = (b + blocksPerWave < nBlocks) ? b + blocksPerWave : nBlocks;
  for (; b < bEnd; ++b) {
    const uint64_t r = b * 32 + c;
    float4 x[4];
    if (r < rows) {
      const float4* src = reinterpret_cast<const float4*>(m + r * 32 + 16 * h);
#pragma unroll
      for (int q = 0; q < 4; ++q) x[q] = src[q];
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q) x[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(x[q].x, pb[4 * q + 0], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(x[q].y, pb[4 * q + 1], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(x[q].z, pb[4 * q + 2], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(x[q].w, pb[4 * q + 3], acc, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const uint64_t ro = b * 32 + (uint64_t)(8 * (v / 4) + 4 * h + (v % 4));
      if (ro < rows) __builtin_nontemporal_store(acc[v], out + ro * 32 + c);
    }
  }
}

// R = 32: out = M P as apply32_kernel, and in the same pass the Gram matrix of the rows just computed:
// the 32 x 32 product tile leaves the matrix unit as sixteen registers whose lane (h, c) entries are
// out[row 8 (v / 4) + 4 h + v % 4][c], i.e. for every v two different rows of the tile with lane c on
// column c -- exactly the operand shape of gram32_partial_kernel -- so sixteen more matrix instructions
// add the tile's out^T out without moving any data.  The partial Gram sums go to the block's scratch slot
// (reduced by gram_reduce_kernel), so M is read once per mode update instead of twice.
__global__ __launch_bounds__(256) void apply_gram32_kernel(const float* __restrict__ m, uint64_t rows,
                                                           const float* __restrict__ p, float* __restrict__ out,
                                                           uint64_t blocksPerWave, double* __restrict__ partial) {
  __shared__ double red[4][1024];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int h = lane >> 5, c = lane & 31;
  float pb[16];
#pragma unroll
  for (int t = 0; t < 16; ++t) pb[t] = p[(16 * h + t) * 32 + c];
  const uint64_t w = (uint64_t)blockIdx.x * 4 + wave;
  const uint64_t nBlocks = (rows + 31) / 32;
  uint64_t b = w * blocksPerWave;
  const uint64_t bEnd = (b + blocksPerWave < nBlocks) ? b + blocksPerWave : nBlocks;
  double acc64[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) acc64[v] = 0.0;
  while (b < bEnd) {
    f32x16 gacc;
#pragma unroll
    for (int v = 0; v < 16; ++v) gacc[v] = 0.f;
    for (int it = 0; it < kGramFlush && b < bEnd; ++it, ++b) {   // fp32 Gram sums over at most 128 rows
      const uint64_t r = b * 32 + c;
      float4 x[4];
      if (r < rows) {
        const float4* src = reinterpret_cast<const float4*>(m + r * 32 + 16 * h);
#pragma unroll
        for (int q = 0; q < 4; ++q) x[q] = src[q];
      } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) x[q] = make_float4(0.f, 0.f, 0.f, 0.f);
      }
      f32x16 acc;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(x[q].x, pb[4 * q + 0], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(x[q].y, pb[4 * q + 1], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(x[q].z, pb[4 * q + 2], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(x[q].w, pb[4 * q + 3], acc, 0, 0, 0);
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const uint64_t ro = b * 32 + (uint64_t)(8 * (v / 4) + 4 * h + (v % 4));
        if (ro < rows) __builtin_nontemporal_store(acc[v], out + ro * 32 + c);
      }
      // rows past the end of the matrix were computed from zeros and add nothing
#pragma unroll
      for (int v = 0; v < 16; ++v) gacc = __builtin_amdgcn_mfma_f32_32x32x2f32(acc[v], acc[v], gacc, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) acc64[v] += (double)gacc[v];
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) red[wave][(8 * (v / 4) + 4 * h + (v % 4)) * 32 + c] = acc64[v];
  __syncthreads();
  double* mine = partial + (size_t)blockIdx.x * 1024;
  for (int e = threadIdx.x; e < 1024; e += 256) mine[e] = (red[0][e] + red[1][e]) + (red[2][e] + red[3][e]);
}

// a[i][r] *= s[r]: the column normalisation of Algorithm "CPD-ALS" when it was put off (rank = 4 << gshift / ...).
__global__ __launch_bounds__(256) void scale_columns_kernel(float4* __restrict__ a, uint64_t nvec,
                                                            const float* __restrict__ s, int vecPerRow) {
  for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (uint64_t)gridDim.x * 256) {
    const float4 sc = reinterpret_cast<const float4*>(s)[i % (uint64_t)vecPerRow];
    float4 v = a[i];
    v.x *= sc.x; v.y *= sc.y; v.z *= sc.z; v.w *= sc.w;
    a[i] = v;
  }
}

// ---------------------------------------------------------------------------------------------------
// Other ranks: plain vector-ALU kernels (correct for any R in the supported list, not tuned).
// ---------------------------------------------------------------------------------------------------
template <int R>
__global__ __launch_bounds__(256) void gram_generic_partial_kernel(const float* __restrict__ a, uint64_t rows,
                                                                   uint64_t rowsPerBlock, double* __restrict__ partial) {
  constexpr int kTile = 32;                                   // rows staged per step
  constexpr int kPer = (R * R + 255) / 256;                   // entries of S per thread
  __shared__ float tile[kTile][R + 1];
  double acc[kPer];
#pragma unroll
  for (int e = 0; e < kPer; ++e) acc[e] = 0.0;
  uint64_t r0 = (uint64_t)blockIdx.x * rowsPerBlock;
  const uint64_t r1 = (r0 + rowsPerBlock < rows) ? r0 + rowsPerBlock : rows;
  for (; r0 < r1; r0 += kTile) {
    __syncthreads();
    for (int e = threadIdx.x; e < kTile * R; e += 256) {
      const uint64_t r = r0 + (uint64_t)(e / R);
      tile[e / R][e % R] = (r < r1) ? a[r * R + (uint64_t)(e % R)] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
      const int id = threadIdx.x + 256 * e;
      if (id < R * R) {
        const int i = id / R, j = id % R;
        float t = 0.f;
#pragma unroll 8
        for (int k = 0; k < kTile; ++k) t = fmaf(tile[k][i], tile[k][j], t);
        acc[e] += (double)t;
      }
    }
  }
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    const int id = threadIdx.x + 256 * e;
    if (id < R * R) partial[(size_t)blockIdx.x * (R * R) + id] = acc[e];
  }
}

template <int R>
__global__ __launch_bounds__(256) void apply_generic_kernel(const float* __restrict__ m, uint64_t rows,
                                                            const float* __restrict__ p,
                                                            float* __restrict__ out) {
  const uint64_t total = rows * (uint64_t)R;
  for (uint64_t id = (uint64_t)blockIdx.x * 256 + threadIdx.x; id < total; id += (uint64_t)gridDim.x * 256) {
    const uint64_t r = id / R;
    const int c = (int)(id % R);
    float t = 0.f;
#pragma unroll 8
    for (int k = 0; k < R; ++k) t = fmaf(m[r * R + k], p[k * R + c], t);
    out[id] = t;
  }
}

// Scratch of the Gram computation: one R x R fp64 slot per block.  At most kGramSlotsMax blocks, fewer when the
// scratch buffer is smaller; any number of blocks >= 1 gives the same sum up to fp64 rounding.
constexpr uint32_t kGramSlotsMax = 1024;
constexpr uint64_t kGramWorkspaceCap = 32ull << 20;   // hbcsf_gram_workspace_bytes never asks for more

uint32_t gram_slots_for(int rank, uint64_t scratchBytes) {
  const uint64_t fit = scratchBytes / ((uint64_t)rank * rank * 8);
  return (uint32_t)(fit < kGramSlotsMax ? fit : kGramSlotsMax);
}

// s (device, [R][R] fp64) = a^T a; scratch holds `slots` R x R fp64 partial sums (slots >= 1).  Nothing has to be
// cleared between calls: every launched block writes its whole slot, and only the launched blocks' slots are read.
void launch_gram(const float* a, uint64_t rows, int rank, double* scratch, uint32_t slots, double* s, int numCU,
                 hipStream_t st) {
  const uint32_t rr = (uint32_t)(rank * rank);
  uint32_t used = 0;
  if (rows > 0 && rank == 32) {
    // enough wavefronts to cover the memory latency, long enough chunks to amortise the final reduction
    uint64_t waves = (uint64_t)numCU * 16;
    if (waves > (uint64_t)slots * 4) waves = (uint64_t)slots * 4;
    uint64_t per = (rows + waves - 1) / waves;
    per = (per + 31) / 32 * 32;
    if (per < 256) per = 256;
    const uint64_t nWaves = (rows + per - 1) / per;
    used = (uint32_t)((nWaves + 3) / 4);
    hipLaunchKernelGGL(gram32_partial_kernel, dim3(used), dim3(256), 0, st, a, rows, per, scratch);
  } else if (rows > 0) {
    uint64_t blocks = (uint64_t)numCU * 8;
    if (blocks > slots) blocks = slots;
    uint64_t per = (rows + blocks - 1) / blocks;
    per = (per + 31) / 32 * 32;
    used = (uint32_t)((rows + per - 1) / per);
    switch (rank) {
      case 8: hipLaunchKernelGGL(gram_generic_partial_kernel<8>, dim3(used), dim3(256), 0, st, a, rows, per, scratch); break;
      case 16: hipLaunchKernelGGL(gram_generic_partial_kernel<16>, dim3(used), dim3(256), 0, st, a, rows, per, scratch); break;
      case 64: hipLaunchKernelGGL(gram_generic_partial_kernel<64>, dim3(used), dim3(256), 0, st, a, rows, per, scratch); break;
      default: hipLaunchKernelGGL(gram_generic_partial_kernel<128>, dim3(used), dim3(256), 0, st, a, rows, per, scratch); break;
    }
  }
  // with no rows no slot is read and the result is all zeros
  hipLaunchKernelGGL(gram_reduce_kernel, dim3((rr + 63) / 64), dim3(1024), 0, st, scratch, used, rr, s);
}

// R = 32 only: out = m p and g (device, [32][32] fp64) = out^T out in one pass over m.
void launch_apply_gram32(const float* m, uint64_t rows, const float* p, float* out, double* scratch,
                         uint32_t slots, double* g, int numCU, hipStream_t st) {
  uint32_t used = 0;
  if (rows > 0) {
    const uint64_t nBlocks = (rows + 31) / 32;
    uint64_t waves = (uint64_t)numCU * 32;
    if (waves > (uint64_t)slots * 4) waves = (uint64_t)slots * 4;
    const uint64_t per = (nBlocks + waves - 1) / waves;
    const uint64_t nWaves = (nBlocks + per - 1) / per;
    used = (uint32_t)((nWaves + 3) / 4);
    hipLaunchKernelGGL(apply_gram32_kernel, dim3(used), dim3(256), 0, st, m, rows, p, out, per, scratch);
  }
  hipLaunchKernelGGL(gram_reduce_kernel, dim3(16), dim3(1024), 0, st, scratch, used, 1024u, g);
}

void launch_scale_columns(float* a, uint64_t rows, int rank, const float* s, int numCU, hipStream_t st) {
  if (rows == 0) return;
  const uint64_t nvec = rows * (uint64_t)(rank / 4);
  uint64_t blocks = (nvec + 255) / 256;
  const uint64_t cap = (uint64_t)numCU * 32;
  if (blocks > cap) blocks = cap;
  hipLaunchKernelGGL(scale_columns_kernel, dim3((unsigned)blocks), dim3(256), 0, st, reinterpret_cast<float4*>(a),
                     nvec, s, rank / 4);
}

void launch_apply(const float* m, uint64_t rows, int rank, const float* p, float* out, int numCU,
                  hipStream_t st) {
  if (rows == 0) return;
  if (rank == 32) {
    const uint64_t nBlocks = (rows + 31) / 32;
    uint64_t waves = (uint64_t)numCU * 32;
    const uint64_t per = (nBlocks + waves - 1) / waves;
    const uint64_t nWaves = (nBlocks + per - 1) / per;
    hipLaunchKernelGGL(apply32_kernel, dim3((unsigned)((nWaves + 3) / 4)), dim3(256), 0, st, m, rows, p, out,
                       per);
    return;
  }
  const uint64_t total = rows * (uint64_t)rank;
  uint64_t want = (total + 255) / 256;
  const uint64_t cap = (uint64_t)numCU * 64;
  const unsigned grid = (unsigned)(want < cap ? want : cap);
  switch (rank) {
    case 8: hipLaunchKernelGGL(apply_generic_kernel<8>, dim3(grid), dim3(256), 0, st, m, rows, p, out); break;
    case 16: hipLaunchKernelGGL(apply_generic_kernel<16>, dim3(grid), dim3(256), 0, st, m, rows, p, out); break;
    case 64: hipLaunchKernelGGL(apply_generic_kernel<64>, dim3(grid), dim3(256), 0, st, m, rows, p, out); break;
    default: hipLaunchKernelGGL(apply_generic_kernel<128>, dim3(grid), dim3(256), 0, st, m, rows, p, out); break;
  }
}

// ---------------------------------------------------------------------------------------------------
// Host R x R algebra (fp64)
// ---------------------------------------------------------------------------------------------------
using Mat = std::vector<double>;

// Eigen-decomposition of a symmetric matrix by cyclic Jacobi rotations: a = q diag(w) q^T.
void jacobi_eig(Mat a, int n, Mat& q, std::vector<double>& w) {
  q.assign((size_t)n * n, 0.0);
  for (int i = 0; i < n; ++i) q[(size_t)i * n + i] = 1.0;
  for (int sweep = 0; sweep < 60; ++sweep) {
    double off = 0.0, diag = 0.0;
    for (int i = 0; i < n; ++i)
      for (int j = 0; j < n; ++j) (i == j ? diag : off) += a[(size_t)i * n + j] * a[(size_t)i * n + j];
    if (off <= 1e-30 * diag || off == 0.0) break;
    for (int p = 0; p < n - 1; ++p) {
      for (int r = p + 1; r < n; ++r) {
        const double apr = a[(size_t)p * n + r];
        if (apr == 0.0) continue;
        const double theta = (a[(size_t)r * n + r] - a[(size_t)p * n + p]) / (2.0 * apr);
        const double t = (theta >= 0 ? 1.0 : -1.0) / (std::fabs(theta) + std::sqrt(theta * theta + 1.0));
        const double cs = 1.0 / std::sqrt(t * t + 1.0), sn = t * cs;
        for (int k = 0; k < n; ++k) {  // columns p, r
          const double akp = a[(size_t)k * n + p], akr = a[(size_t)k * n + r];
          a[(size_t)k * n + p] = cs * akp - sn * akr;
          a[(size_t)k * n + r] = sn * akp + cs * akr;
        }
        for (int k = 0; k < n; ++k) {  // rows p, r
          const double apk = a[(size_t)p * n + k], ark = a[(size_t)r * n + k];
          a[(size_t)p * n + k] = cs * apk - sn * ark;
          a[(size_t)r * n + k] = sn * apk + cs * ark;
        }
        for (int k = 0; k < n; ++k) {
          const double qkp = q[(size_t)k * n + p], qkr = q[(size_t)k * n + r];
          q[(size_t)k * n + p] = cs * qkp - sn * qkr;
          q[(size_t)k * n + r] = sn * qkp + cs * qkr;
        }
      }
    }
  }
  w.resize(n);
  for (int i = 0; i < n; ++i) w[i] = a[(size_t)i * n + i];
}

// Moore-Penrose pseudo-inverse of a symmetric matrix: eigenvalues below 1e-15 of the largest magnitude
// count as zero (the cut-off numpy.linalg.pinv applies to singular values).
Mat sym_pinv(const Mat& v, int n) {
  Mat q;
  std::vector<double> w;
  jacobi_eig(v, n, q, w);
  double wmax = 0.0;
  for (double x : w) wmax = std::fmax(wmax, std::fabs(x));
  Mat out((size_t)n * n, 0.0);
  for (int k = 0; k < n; ++k) {
    if (std::fabs(w[k]) <= 1e-15 * wmax) continue;
    const double inv = 1.0 / w[k];
    for (int i = 0; i < n; ++i) {
      const double qi = q[(size_t)i * n + k] * inv;
      for (int j = 0; j < n; ++j) out[(size_t)i * n + j] += qi * q[(size_t)j * n + k];
    }
  }
  return out;
}

// Inverse of a symmetric positive definite matrix by Cholesky factorisation; false when a pivot is not
// safely positive (then the caller takes the eigenvalue route, which handles rank deficiency).
bool spd_inverse(const Mat& v, int n, Mat& out) {
  Mat l((size_t)n * n, 0.0);
  double dmax = 0.0;
  for (int i = 0; i < n; ++i) dmax = std::fmax(dmax, v[(size_t)i * n + i]);
  for (int j = 0; j < n; ++j) {
    double d = v[(size_t)j * n + j];
    for (int k = 0; k < j; ++k) d -= l[(size_t)j * n + k] * l[(size_t)j * n + k];
    if (!(d > 1e-10 * dmax)) return false;
    const double ljj = std::sqrt(d);
    l[(size_t)j * n + j] = ljj;
    for (int i = j + 1; i < n; ++i) {
      double x = v[(size_t)i * n + j];
      for (int k = 0; k < j; ++k) x -= l[(size_t)i * n + k] * l[(size_t)j * n + k];
      l[(size_t)i * n + j] = x / ljj;
    }
  }
  // li = l^-1 (lower triangular), then v^-1 = li^T li
  Mat li((size_t)n * n, 0.0);
  for (int c = 0; c < n; ++c) {
    li[(size_t)c * n + c] = 1.0 / l[(size_t)c * n + c];
    for (int i = c + 1; i < n; ++i) {
      double x = 0.0;
      for (int k = c; k < i; ++k) x -= l[(size_t)i * n + k] * li[(size_t)k * n + c];
      li[(size_t)i * n + c] = x / l[(size_t)i * n + i];
    }
  }
  out.assign((size_t)n * n, 0.0);
  for (int i = 0; i < n; ++i)
    for (int j = 0; j <= i; ++j) {
      double x = 0.0;
      for (int k = i; k < n; ++k) x += li[(size_t)k * n + i] * li[(size_t)k * n + j];
      out[(size_t)i * n + j] = x;
      out[(size_t)j * n + i] = x;
    }
  return true;
}

// The pseudo-inverse the update needs: the plain inverse when the matrix is safely positive definite
// (the two coincide there), the eigenvalue form otherwise.
Mat pinv_of_gram_product(const Mat& v, int n) {
  Mat out;
  if (spd_inverse(v, n, out)) return out;
  return sym_pinv(v, n);
}

Mat matmul(const Mat& a, const Mat& b, int n) {
  Mat c((size_t)n * n, 0.0);
  for (int i = 0; i < n; ++i)
    for (int k = 0; k < n; ++k) {
      const double aik = a[(size_t)i * n + k];
      for (int j = 0; j < n; ++j) c[(size_t)i * n + j] += aik * b[(size_t)k * n + j];
    }
  return c;
}

uint64_t round256(uint64_t v) { return (v + 255) / 256 * 256; }

bool rank_ok(int rank) { return rank == 8 || rank == 16 || rank == 32 || rank == 64 || rank == 128; }

}  // namespace

struct hbcsf_als {
  const hbcsf_tensor* t = nullptr;
  int rank = 0;
  float* m = nullptr;    // workspace: MTTKRP output of the mode being updated [max dim][R]
  double* s = nullptr;   // workspace: Gram matrix [R][R]
  double* gramScratch = nullptr;  // workspace: per-block partial sums of the Gram kernel
  uint32_t gramSlots = 0;
  float* p = nullptr;    // workspace: right-hand R x R matrix of the update [R][R], then one [R] column-scale
                         // vector per mode
  double* hostS = nullptr;  // pinned staging
  float* hostP = nullptr;   // pinned staging
  float* hostLambda = nullptr;
  float* hostScale = nullptr;   // pinned staging: [order][R] column factors for the put-off normalisation
  Mat gram[HBCSF_MAX_ORDER];  // Gram matrices of the factors as stored in device memory after the last iteration
  // The algorithm's factor A_m is the stored matrix with column r divided by colScale[m][r].  All ones when
  // the factors were left normalised; the column norms when the normalisation was put off (lazy flag).
  std::vector<double> colScale[HBCSF_MAX_ORDER];
  bool gramsValid = false;
  hipEvent_t ev[HBCSF_MAX_ORDER][5];
  int eventsCreated = 0;  // events are created in order; this many exist
  float phaseMs[4] = {0, 0, 0, 0};  // MTTKRP, Gram (with its read-back), host algebra, apply: last iteration

  hbcsf_als() = default;
  hbcsf_als(const hbcsf_als&) = delete;
  hbcsf_als& operator=(const hbcsf_als&) = delete;
  ~hbcsf_als() {
    if (hostS) (void)hipHostFree(hostS);
    for (int k = 0; k < eventsCreated; ++k) (void)hipEventDestroy(ev[k / 5][k % 5]);
  }
};

// ---------------------------------------------------------------------------------------------------
// Scratch owned by the library, for hbcsf_gram_noalloc: callers that may not allocate device memory (code
// under graph capture, serving loops, harnesses that forbid it) get the Gram computation's partial-sum
// slots from this array instead of a workspace argument.  Every device the library runs on holds its own
// copy, at its own address, until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the address that call returns is what kernels and copies are given.
// ---------------------------------------------------------------------------------------------------
constexpr uint64_t kStaticScratchBytes = 8ull << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
struct DeviceScratch {
  void* ptr = nullptr;  // device address of `scratch` on this device
  int numCU = 0;
};
DeviceScratch g_scratch[kMaxDevices];
std::mutex g_scratchMutex;

int gram_check(const float* a, int rank, const double* s) {
  if (!a || !s) return fail(HBCSF_EINVAL, "null argument");
  if (!rank_ok(rank)) return fail(HBCSF_EINVAL, "rank must be 8, 16, 32, 64 or 128");
  if (((uintptr_t)a & 15) != 0) return fail(HBCSF_EINVAL, "the matrix must be 16-byte aligned");
  if (((uintptr_t)s & 7) != 0) return fail(HBCSF_EINVAL, "the result must be 8-byte aligned");
  return HBCSF_OK;
}

int current_cu_count(int* cu) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
  e = hipDeviceGetAttribute(cu, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return fail_hip(e, "hipDeviceGetAttribute");
  if (*cu <= 0) *cu = 256;
  return HBCSF_OK;
}

}  // namespace

namespace {

// Scales the columns of every stored factor whose normalisation was put off, so that the stored matrices are the
// algorithm's unit-norm factors again; the Gram matrices the state keeps are scaled with them.
int apply_pending_normalisation(hbcsf_als* a, float* const* factors, hipStream_t st) {
  const hbcsf_tensor* t = a->t;
  const int order = t->order, R = a->rank;
  for (int m = 0; m < order; ++m) {
    bool pending = false;
    for (int r = 0; r < R; ++r) pending = pending || a->colScale[m][r] != 1.0;
    if (!pending) continue;
    float* hs = a->hostScale + (size_t)m * R;
    float* ds = a->p + (size_t)R * R + (size_t)m * R;
    for (int r = 0; r < R; ++r) hs[r] = (float)(1.0 / a->colScale[m][r]);
    hipError_t e = hipMemcpyAsync(ds, hs, (size_t)R * 4, hipMemcpyHostToDevice, st);
    if (e != hipSuccess) return fail_hip(e, "hipMemcpyAsync");
    launch_scale_columns(factors[m], t->dims[m], R, ds, t->numCU, st);
    e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(e, "column scaling kernel launch");
    if (a->gramsValid)
      for (int i = 0; i < R; ++i)
        for (int j = 0; j < R; ++j) a->gram[m][(size_t)i * R + j] /= a->colScale[m][i] * a->colScale[m][j];
    a->colScale[m].assign((size_t)R, 1.0);
  }
  return HBCSF_OK;
}

}  // namespace

extern "C" {

int hbcsf_gram_workspace_bytes(int rank, uint64_t* bytes) try {
  if (!bytes) return fail(HBCSF_EINVAL, "null argument");
  if (!rank_ok(rank)) return fail(HBCSF_EINVAL, "rank must be 8, 16, 32, 64 or 128");
  *bytes = (uint64_t)gram_slots_for(rank, kGramWorkspaceCap) * (uint64_t)rank * rank * 8;
  return HBCSF_OK;
} HBCSF_CATCH_ALL

int hbcsf_gram(const float* a, uint64_t rows, int rank, void* workspace, uint64_t workspace_bytes, double* s,
               void* hip_stream) try {
  const int rc = gram_check(a, rank, s);
  if (rc != HBCSF_OK) return rc;
  if (!workspace) return fail(HBCSF_EINVAL, "null argument");
  if (((uintptr_t)workspace & 255) != 0) return fail(HBCSF_EINVAL, "workspace must be 256-byte aligned");
  const uint32_t slots = gram_slots_for(rank, workspace_bytes);
  if (slots == 0) return fail(HBCSF_ENOMEM, "workspace holds less than one rank x rank fp64 matrix");
  int cu = 0;
  const int rd = current_cu_count(&cu);
  if (rd != HBCSF_OK) return rd;
  launch_gram(a, rows, rank, (double*)workspace, slots, s, cu, (hipStream_t)hip_stream);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail_hip(e, "Gram kernel launch");
  return HBCSF_OK;
} HBCSF_CATCH_ALL

int hbcsf_gram_noalloc(const float* a, uint64_t rows, int rank, double* s, void* hip_stream) try {
  const int rc = gram_check(a, rank, s);
  if (rc != HBCSF_OK) return rc;
  if ((uint64_t)rank * rank * 8 > kStaticScratchBytes)
    return fail(HBCSF_EINVAL, "rank is beyond what the library's own scratch holds (one rank x rank fp64 slot)");
  int dev = 0, cu = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(HBCSF_EINVAL, "device ordinal beyond the library's per-device table");
  DeviceScratch& d = g_scratch[dev];
  {
    // once per device, with that device current: the array's address on this device (each device has its own copy)
    std::lock_guard<std::mutex> lock(g_scratchMutex);
    if (!d.ptr) {
      void* p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess) return fail_hip(e, "hipGetSymbolAddress");
      if (!p || ((uintptr_t)p & 255) != 0) return fail(HBCSF_EHIP, "the scratch array has no usable device address");
      e = hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev);
      if (e != hipSuccess) return fail_hip(e, "hipDeviceGetAttribute");
      d.numCU = cu > 0 ? cu : 256;
      d.ptr = p;
    }
  }
  launch_gram(a, rows, rank, (double*)d.ptr, gram_slots_for(rank, kStaticScratchBytes), s, d.numCU,
              (hipStream_t)hip_stream);
  e = hipGetLastError();
  if (e != hipSuccess) return fail_hip(e, "Gram kernel launch");
  return HBCSF_OK;
} HBCSF_CATCH_ALL

int hbcsf_als_workspace_bytes(const hbcsf_tensor* t, int rank, uint64_t* bytes) try {
  if (!t || !bytes) return fail(HBCSF_EINVAL, "null argument");
  if (!rank_ok(rank)) return fail(HBCSF_EINVAL, "rank must be 8, 16, 32, 64 or 128");
  uint64_t maxDim = 0;
  for (int m = 0; m < t->order; ++m) maxDim = t->dims[m] > maxDim ? t->dims[m] : maxDim;
  uint64_t gramBytes = 0;
  (void)hbcsf_gram_workspace_bytes(rank, &gramBytes);
  *bytes = round256(maxDim * (uint64_t)rank * 4) + round256((uint64_t)rank * rank * 8) +
           round256(((uint64_t)rank * rank + (uint64_t)HBCSF_MAX_ORDER * rank) * 4) + round256(gramBytes);
  return HBCSF_OK;
} HBCSF_CATCH_ALL

int hbcsf_als_create(const hbcsf_tensor* t, int rank, void* workspace, uint64_t workspace_bytes,
                     hbcsf_als** out) try {
  if (!out) return fail(HBCSF_EINVAL, "out is null");
  *out = nullptr;
  if (!t || !workspace) return fail(HBCSF_EINVAL, "null argument");
  if (!t->uploaded) return fail(HBCSF_ESTATE, "hbcsf_upload has not been called");
  uint64_t need = 0;
  const int rc = hbcsf_als_workspace_bytes(t, rank, &need);
  if (rc != HBCSF_OK) return rc;
  if (workspace_bytes < need) return fail(HBCSF_ENOMEM, "workspace is smaller than hbcsf_als_workspace_bytes");
  if (((uintptr_t)workspace & 255) != 0) return fail(HBCSF_EINVAL, "workspace must be 256-byte aligned");
  std::unique_ptr<hbcsf_als> a(new (std::nothrow) hbcsf_als);
  if (!a) return fail(HBCSF_ENOMEM, "out of host memory");
  a->t = t;
  a->rank = rank;
  uint64_t maxDim = 0;
  for (int m = 0; m < t->order; ++m) maxDim = t->dims[m] > maxDim ? t->dims[m] : maxDim;
  uint8_t* w = (uint8_t*)workspace;
  a->m = (float*)w;
  w += round256(maxDim * (uint64_t)rank * 4);
  a->s = (double*)w;
  w += round256((uint64_t)rank * rank * 8);
  a->p = (float*)w;
  w += round256(((uint64_t)rank * rank + (uint64_t)HBCSF_MAX_ORDER * rank) * 4);
  a->gramScratch = (double*)w;
  uint64_t gramBytes = 0;
  (void)hbcsf_gram_workspace_bytes(rank, &gramBytes);
  a->gramSlots = gram_slots_for(rank, gramBytes);
  const size_t rr = (size_t)rank * rank;
  hipError_t e = hipHostMalloc((void**)&a->hostS,
                               rr * 8 + HBCSF_MAX_ORDER * rr * 4 + (size_t)rank * 4 + (size_t)HBCSF_MAX_ORDER * rank * 4,
                               hipHostMallocDefault);
  if (e != hipSuccess) return fail_hip(e, "hipHostMalloc");
  a->hostP = (float*)(a->hostS + rr);
  a->hostLambda = a->hostP + HBCSF_MAX_ORDER * rr;
  a->hostScale = a->hostLambda + rank;
  for (int m = 0; m < t->order; ++m) a->colScale[m].assign((size_t)rank, 1.0);
  for (int k = 0; k < HBCSF_MAX_ORDER * 5; ++k) {
    e = hipEventCreate(&a->ev[k / 5][k % 5]);
    if (e != hipSuccess) return fail_hip(e, "hipEventCreate");  // the destructor releases what exists
    a->eventsCreated = k + 1;
  }
  *out = a.release();
  return HBCSF_OK;
} HBCSF_CATCH_ALL

int hbcsf_als_iteration(hbcsf_als* a, float* const* factors, float* lambda, int flags, double* fit,
                        void* hip_stream) try {
  if (!a || !factors) return fail(HBCSF_EINVAL, "null argument");
  const hbcsf_tensor* t = a->t;
  const int order = t->order, R = a->rank;
  const size_t rr = (size_t)R * R;
  for (int m = 0; m < order; ++m)
    if (!factors[m]) return fail(HBCSF_EINVAL, "a factor pointer is null");
  if (flags & ~(HBCSF_ALS_KEEP_GRAMS | HBCSF_ALS_LAZY_NORMALISATION)) return fail(HBCSF_EINVAL, "unknown flag");
  const bool lazy = (flags & HBCSF_ALS_LAZY_NORMALISATION) != 0;
  // the product kernel that also forms the new factor's Gram matrix exists for R = 32
  const bool fused = lazy && R == 32;
  hipStream_t st = (hipStream_t)hip_stream;
  hipError_t e;

  auto gram_to_host = [&](const float* src, uint64_t rows, Mat& dst) -> int {
    launch_gram(src, rows, R, a->gramScratch, a->gramSlots, a->s, t->numCU, st);
    e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(e, "Gram kernel launch");
    e = hipMemcpyAsync(a->hostS, a->s, rr * 8, hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) return fail_hip(e, "hipMemcpyAsync");
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return fail_hip(e, "hipStreamSynchronize");
    dst.assign(a->hostS, a->hostS + rr);
    return HBCSF_OK;
  };

  // Gram matrices of the factors that are read before they are updated (all but the first mode's).  Without
  // the keep flag the caller may have replaced the factors: they are then taken as they are (scale 1).
  if (!(flags & HBCSF_ALS_KEEP_GRAMS) || !a->gramsValid) {
    for (int m = 0; m < order; ++m) a->colScale[m].assign((size_t)R, 1.0);
    for (int m = 1; m < order; ++m) {
      const int rc = gram_to_host(factors[m], t->dims[m], a->gram[m]);
      if (rc != HBCSF_OK) return rc;
    }
  }
  a->gramsValid = false;

  // Book-keeping: the algorithm's current factor A_m is stored_m diag(1 / c_m) with c_m = colScale[m]; algGram[m]
  // is its Gram matrix.  Column scaling commutes with every step of the update, so the device works on the
  // stored matrices and the host folds the diagonals into the R x R matrices.
  Mat norms[HBCSF_MAX_ORDER];
  Mat algGram[HBCSF_MAX_ORDER];
  for (int m = 1; m < order; ++m) {
    algGram[m] = a->gram[m];
    for (int i = 0; i < R; ++i)
      for (int j = 0; j < R; ++j) algGram[m][(size_t)i * R + j] /= a->colScale[m][i] * a->colScale[m][j];
  }
  double inner = 0.0;

  for (int n = 0; n < order; ++n) {
    const float* facs[HBCSF_MAX_ORDER];
    for (int m = 0; m < order; ++m) facs[m] = factors[m];
    (void)hipEventRecord(a->ev[n][0], st);
    const int rc = hbcsf_mttkrp(t, n, R, facs, a->m, st);
    if (rc != HBCSF_OK) return rc;
    (void)hipEventRecord(a->ev[n][1], st);
    // M of the algorithm = M of the device diag(d), d_r = product over the other modes of 1 / c_m[r]
    std::vector<double> d((size_t)R, 1.0);
    for (int m = 0; m < order; ++m)
      if (m != n)
        for (int r = 0; r < R; ++r) d[r] /= a->colScale[m][r];
    Mat V(rr, 1.0);
    for (int m = 0; m < order; ++m)
      if (m != n)
        for (size_t k = 0; k < rr; ++k) V[k] *= algGram[m][k];
    float* hostP = a->hostP + (size_t)n * rr;  // one staging copy per mode: no wait before it is reused
    norms[n].assign(R, 1.0);
    if (fused) {
      // A_n = M V^+ written unnormalised, its Gram matrix G formed in the same pass; <X, model> = trace(M^T A_n)
      // = trace(V G) because V^+ V V^+ = V^+.
      (void)hipEventRecord(a->ev[n][2], st);
      const Mat Vp = pinv_of_gram_product(V, R);
      for (int i = 0; i < R; ++i)
        for (int j = 0; j < R; ++j) hostP[(size_t)i * R + j] = (float)(d[i] * Vp[(size_t)i * R + j]);
      (void)hipEventRecord(a->ev[n][3], st);
      e = hipMemcpyAsync(a->p, hostP, rr * 4, hipMemcpyHostToDevice, st);
      if (e != hipSuccess) return fail_hip(e, "hipMemcpyAsync");
      launch_apply_gram32(a->m, t->dims[n], a->p, factors[n], a->gramScratch, a->gramSlots, a->s, t->numCU, st);
      e = hipGetLastError();
      if (e != hipSuccess) return fail_hip(e, "product kernel launch");
      e = hipMemcpyAsync(a->hostS, a->s, rr * 8, hipMemcpyDeviceToHost, st);
      if (e != hipSuccess) return fail_hip(e, "hipMemcpyAsync");
      e = hipStreamSynchronize(st);
      if (e != hipSuccess) return fail_hip(e, "hipStreamSynchronize");
      (void)hipEventRecord(a->ev[n][4], st);
      algGram[n].assign(a->hostS, a->hostS + rr);
      a->gram[n] = algGram[n];                 // stored = the algorithm's unnormalised factor
      a->colScale[n].assign((size_t)R, 1.0);
      for (int r = 0; r < R; ++r) {
        const double g = algGram[n][(size_t)r * R + r];
        norms[n][r] = g > 0.0 ? std::sqrt(g) : 1.0;
      }
      if (n == order - 1) {
        inner = 0.0;
        for (size_t k = 0; k < rr; ++k) inner += V[k] * algGram[n][k];   // both symmetric: trace(V G)
      }
    } else {
      Mat S;
      const int rg = gram_to_host(a->m, t->dims[n], S);
      if (rg != HBCSF_OK) return rg;
      (void)hipEventRecord(a->ev[n][2], st);
      for (int i = 0; i < R; ++i)
        for (int j = 0; j < R; ++j) S[(size_t)i * R + j] *= d[i] * d[j];
      const Mat Vp = pinv_of_gram_product(V, R);
      algGram[n] = matmul(matmul(Vp, S, R), Vp, R);   // A_n^T A_n = V^+ S V^+ without another pass
      for (int r = 0; r < R; ++r) {
        const double g = algGram[n][(size_t)r * R + r];
        norms[n][r] = g > 0.0 ? std::sqrt(g) : 1.0;
      }
      // the factor is written with unit-norm columns at once: stored = A_n diag(1 / norms), so c_n = 1 / norms
      // until the algorithm's closing normalisation makes it 1
      for (int i = 0; i < R; ++i)
        for (int j = 0; j < R; ++j) hostP[(size_t)i * R + j] = (float)(d[i] * Vp[(size_t)i * R + j] / norms[n][j]);
      if (n == order - 1) {
        inner = 0.0;  // <X, model> = trace(M^T A_n) = trace(S V^+)
        for (int i = 0; i < R; ++i)
          for (int j = 0; j < R; ++j) inner += S[(size_t)i * R + j] * Vp[(size_t)j * R + i];
      }
      (void)hipEventRecord(a->ev[n][3], st);
      e = hipMemcpyAsync(a->p, hostP, rr * 4, hipMemcpyHostToDevice, st);
      if (e != hipSuccess) return fail_hip(e, "hipMemcpyAsync");
      launch_apply(a->m, t->dims[n], R, a->p, factors[n], t->numCU, st);
      e = hipGetLastError();
      if (e != hipSuccess) return fail_hip(e, "apply kernel launch");
      (void)hipEventRecord(a->ev[n][4], st);
      a->gram[n] = algGram[n];
      for (int i = 0; i < R; ++i)
        for (int j = 0; j < R; ++j) a->gram[n][(size_t)i * R + j] /= norms[n][i] * norms[n][j];
      for (int r = 0; r < R; ++r) a->colScale[n][r] = 1.0 / norms[n][r];
    }
  }

  // lambda: product over the modes of the column norms; the model's squared norm from the Gram matrices of the
  // unnormalised factors
  double modelSq = 0.0;
  for (size_t k = 0; k < rr; ++k) {
    double prod = 1.0;
    for (int m = 0; m < order; ++m) prod *= algGram[m][k];
    modelSq += prod;
  }
  // the algorithm's closing normalisation: A_m <- A_m diag(1 / norms_m), i.e. c_m <- c_m norms_m
  std::vector<double> lam((size_t)R, 1.0);
  for (int m = 0; m < order; ++m)
    for (int r = 0; r < R; ++r) {
      a->colScale[m][r] *= norms[m][r];
      if (std::fabs(a->colScale[m][r] - 1.0) < 1e-12) a->colScale[m][r] = 1.0;   // written normalised already
      lam[r] *= norms[m][r];
    }
  a->gramsValid = true;
  if (!lazy) {
    const int rn = apply_pending_normalisation(a, factors, st);
    if (rn != HBCSF_OK) return rn;
  }
  if (lambda) {
    for (int r = 0; r < R; ++r) a->hostLambda[r] = (float)lam[r];
    e = hipMemcpyAsync(lambda, a->hostLambda, (size_t)R * 4, hipMemcpyHostToDevice, st);
    if (e != hipSuccess) return fail_hip(e, "hipMemcpyAsync");
  }
  e = hipStreamSynchronize(st);
  if (e != hipSuccess) return fail_hip(e, "hipStreamSynchronize");
  if (fit) {
    const double res = t->normSq - 2.0 * inner + modelSq;
    *fit = t->normSq > 0.0 ? 1.0 - std::sqrt(res > 0.0 ? res : 0.0) / std::sqrt(t->normSq) : 0.0;
  }
  for (int k = 0; k < 4; ++k) a->phaseMs[k] = 0.f;
  for (int n = 0; n < order; ++n)
    for (int k = 0; k < 4; ++k) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, a->ev[n][k], a->ev[n][k + 1]) == hipSuccess) a->phaseMs[k] += ms;
    }
  return HBCSF_OK;
} HBCSF_CATCH_ALL

int hbcsf_als_normalise(hbcsf_als* a, float* const* factors, void* hip_stream) try {
  if (!a || !factors) return fail(HBCSF_EINVAL, "null argument");
  for (int m = 0; m < a->t->order; ++m)
    if (!factors[m]) return fail(HBCSF_EINVAL, "a factor pointer is null");
  const int rc = apply_pending_normalisation(a, factors, (hipStream_t)hip_stream);
  if (rc != HBCSF_OK) return rc;
  const hipError_t e = hipStreamSynchronize((hipStream_t)hip_stream);
  if (e != hipSuccess) return fail_hip(e, "hipStreamSynchronize");
  return HBCSF_OK;
} HBCSF_CATCH_ALL

int hbcsf_als_run(hbcsf_als* a, float* const* factors, float* lambda, int max_iterations, double tolerance,
                  int* iterations_done, double* fit, void* hip_stream) try {
  if (!a || !factors) return fail(HBCSF_EINVAL, "null argument");
  if (max_iterations < 1) return fail(HBCSF_EINVAL, "max_iterations must be at least 1");
  double prev = 0.0, cur = 0.0;
  int it = 0;
  for (; it < max_iterations; ++it) {
    const int rc = hbcsf_als_iteration(a, factors, lambda,
                                       (it > 0 ? HBCSF_ALS_KEEP_GRAMS : 0) | HBCSF_ALS_LAZY_NORMALISATION, &cur,
                                       hip_stream);
    if (rc != HBCSF_OK) return rc;
    if (it > 0 && std::fabs(cur - prev) < tolerance) {
      ++it;
      break;
    }
    prev = cur;
  }
  const int rn = hbcsf_als_normalise(a, factors, hip_stream);
  if (rn != HBCSF_OK) return rn;
  if (iterations_done) *iterations_done = it;
  if (fit) *fit = cur;
  return HBCSF_OK;
} HBCSF_CATCH_ALL

int hbcsf_sym_pinv(const double* v, int n, double* out) try {
  if (!v || !out) return fail(HBCSF_EINVAL, "null argument");
  if (n < 1 || n > 128) return fail(HBCSF_EINVAL, "n must be in 1 .. 128");
  const Mat in(v, v + (size_t)n * n);
  const Mat r = pinv_of_gram_product(in, n);
  std::memcpy(out, r.data(), (size_t)n * n * sizeof(double));
  return HBCSF_OK;
} HBCSF_CATCH_ALL

int hbcsf_als_phase_ms(const hbcsf_als* a, float ms[4]) try {
  if (!a || !ms) return fail(HBCSF_EINVAL, "null argument");
  for (int k = 0; k < 4; ++k) ms[k] = a->phaseMs[k];
  return HBCSF_OK;
} HBCSF_CATCH_ALL

void hbcsf_als_free(hbcsf_als* a) { delete a; }

}  // extern "C"
