// Seeded synthetic inputs for sparse-MTTKRP tests and benchmarks.
//
// This file only makes inputs: coordinate lists with power-law (bounded Zipf)
// or uniform index laws, values, and dense factor matrices.  It contains none
// of the MTTKRP arithmetic and is shared by the CPU oracle's tests and the GPU
// library's tests alike.
//
// Every random number is a pure function of (seed, stream, counter), so the
// output does not depend on the thread count.
//
// The stand-in tensors replace the FROSTT / HaTen2 tensors of the paper's
// Table III (3M-144M nonzeros, orders 3-4, strongly skewed slice and fiber
// lengths), which are not available offline.

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <memory>
#include <vector>

#include <omp.h>

namespace {

inline uint64_t mix64(uint64_t z) {
  z += 0x9e3779b97f4a7c15ull;
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
  return z ^ (z >> 31);
}

// Counter-based generator: 64 random bits for (seed, stream, counter).
inline uint64_t rnd64(uint64_t seed, uint64_t stream, uint64_t ctr) {
  return mix64(mix64(seed ^ mix64(stream * 0x632be59bd9b4e019ull + 1)) + ctr * 0x9e3779b97f4a7c15ull);
}

inline double u01(uint64_t x) { return (double)(x >> 11) * (1.0 / 9007199254740992.0); }

// A bijection on 64-bit words and its inverse; used to put the distinct
// coordinates into a deterministic pseudo-random order.
constexpr uint64_t kMulA = 0xbf58476d1ce4e5b9ull;
constexpr uint64_t kMulB = 0x94d049bb133111ebull;

inline uint64_t scramble(uint64_t z) {
  z = (z ^ (z >> 30)) * kMulA;
  z = (z ^ (z >> 27)) * kMulB;
  return z ^ (z >> 31);
}

inline uint64_t inv_odd(uint64_t a) {  // multiplicative inverse modulo 2^64
  uint64_t x = a;
  for (int i = 0; i < 6; ++i) x *= 2 - a * x;
  return x;
}

inline uint64_t unscramble(uint64_t z) {
  static const uint64_t ia = inv_odd(kMulA), ib = inv_odd(kMulB);
  z = z ^ (z >> 31) ^ (z >> 62);
  z *= ib;
  z = z ^ (z >> 27) ^ (z >> 54);
  z *= ia;
  z = z ^ (z >> 30) ^ (z >> 60);
  return z;
}

// Bounded Zipf law on ranks 1..n, P(rank = t) proportional to t^-alpha, sampled
// by inverting the cumulative table with a guide table for O(1) expected cost.
struct IndexLaw {
  uint64_t n = 0;
  bool uniform = true;
  std::vector<double> cdf;      // cdf[t] = P(rank <= t+1)
  std::vector<uint32_t> guide;  // guide[g] = first t with cdf[t] > g/n
  std::vector<uint32_t> perm;   // rank -> index

  void build(uint64_t dim, double alpha, uint64_t seed, uint64_t stream) {
    n = dim;
    uniform = !(alpha > 0.0);
    if (uniform) return;
    cdf.resize(n);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < (int64_t)n; ++t) cdf[t] = std::pow((double)(t + 1), -alpha);
    double acc = 0.0;
    for (uint64_t t = 0; t < n; ++t) { acc += cdf[t]; cdf[t] = acc; }
    const double inv = 1.0 / acc;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < (int64_t)n; ++t) cdf[t] *= inv;
    cdf[n - 1] = 2.0;  // sentinel above any u in [0,1)
    guide.resize(n);
    uint64_t t = 0;
    for (uint64_t g = 0; g < n; ++g) {
      const double u = (double)g / (double)n;
      while (cdf[t] <= u) ++t;
      guide[g] = (uint32_t)t;
    }
    perm.resize(n);
    for (uint64_t i = 0; i < n; ++i) perm[i] = (uint32_t)i;
    for (uint64_t i = n - 1; i > 0; --i) {  // Fisher-Yates
      const uint64_t j = rnd64(seed, stream, i) % (i + 1);
      std::swap(perm[i], perm[j]);
    }
  }

  inline uint32_t sample(double u) const {
    if (uniform) {
      uint64_t i = (uint64_t)(u * (double)n);
      return (uint32_t)(i < n ? i : n - 1);
    }
    uint64_t g = (uint64_t)(u * (double)n);
    if (g >= n) g = n - 1;
    uint64_t t = guide[g];
    while (cdf[t] <= u) ++t;
    return perm[t];
  }
};

inline int bits_for(uint64_t dim) {
  int b = 1;
  while ((1ull << b) < dim) ++b;
  return b;
}

// Parallel least-significant-digit radix sort of 64-bit words.
void radix_sort_u64(std::vector<uint64_t>& a) {
  const size_t n = a.size();
  if (n < 2) return;
  std::vector<uint64_t> b(n);
  const int kBits = 11, kBuckets = 1 << kBits;
  const int nt = omp_get_max_threads();
  std::vector<size_t> hist((size_t)nt * kBuckets);
  uint64_t* src = a.data();
  uint64_t* dst = b.data();
  for (int shift = 0; shift < 64; shift += kBits) {
    std::fill(hist.begin(), hist.end(), 0);
    // chunk numbers, not thread numbers, index the histograms: any team size gives the same result
#pragma omp parallel
    {
#pragma omp for schedule(static, 1)
      for (int c = 0; c < nt; ++c) {
        const size_t lo = n * c / nt, hi = n * (c + 1) / nt;
        size_t* h = &hist[(size_t)c * kBuckets];
        for (size_t i = lo; i < hi; ++i) ++h[(src[i] >> shift) & (kBuckets - 1)];
      }
#pragma omp single
      {
        size_t run = 0;
        for (int d = 0; d < kBuckets; ++d)
          for (int tt = 0; tt < nt; ++tt) {
            size_t c = hist[(size_t)tt * kBuckets + d];
            hist[(size_t)tt * kBuckets + d] = run;
            run += c;
          }
      }
#pragma omp for schedule(static, 1)
      for (int c = 0; c < nt; ++c) {
        const size_t lo = n * c / nt, hi = n * (c + 1) / nt;
        size_t* h = &hist[(size_t)c * kBuckets];
        for (size_t i = lo; i < hi; ++i) dst[h[(src[i] >> shift) & (kBuckets - 1)]++] = src[i];
      }
    }
    std::swap(src, dst);
  }
  if (src != a.data()) std::memcpy(a.data(), src, n * sizeof(uint64_t));
}

}  // namespace

extern "C" {

// Draws coordinates independently per mode (bounded Zipf with exponent
// alpha[m] over a seeded random permutation of 0..dims[m]-1; alpha[m] <= 0
// means uniform), merges duplicates, and writes the distinct coordinates in a
// deterministic pseudo-random order.
//
//   topup = 1: keep drawing until exactly `nnz` distinct coordinates exist and
//              keep the first `nnz` distinct ones in draw order.
//   topup = 0: draw exactly `nnz` coordinates and merge (fewer are stored).
//
// inds[m] must hold room for `nnz` uint32 each, vals for `nnz` floats (values
// are U[-1,1) drawn for the merged set).  Returns 0, or a negative code:
// -1 bad argument, -2 packed coordinate needs more than 63 bits, -3 the index
// space cannot supply `nnz` distinct coordinates within 64*nnz draws.
int synth_tensor(int order, const uint64_t* dims, const double* alpha, uint64_t nnz,
                 uint64_t seed, int topup, uint32_t* const* inds, float* vals,
                 uint64_t* out_nnz, uint64_t* out_draws) {
  if (order < 1 || order > 8 || !dims || !alpha || !inds || !vals || nnz == 0) return -1;
  int bits[8], shift[8], total = 0;
  for (int m = order - 1; m >= 0; --m) {
    if (dims[m] == 0 || dims[m] > 0xffffffffull) return -1;
    bits[m] = bits_for(dims[m]);
    shift[m] = total;
    total += bits[m];
  }
  if (total > 63) return -2;
  long double space = 1.0L;
  for (int m = 0; m < order; ++m) space *= (long double)dims[m];
  if (topup && (long double)nnz > space) return -3;

  std::vector<IndexLaw> law(order);
  for (int m = 0; m < order; ++m) law[m].build(dims[m], alpha[m], seed, 100 + m);

  uint64_t cap = 16;
  while (cap < 2 * nnz) cap <<= 1;
  const uint64_t kEmpty = ~0ull;
  std::unique_ptr<std::atomic<uint64_t>[]> table(new std::atomic<uint64_t>[cap]);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)cap; ++i) table[i].store(kEmpty, std::memory_order_relaxed);

  const int nt = omp_get_max_threads();
  std::vector<std::vector<uint64_t>> fresh(nt);
  uint64_t count = 0, draws = 0;
  const uint64_t max_draws = 64 * nnz + 1024;
  while (count < nnz) {
    // A block of `remaining` draws can add at most `remaining` coordinates, so
    // the count never overshoots and the result is the first nnz distinct
    // coordinates in draw order whatever the thread schedule.
    const uint64_t block = topup ? (nnz - count) : nnz;
    if (draws + block > max_draws) return -3;
    uint64_t added = 0;
#pragma omp parallel num_threads(nt) reduction(+ : added)
    {
      std::vector<uint64_t>& mine = fresh[omp_get_thread_num()];
#pragma omp for schedule(static)
      for (int64_t d = (int64_t)draws; d < (int64_t)(draws + block); ++d) {
        uint64_t key = 0;
        for (int m = 0; m < order; ++m)
          key |= (uint64_t)law[m].sample(u01(rnd64(seed, m, (uint64_t)d))) << shift[m];
        uint64_t h = scramble(key) & (cap - 1);
        for (;;) {
          uint64_t cur = table[h].load(std::memory_order_relaxed);
          if (cur == key) break;
          if (cur == kEmpty) {
            if (table[h].compare_exchange_strong(cur, key, std::memory_order_relaxed)) {
              mine.push_back(key);
              ++added;
              break;
            }
            if (cur == key) break;
          }
          h = (h + 1) & (cap - 1);
        }
      }
    }
    count += added;
    draws += block;
    if (!topup) break;
  }
  table.reset();

  std::vector<uint64_t> keys;
  keys.reserve(count);
  for (auto& f : fresh) {
    keys.insert(keys.end(), f.begin(), f.end());
    std::vector<uint64_t>().swap(f);
  }
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)count; ++i) keys[i] = scramble(keys[i] ^ seed);
  radix_sort_u64(keys);
#pragma omp parallel for schedule(static)
  for (int64_t z = 0; z < (int64_t)count; ++z) {
    const uint64_t key = unscramble(keys[z]) ^ seed;
    for (int m = 0; m < order; ++m)
      inds[m][z] = (uint32_t)((key >> shift[m]) & ((1ull << bits[m]) - 1));
    vals[z] = (float)(2.0 * u01(rnd64(seed, 50, (uint64_t)z)) - 1.0);
  }
  if (out_nnz) *out_nnz = count;
  if (out_draws) *out_draws = draws;
  return 0;
}

// dst[i] = lo + (hi-lo)*U[0,1) for i < n, a pure function of (seed, i).
void synth_fill_uniform(float* dst, uint64_t n, uint64_t seed, float lo, float hi) {
  const double w = (double)hi - (double)lo;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)n; ++i)
    dst[i] = (float)((double)lo + w * u01(rnd64(seed, 60, (uint64_t)i)));
}

uint64_t synth_scramble(uint64_t x) { return scramble(x); }
uint64_t synth_unscramble(uint64_t x) { return unscramble(x); }

}  // extern "C"
