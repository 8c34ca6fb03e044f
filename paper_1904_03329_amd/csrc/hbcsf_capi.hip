// C-ABI layer: argument checks, device arena bookkeeping and kernel launches.

#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <memory>
#include <new>
#include <string>
#include <vector>

#include "hbcsf.h"
#include "hbcsf_device.h"
#include "hbcsf_internal.h"
#include "hbcsf_tensor.h"

using namespace hbcsf;

namespace {

thread_local std::string g_err;

}  // namespace

namespace hbcsf {

int fail(int code, const std::string& msg) {
  g_err = msg;
  return code;
}

int fail_hip(hipError_t e, const char* what) {
  g_err = std::string(what) + ": " + hipGetErrorString(e);
  return HBCSF_EHIP;
}

int fail_exception() noexcept {
  int code = HBCSF_EINVAL;
  try {
    try {
      throw;
    } catch (const std::bad_alloc&) {
      code = HBCSF_ENOMEM;
      g_err = "out of host memory";
    } catch (const std::exception& e) {
      g_err = std::string("unexpected C++ exception: ") + e.what();
    } catch (...) {
      g_err = "unexpected C++ exception";
    }
  } catch (...) {
    g_err.clear();  // even the message could not be stored
  }
  return code;
}

}  // namespace hbcsf

namespace {

bool pow2_in(uint32_t v, uint32_t lo, uint32_t hi) { return v >= lo && v <= hi && (v & (v - 1)) == 0; }

uint32_t round_up8(uint64_t v) { return (uint32_t)((v + 7) / 8 * 8); }

// Single representation: mode-`mode` MTTKRP from mode 0's B-CSF tree, the target at tree level T >= 1.  The
// output is zero-filled, then every level-T segment (T = leaf: every nonzero) adds its contribution atomically.
int mttkrp_from_mode0(const hbcsf_tensor* t, int mode, int rank, const float* const* factors, float* out,
                      hipStream_t s) {
  if (rank != 32) return fail(HBCSF_EINVAL, "single representation: modes other than 0 need rank 32");
  if (!factors[0]) return fail(HBCSF_EINVAL, "a factor pointer is null");
  const ModeFormat& f = *t->modes[0];
  const int N = t->order;
  const int G = 8, NG = 8;
  int level = 0;
  for (int l = 1; l < N; ++l)
    if (f.levelMode[l] == mode) level = l;
  if (level == 0) return fail(HBCSF_EINVAL, "mode out of range");
  const uint8_t* base = t->arena + f.devOffset;
  const GroupFormat& gf = f.g[kCsf];
  const uint64_t nvec = t->dims[mode] * (uint64_t)G;
  uint64_t zb = (nvec + 255) / 256;
  const uint64_t cap = (uint64_t)t->numCU * 32;
  if (zb > cap) zb = cap;
  if (zb == 0) zb = 1;
  hipError_t e = launch_zero_rows(out, nvec, (uint32_t)zb, s);
  if (e != hipSuccess) return fail_hip(e, "launch of the zero-fill kernel");
  if (gf.nnz == 0) return HBCSF_OK;
  GroupArgs a;
  std::memset(&a, 0, sizeof(a));
  bool wide = false;
  for (int l = 0; l < N; ++l) {
    a.ind[l] = gf.ind[l].present ? (const uint32_t*)(base + gf.ind[l].off) : nullptr;
    a.ptr[l] = gf.ptr[l].present ? (const uint32_t*)(base + gf.ptr[l].off) : nullptr;
    a.runFirst[l] = gf.runFirst[l].present ? (const uint32_t*)(base + gf.runFirst[l].off) : nullptr;
    a.fac[l] = l == level ? nullptr : factors[f.levelMode[l]];
    if (l != level) wide = wide || t->dims[f.levelMode[l]] * (uint64_t)rank * 4ull >= (1ull << 32);
  }
  uint32_t lshift = 0;
  while ((1u << lshift) < f.L) ++lshift;
  a.val = (const float*)(base + gf.val.off);
  a.out = out;
  a.nnz = (uint32_t)gf.nnz;
  a.runs = (uint32_t)gf.runs;
  a.lshift = lshift;
  a.nUnits = (uint32_t)((gf.runs + NG - 1) / NG);
  const uint64_t target = (uint64_t)t->numCU * (t->wavesPerCU ? t->wavesPerCU : 128);
  uint64_t upw = t->sliceThreshold ? t->sliceThreshold / ((uint64_t)NG * f.L) : (a.nUnits + target - 1) / target;
  if (upw == 0) upw = 1;
  a.unitsPerWave = (uint32_t)upw;
  a.nSpans = (uint32_t)((a.nUnits + upw - 1) / upw);
  const int RW = N == 3 ? 4 : 8;
  const size_t ldsWave = (size_t)NG * (f.L + 1) * RW * 4;
  int wpb = 4;
  while (wpb > 1 && ldsWave * wpb > 48 * 1024) wpb >>= 1;
  const uint32_t threads = 64 * wpb;
  e = N == 3   ? launch_nonroot_n3(level, wide, a, threads, ldsWave * wpb, s)
      : N == 4 ? launch_nonroot_n4(level, wide, a, threads, ldsWave * wpb, s)
               : launch_nonroot_n5(level, wide, a, threads, ldsWave * wpb, s);
  if (e != hipSuccess) return fail_hip(e, "launch of the single-representation kernel");
  return HBCSF_OK;
}

}  // namespace

extern "C" {

int hbcsf_build_format(int order, const uint64_t* dims, uint64_t nnz, const uint32_t* const* inds,
                       const float* vals, const hbcsf_opts* opts, hbcsf_tensor** out) try {
  if (!out) return fail(HBCSF_EINVAL, "out is null");
  *out = nullptr;
  if (order < 3 || order > HBCSF_MAX_ORDER) return fail(HBCSF_EINVAL, "order must be 3, 4 or 5");
  if (!dims) return fail(HBCSF_EINVAL, "dims is null");
  if (nnz > 0 && (!inds || !vals)) return fail(HBCSF_EINVAL, "inds or vals is null");
  if (nnz >= 0xffff0000ull) return fail(HBCSF_ERANGE, "nnz must be below 2^32 - 2^16");
  for (int m = 0; m < order; ++m) {
    if (dims[m] == 0 || dims[m] > 0x7ffffffeull) return fail(HBCSF_ERANGE, "each dimension must be in 1 .. 2^31-2");
    if (nnz > 0 && !inds[m]) return fail(HBCSF_EINVAL, "an index array is null");
  }
  hbcsf_opts o{};
  if (opts) o = *opts;
  if (o.fiber_threshold == 0) o.fiber_threshold = default_fiber_threshold(order);
  if (!pow2_in(o.fiber_threshold, 8, 64)) return fail(HBCSF_EINVAL, "fiber_threshold must be 8, 16, 32 or 64");
  if (o.mode_order_policy > 2) return fail(HBCSF_EINVAL, "mode_order_policy must be 0, 1 or 2");
  if (o.group_mask > 4) return fail(HBCSF_EINVAL, "group_mask must be 0..4");
  if (o.hybrid_granularity > 1) return fail(HBCSF_EINVAL, "hybrid_granularity must be 0 or 1");
  if (o.coo_row_flags > 1) return fail(HBCSF_EINVAL, "coo_row_flags must be 0 or 1");
  if (o.mid_blocking > 13) return fail(HBCSF_EINVAL, "mid_blocking must be 0 or 1 (off) or 2..13 bits");
  if (o.single_representation > 1) return fail(HBCSF_EINVAL, "single_representation must be 0 or 1");
  if (o.single_representation) {
    if ((opts->fiber_threshold && opts->fiber_threshold != default_fiber_threshold(order)) || o.group_mask ||
        o.hybrid_granularity || o.coo_row_flags || o.mid_blocking > 1)
      return fail(HBCSF_EINVAL, "single_representation goes with default options only");
    o.group_mask = 4;  // plain B-CSF: the kernel for the other modes walks one group
  }
  std::unique_ptr<hbcsf_tensor> t(new (std::nothrow) hbcsf_tensor);
  if (!t) return fail(HBCSF_ENOMEM, "out of host memory");
  t->order = order;
  t->nnz = nnz;
  t->opts = o;
  t->sliceThreshold = o.slice_threshold;
  t->steps = default_steps(order);
  for (int m = 0; m < order; ++m) t->dims[m] = dims[m];
  double sq = 0.0;
  for (uint64_t z = 0; z < nnz; ++z) sq += (double)vals[z] * (double)vals[z];
  t->normSq = sq;
  t->single = o.single_representation == 1;
  uint64_t off = 0;
  for (int m = 0; m < (t->single ? 1 : order); ++m) {
    t->modes[m].reset(new (std::nothrow) ModeFormat);
    if (!t->modes[m]) return fail(HBCSF_ENOMEM, "out of host memory");
    std::string err;
    const int rc = build_mode(order, dims, nnz, inds, vals, o, m, t->modes[m].get(), &err);
    if (rc != HBCSF_OK) return fail(rc, err);
    t->modes[m]->devOffset = off;
    off += t->modes[m]->blobBytes;
  }
  t->arenaBytes = off;
  *out = t.release();
  return HBCSF_OK;
} HBCSF_CATCH_ALL

int hbcsf_device_bytes(const hbcsf_tensor* t, uint64_t* bytes) try {
  if (!t || !bytes) return fail(HBCSF_EINVAL, "null argument");
  *bytes = t->arenaBytes;
  return HBCSF_OK;
} HBCSF_CATCH_ALL

int hbcsf_upload(hbcsf_tensor* t, void* device_arena, uint64_t bytes, void* hip_stream) try {
  if (!t || !device_arena) return fail(HBCSF_EINVAL, "null argument");
  const int nModes = t->single ? 1 : t->order;
  for (int m = 0; m < nModes; ++m)
    if (!t->modes[m]->blob) return fail(HBCSF_ESTATE, "the format was built on the device: it is already resident");
  if (bytes < t->arenaBytes) return fail(HBCSF_ENOMEM, "device arena is smaller than hbcsf_device_bytes");
  if (((uintptr_t)device_arena & (kAlign - 1)) != 0) return fail(HBCSF_EINVAL, "device arena must be 256-byte aligned");
  hipStream_t s = (hipStream_t)hip_stream;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
  int cu = 0;
  e = hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return fail_hip(e, "hipDeviceGetAttribute");
  t->numCU = cu > 0 ? cu : 256;
  for (int m = 0; m < nModes; ++m) {
    const ModeFormat& f = *t->modes[m];
    e = hipMemcpyAsync((uint8_t*)device_arena + f.devOffset, f.blob, f.blobBytes, hipMemcpyHostToDevice, s);
    if (e != hipSuccess) return fail_hip(e, "hipMemcpyAsync");
  }
  e = hipStreamSynchronize(s);
  if (e != hipSuccess) return fail_hip(e, "hipStreamSynchronize");
  t->arena = (uint8_t*)device_arena;
  t->uploaded = true;
  return HBCSF_OK;
} HBCSF_CATCH_ALL

}  // extern "C"

namespace {

// The MTTKRP of both element types: `elem` = bytes per element of the factor matrices and the output (4: fp32,
// 8: fp64; the tensor's values are fp32 either way).  The kernels see a row as G = rank * elem / 16 lanes of 16 bytes
// and GroupArgs' float pointers as row addresses, so everything below the launch dispatch is shared.
int mttkrp_any(const hbcsf_tensor* t, int mode, int rank, int elem, const float* const* factors, float* out,
               void* hip_stream) {
  if (!t || !factors || !out) return fail(HBCSF_EINVAL, "null argument");
  if (mode < 0 || mode >= t->order) return fail(HBCSF_EINVAL, "mode out of range");
  const bool f64 = elem == 8;
  if (!f64 && !(rank == 8 || rank == 16 || rank == 32 || rank == 64 || rank == 128))
    return fail(HBCSF_EINVAL, "rank must be 8, 16, 32, 64 or 128");
  if (f64 && !(rank == 16 || rank == 32 || rank == 64)) return fail(HBCSF_EINVAL, "fp64: rank must be 16, 32 or 64");
  if (f64 && t->single) return fail(HBCSF_EINVAL, "fp64: the single-representation variant is fp32 only");
  if (!t->uploaded) return fail(HBCSF_ESTATE, "hbcsf_upload has not been called");
  if (((uintptr_t)out & 15) != 0) return fail(HBCSF_EINVAL, "out must be 16-byte aligned");
  for (int m = 0; m < t->order; ++m) {
    if (m == mode) continue;
    if (!factors[m]) return fail(HBCSF_EINVAL, "a factor pointer is null");
    if (((uintptr_t)factors[m] & 15) != 0) return fail(HBCSF_EINVAL, "factors must be 16-byte aligned");
  }
  if (t->single && mode != 0) return mttkrp_from_mode0(t, mode, rank, factors, out, (hipStream_t)hip_stream);
  const ModeFormat& f = *t->modes[mode];
  const int N = t->order;
  const int G = rank * elem / 16;
  const int NG = 64 / G;
  const uint32_t L = f.L;
  uint32_t lshift = 0;
  while ((1u << lshift) < L) ++lshift;
  hipStream_t s = (hipStream_t)hip_stream;
  const uint8_t* base = t->arena + f.devOffset;
  const uint64_t rowBytes = (uint64_t)rank * (uint64_t)elem;
  hipError_t e;

  hbcsf_tensor::EventSet* es = nullptr;
  if (!t->ring.empty()) {
    es = &t->ring[t->calls % t->ring.size()];
    es->valid = false;
    e = hipEventRecord(es->ev[0], s);
    if (e != hipSuccess) return fail_hip(e, "hipEventRecord");
  }

  auto group_args = [&](int g) {
    const GroupFormat& gf = f.g[g];
    GroupArgs a;
    std::memset(&a, 0, sizeof(a));
    for (int l = 0; l < N; ++l) {
      a.ind[l] = gf.ind[l].present ? (const uint32_t*)(base + gf.ind[l].off) : nullptr;
      a.ptr[l] = gf.ptr[l].present ? (const uint32_t*)(base + gf.ptr[l].off) : nullptr;
      a.runFirst[l] = gf.runFirst[l].present ? (const uint32_t*)(base + gf.runFirst[l].off) : nullptr;
      a.fac[l] = l == 0 ? nullptr : factors[f.levelMode[l]];
    }
    return a;
  };
  bool wide = false;  // some gathered factor matrix needs 64-bit row addressing
  for (int l = 1; l < N; ++l) wide = wide || t->dims[f.levelMode[l]] * rowBytes >= (1ull << 32);

  // 1. define every output row that no plain store will write; the COO group's rows are written
  //    in the same pass
  // (measured: the fused pass saves a launch on small outputs but hides latency worse on large ones)
  // (without stored root indices only the fused pass can place the COO group's rows)
  const bool wantFuse = f.cooRowFlags || t->fuseCoo == 1 ||
                        (t->fuseCoo == 2 && f.rows * rowBytes <= (64ull << 20));
  const bool fuseCoo = wantFuse && (t->kernelMask & 3u) == 3u && f.g[kCoo].nnz > 0;
  if (t->kernelMask & 1u) {
    // one wavefront per 8 x 32 rows, capped at 64 wavefronts per compute unit
    uint64_t blocks = ((f.rows + 255) / 256 + 3) / 4;
    const uint64_t cap = (uint64_t)t->numCU * 16;
    if (blocks > cap) blocks = cap;
    if (blocks == 0) blocks = 1;
    if (fuseCoo) {
      blocks = ((f.rows + 31) / 32 + 3) / 4;  // the fused pass takes one 32-row word per wavefront iteration
      if (blocks > cap) blocks = cap;
      if (blocks == 0) blocks = 1;
      GroupArgs a = group_args(kCoo);
      a.val = (const float*)(base + f.g[kCoo].val.off);
      a.out = out;
      a.nnz = (uint32_t)f.g[kCoo].nnz;
      e = launch_define_coo(f64, N, G, wide, a, (const uint32_t*)(base + f.ownedBits.off),
                            (const uint32_t*)(base + f.cooBits.off), (const uint32_t*)(base + f.cooPtr.off),
                            f.rows, (uint32_t)blocks, s);
    } else {
      e = launch_define(out, (const uint32_t*)(base + f.ownedBits.off), f.rows, G, (uint32_t)blocks, s);
    }
    if (e != hipSuccess) return fail_hip(e, "launch of the output-definition kernel");
    if (es) es->launched[0] = true;
  } else if (es) {
    es->launched[0] = false;
  }
  if (es) (void)hipEventRecord(es->ev[1], s);

  // 2. the three group kernels (execute step of Algorithm "HB-CSF-MTTKRP")
  for (int g = 0; g < 3; ++g) {
    const GroupFormat& gf = f.g[g];
    bool launched = false;
    if (gf.nnz > 0 && (t->kernelMask & (2u << g)) && !(g == kCoo && (fuseCoo || f.cooRowFlags))) {
      GroupArgs a = group_args(g);
      a.val = (const float*)(base + gf.val.off);
      a.out = out;
      a.nnz = (uint32_t)gf.nnz;
      a.runs = (uint32_t)gf.runs;
      a.lshift = lshift;
      a.nUnits = (uint32_t)((gf.runs + NG - 1) / NG);
      a.trace = t->trace;
      a.traceCapacity = (uint32_t)t->traceCapacity;
      uint32_t blocks, threads;
      size_t lds = 0;
      if (g == kCoo) {
        threads = 256;
        const uint64_t perBlock = 64 * 4;  // 64 nonzeros per wavefront and iteration
        uint64_t b = (gf.nnz + perBlock - 1) / perBlock;
        const uint64_t cap = (uint64_t)t->numCU * 16;
        if (b > cap) b = cap;
        blocks = round_up8(b);
        a.unitsPerWave = 0;
      } else {
        int RW = N == 3 ? 4 : 8;  // LDS words per nonzero record
        size_t ldsWave = (size_t)NG * (L + 1) * RW * 4;
        // B-CSF tuning variant: the fiber-level rows gathered densely through an LDS row cache (off by default:
        // it lowered the vector-memory instruction count as intended but lengthened every block's dependent chain
        // and measured 40-100 % slower on the benchmark tensors)
        a.denseMid = 0;
        if (g == kCsf && t->denseMid == 1 && dense_mid_available(N, G, lshift)) {
          a.denseMid = 1;
          ldsWave += dense_mid_lds_bytes(G);
        } else if (g == kCsf && N == 4) {
          // the order-4 B-CSF kernel packs a record into 4 words and keeps the slices' rows in a list of NG * L words
          RW = 4;
          ldsWave = (size_t)NG * (L + 1) * RW * 4 + (size_t)NG * L * 4;
        }
        int wpb = 4;
        while (wpb > 1 && ldsWave * wpb > 48 * 1024) wpb >>= 1;
        threads = 64 * wpb;
        lds = ldsWave * wpb;
        uint64_t upw;
        if (t->sliceThreshold) {
          upw = t->sliceThreshold / ((uint64_t)NG * L);
        } else {
          const uint64_t target = (uint64_t)t->numCU * (t->wavesPerCU ? t->wavesPerCU : 128);
          upw = (a.nUnits + target - 1) / target;
        }
        if (upw == 0) upw = 1;
        a.unitsPerWave = (uint32_t)upw;
        a.nSpans = (uint32_t)((a.nUnits + upw - 1) / upw);
        a.persistent = t->persistent ? 1u : 0u;
        a.streamLevel = 0;
        if (g == kCsf)
          for (int l = 1; l < N - 1; ++l)
            if (t->dims[f.levelMode[l]] * rowBytes >= t->streamBytes) a.streamLevel |= 1u << l;
        blocks = (uint32_t)t->numCU;  // the launcher sizes the grid
      }
      e = launch_group(f64, g, N, G, t->steps, wide, a, blocks, threads, lds, s);
      if (e != hipSuccess) return fail_hip(e, "launch of a group kernel");
      launched = true;
    }
    if (es) {
      es->launched[1 + g] = launched;
      (void)hipEventRecord(es->ev[2 + g], s);
    }
  }
  if (es) {
    es->valid = true;
    ++t->calls;
  }
  return HBCSF_OK;
}

}  // namespace

extern "C" {

int hbcsf_mttkrp(const hbcsf_tensor* t, int mode, int rank, const float* const* factors, float* out,
                 void* hip_stream) try {
  return mttkrp_any(t, mode, rank, 4, factors, out, hip_stream);
} HBCSF_CATCH_ALL

int hbcsf_mttkrp_f64(const hbcsf_tensor* t, int mode, int rank, const double* const* factors, double* out,
                     void* hip_stream) try {
  return mttkrp_any(t, mode, rank, 8, reinterpret_cast<const float* const*>(factors), reinterpret_cast<float*>(out),
                    hip_stream);
} HBCSF_CATCH_ALL

int hbcsf_get_stats(const hbcsf_tensor* t, int mode, hbcsf_stats* stats) try {
  if (!t || !stats) return fail(HBCSF_EINVAL, "null argument");
  if (mode < 0 || mode >= t->order) return fail(HBCSF_EINVAL, "mode out of range");
  if (t->single && mode != 0) return fail(HBCSF_ESTATE, "single representation: only mode 0 is stored");
  *stats = t->modes[mode]->stats;
  return HBCSF_OK;
} HBCSF_CATCH_ALL

int hbcsf_host_array(const hbcsf_tensor* t, int mode, int group, int level, int array_id,
                     const void** ptr, uint64_t* count) try {
  if (!t || !ptr || !count) return fail(HBCSF_EINVAL, "null argument");
  if (mode < 0 || mode >= t->order) return fail(HBCSF_EINVAL, "mode out of range");
  if (t->single && mode != 0) return fail(HBCSF_ESTATE, "single representation: only mode 0 is stored");
  const ModeFormat& f = *t->modes[mode];
  const ArrayRef* r = nullptr;
  if (array_id == HBCSF_ARR_OWNED_BITS) {
    r = &f.ownedBits;
  } else if (array_id == HBCSF_ARR_COO_BITS) {
    r = &f.cooBits;
  } else if (array_id == HBCSF_ARR_COO_PTR) {
    r = &f.cooPtr;
  } else {
    if (group < 0 || group > 2 || level < 0 || level >= t->order) return fail(HBCSF_EINVAL, "group or level out of range");
    const GroupFormat& g = f.g[group];
    if (array_id == HBCSF_ARR_IND) r = &g.ind[level];
    else if (array_id == HBCSF_ARR_PTR) r = &g.ptr[level];
    else if (array_id == HBCSF_ARR_VAL) r = &g.val;
    else if (array_id == HBCSF_ARR_RUNFIRST) r = &g.runFirst[level];
  }
  if (!r || !r->present) return fail(HBCSF_EINVAL, "this group has no such array");
  if (!f.blob) return fail(HBCSF_ESTATE, "the format was built on the device: call hbcsf_download first");
  *ptr = f.blob + r->off;
  *count = r->count;
  return HBCSF_OK;
} HBCSF_CATCH_ALL

int hbcsf_tune(hbcsf_tensor* t, int key, uint64_t value) try {
  if (!t) return fail(HBCSF_EINVAL, "null argument");
  if (key == HBCSF_TUNE_SLICE_THRESHOLD) {
    t->sliceThreshold = value;
    return HBCSF_OK;
  }
  if (key == HBCSF_TUNE_PROFILE) {
    if (value > 65536) return fail(HBCSF_EINVAL, "at most 65536 profiled calls are kept");
    for (auto& es : t->ring)
      for (int i = 0; i < 5; ++i) (void)hipEventDestroy(es.ev[i]);
    t->ring.clear();
    t->calls = 0;
    t->ring.resize((size_t)value);
    size_t made = 0;  // events created so far, in ring order
    for (auto& es : t->ring)
      for (int i = 0; i < 5; ++i, ++made) {
        hipError_t e = hipEventCreate(&es.ev[i]);
        if (e != hipSuccess) {
          for (size_t k = 0; k < made; ++k) (void)hipEventDestroy(t->ring[k / 5].ev[k % 5]);
          t->ring.clear();
          return fail_hip(e, "hipEventCreate");
        }
      }
    return HBCSF_OK;
  }
  if (key == HBCSF_TUNE_WAVES_PER_CU) {
    if (value > 1024) return fail(HBCSF_EINVAL, "waves per CU must be at most 1024");
    t->wavesPerCU = value;
    return HBCSF_OK;
  }
  if (key == HBCSF_TUNE_TRACE_BUFFER) {
    if (value & 7) return fail(HBCSF_EINVAL, "the trace buffer must be 8-byte aligned");
    t->trace = (unsigned long long*)(uintptr_t)value;
    if (!t->trace) t->traceCapacity = 0;
    return HBCSF_OK;
  }
  if (key == HBCSF_TUNE_TRACE_CAPACITY) {
    if (value > 0xffffffffull) return fail(HBCSF_EINVAL, "trace capacity too large");
    t->traceCapacity = value;
    return HBCSF_OK;
  }
  if (key == HBCSF_TUNE_STREAM_BYTES) {
    t->streamBytes = value ? value : ~0ull;  // 0 = never
    return HBCSF_OK;
  }
  if (key == HBCSF_TUNE_FUSE_COO) {
    if (value > 2) return fail(HBCSF_EINVAL, "fuse mode must be 0, 1 or 2");
    t->fuseCoo = (int)value;
    return HBCSF_OK;
  }
  if (key == HBCSF_TUNE_PERSISTENT) {
    t->persistent = value != 0;
    return HBCSF_OK;
  }
  if (key == HBCSF_TUNE_KERNEL_MASK) {
    if (value > 15) return fail(HBCSF_EINVAL, "kernel mask must be 0..15");
    t->kernelMask = (uint32_t)value;
    return HBCSF_OK;
  }
  if (key == HBCSF_TUNE_DENSE_MID) {
    if (value > 1) return fail(HBCSF_EINVAL, "dense-gather mode must be 0 or 1");
    t->denseMid = (int)value;
    return HBCSF_OK;
  }
  if (key == HBCSF_TUNE_STEPS) {
    if (value != 4 && value != 8) return fail(HBCSF_EINVAL, "steps must be 4 or 8");
    t->steps = (int)value;
    return HBCSF_OK;
  }
  return fail(HBCSF_EINVAL, "unknown tuning key");
} HBCSF_CATCH_ALL

int hbcsf_kernel_ms(hbcsf_tensor* t, uint32_t calls_back, float ms[4]) try {
  if (!t || !ms) return fail(HBCSF_EINVAL, "null argument");
  if (t->ring.empty() || calls_back >= t->ring.size() || calls_back >= t->calls)
    return fail(HBCSF_ESTATE, "no profiled hbcsf_mttkrp call that far back");
  const hbcsf_tensor::EventSet& es = t->ring[(t->calls - 1 - calls_back) % t->ring.size()];
  if (!es.valid) return fail(HBCSF_ESTATE, "that call did not complete its launches");
  hipError_t e = hipEventSynchronize(es.ev[4]);
  if (e != hipSuccess) return fail_hip(e, "hipEventSynchronize");
  for (int i = 0; i < 4; ++i) {
    ms[i] = 0.f;
    if (!es.launched[i]) continue;
    e = hipEventElapsedTime(&ms[i], es.ev[i], es.ev[i + 1]);
    if (e != hipSuccess) return fail_hip(e, "hipEventElapsedTime");
  }
  return HBCSF_OK;
} HBCSF_CATCH_ALL

int hbcsf_probe_row_gather(const uint32_t* idx, uint64_t n, const float* table, uint64_t table_rows,
                           int active_lane_groups, float* sink, void* hip_stream, uint64_t* rows_gathered,
                           uint64_t* load_instructions) try {
  if (!idx || !table || !sink || !rows_gathered) return fail(HBCSF_EINVAL, "null argument");
  if (active_lane_groups < 1 || active_lane_groups > 8) return fail(HBCSF_EINVAL, "active lane groups must be 1..8");
  if (table_rows == 0 || n < 64 * 1024) return fail(HBCSF_EINVAL, "need a table and at least 65536 indices");
  int dev = 0, cu = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
  e = hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return fail_hip(e, "hipDeviceGetAttribute");
  uint64_t waves = (uint64_t)(cu > 0 ? cu : 256) * 64;
  uint64_t perWave = n / waves / 64 * 64;
  while (perWave == 0 && waves > 4) {
    waves /= 2;
    perWave = n / waves / 64 * 64;
  }
  waves = waves / 4 * 4;
  if (perWave == 0 || waves == 0) return fail(HBCSF_EINVAL, "too few indices");
  e = launch_probe_gather(idx, n, table, sink, (uint32_t)waves, (uint32_t)perWave, active_lane_groups,
                          (hipStream_t)hip_stream);
  if (e != hipSuccess) return fail_hip(e, "launch of the gather probe");
  *rows_gathered = waves * perWave / 8 * (uint64_t)active_lane_groups;
  if (load_instructions) *load_instructions = waves * perWave / 8;  // row loads: one per 8 index entries walked
  return HBCSF_OK;
} HBCSF_CATCH_ALL

void hbcsf_free(hbcsf_tensor* t) {
  if (!t) return;
  for (auto& es : t->ring)
    for (int i = 0; i < 5; ++i) (void)hipEventDestroy(es.ev[i]);
  delete t;
}

const char* hbcsf_strerror(int code) {
  switch (code) {
    case HBCSF_OK: return "ok";
    case HBCSF_EINVAL: return "invalid argument";
    case HBCSF_ERANGE: return "index or size out of range";
    case HBCSF_ENOMEM: return "out of memory or arena too small";
    case HBCSF_ESTATE: return "call out of order";
    case HBCSF_EHIP: return "HIP call failed";
    default: return "unknown error code";
  }
}

const char* hbcsf_last_error(void) { return g_err.c_str(); }

}  // extern "C"
