// Host-side format builder: COO -> per-mode HB-CSF (Sections III-B, IV, V).
//
// For the root mode n the nonzeros are sorted by (root, middle level(s), leaf) index, which
// gives the compressed-sparse-fiber tree (Section III-B).  Each slice is then put into one of
// three groups (Section V and Section VI-D: one nonzero -> COO; every fiber a single nonzero
// -> CSL; otherwise CSF).  Inside the CSL and CSF groups the group's nonzero stream is cut
// into runs of T_f nonzeros: a fiber is cut wherever it crosses a run boundary (fbr-split,
// Sections IV-B and VI-B, so no segment exceeds T_f nonzeros), and a slice that crosses a run
// boundary is handled by several lane groups whose partial rows are merged with atomic adds
// (slc-split, Section IV-A: slices stay whole in the arrays, more workers are assigned).
// The run tables say which slice / segment holds the first nonzero of each run.

#include "hbcsf_internal.h"

#include <algorithm>
#include <chrono>
#include <cstring>
#include <memory>

#include <omp.h>

namespace hbcsf {
namespace {

// Stable parallel LSD radix sort of (key, payload) pairs on the low `totalBits` bits.
// On return k / v point at the sorted data (either the first or the second buffer pair).
template <typename Key>
void radix_sort_pairs(Key*& k, uint32_t*& v, Key*& k2, uint32_t*& v2, size_t n, int totalBits) {
  if (n < 2 || totalBits <= 0) return;
  const int passes = (totalBits + 11) / 12;
  const int digit = (totalBits + passes - 1) / passes;
  const size_t buckets = (size_t)1 << digit;
  const int nt = omp_get_max_threads();
  std::vector<size_t> hist((size_t)nt * buckets);
  for (int pass = 0; pass < passes; ++pass) {
    const int shift = pass * digit;
    std::fill(hist.begin(), hist.end(), 0);
    const Key* src = k;
    const uint32_t* srcv = v;
    Key* dst = k2;
    uint32_t* dstv = v2;
    // The data is cut into nt chunks and the loops run over chunk numbers, so the result does not depend on how
    // many threads the runtime really grants.
#pragma omp parallel
    {
#pragma omp for schedule(static, 1)
      for (int c = 0; c < nt; ++c) {
        const size_t lo = n * (size_t)c / nt, hi = n * (size_t)(c + 1) / nt;
        size_t* h = &hist[(size_t)c * buckets];
        for (size_t i = lo; i < hi; ++i) ++h[(size_t)(src[i] >> shift) & (buckets - 1)];
      }
#pragma omp single
      {
        size_t run = 0;
        for (size_t d = 0; d < buckets; ++d)
          for (int tt = 0; tt < nt; ++tt) {
            const size_t c = hist[(size_t)tt * buckets + d];
            hist[(size_t)tt * buckets + d] = run;
            run += c;
          }
      }
#pragma omp for schedule(static, 1)
      for (int c = 0; c < nt; ++c) {
        const size_t lo = n * (size_t)c / nt, hi = n * (size_t)(c + 1) / nt;
        size_t* h = &hist[(size_t)c * buckets];
        for (size_t i = lo; i < hi; ++i) {
          const size_t at = h[(size_t)(src[i] >> shift) & (buckets - 1)]++;
          dst[at] = src[i];
          dstv[at] = srcv[i];
        }
      }
    }
    std::swap(k, k2);
    std::swap(v, v2);
  }
}

template <typename Key>
int build_mode_t(int order, const uint64_t* dims, uint64_t nnz, const uint32_t* const* inds,
                 const float* vals, const hbcsf_opts& opts, int mode, ModeFormat* out,
                 std::string* err) {
  const auto t_begin = std::chrono::steady_clock::now();
  const int N = order;
  const uint32_t L = opts.fiber_threshold ? opts.fiber_threshold : 64;
  const uint32_t gmask = opts.group_mask == 0 ? 3u : (opts.group_mask & 3u);
  const int bb = mid_block_bits(order, dims, opts, mode);   // level-1 blocking: block number above the root in the key
  const bool cooOn = (gmask & 1u) && bb == 0, cslOn = gmask & 2u;

  // Tree levels: root = the target mode; the other modes ordered by the policy.
  int lv[HBCSF_MAX_ORDER];
  level_order(N, dims, mode, opts.mode_order_policy, lv);
  int bits[HBCSF_MAX_ORDER], shift[HBCSF_MAX_ORDER];
  uint64_t mask[HBCSF_MAX_ORDER];
  int total = 0;
  for (int l = N - 1; l >= 0; --l) {
    bits[l] = bits_for(dims[lv[l]]);
    shift[l] = total;
    mask[l] = (1ull << bits[l]) - 1;
    total += bits[l];
  }

  out->order = N;
  out->mode = mode;
  out->L = L;
  out->cooRowFlags = opts.coo_row_flags == 1;
  out->blockBits = bb;
  out->rows = dims[mode];
  for (int l = 0; l < N; ++l) out->levelMode[l] = lv[l];

  // ---- sort by packed (root, ..., leaf) key; the value rides along as payload ----
  const size_t M = (size_t)nnz;
  std::unique_ptr<Key[]> kbuf1(new (std::nothrow) Key[M + 1]), kbuf2(new (std::nothrow) Key[M + 1]);
  std::unique_ptr<uint32_t[]> vbuf1(new (std::nothrow) uint32_t[M + 1]), vbuf2(new (std::nothrow) uint32_t[M + 1]);
  if (!kbuf1 || !kbuf2 || !vbuf1 || !vbuf2) {
    *err = "out of host memory while sorting";
    return HBCSF_ENOMEM;
  }
  Key* K = kbuf1.get();
  Key* K2 = kbuf2.get();
  uint32_t* V = vbuf1.get();
  uint32_t* V2 = vbuf2.get();
  int bad = 0;
  int unsorted = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
  for (int64_t z = 0; z < (int64_t)M; ++z) {
    Key key = 0;
    for (int l = 0; l < N; ++l) {
      const uint32_t i = inds[lv[l]][z];
      if ((uint64_t)i >= dims[lv[l]]) bad |= 1;
      key |= (Key)i << shift[l];
    }
    if (bb) key |= (Key)(inds[lv[1]][z] >> (bits[1] - bb)) << total;
    K[z] = key;
    uint32_t vb;
    std::memcpy(&vb, &vals[z], 4);
    V[z] = vb;
  }
  if (bad) {
    *err = "an index is not below its dimension";
    return HBCSF_ERANGE;
  }
#pragma omp parallel for schedule(static) reduction(| : unsorted)
  for (int64_t z = 1; z < (int64_t)M; ++z)
    if (K[z] < K[z - 1]) unsorted |= 1;
  if (unsorted) radix_sort_pairs<Key>(K, V, K2, V2, M, total + bb);
  if (K == kbuf1.get()) { kbuf2.reset(); vbuf2.reset(); } else { kbuf1.reset(); vbuf1.reset(); }

  auto idx = [&](int l, size_t p) -> uint32_t { return (uint32_t)((uint64_t)(K[p] >> shift[l]) & mask[l]); };
  auto fresh = [&](int l, size_t p) -> bool { return p == 0 || (K[p] >> shift[l]) != (K[p - 1] >> shift[l]); };

  // ---- slices ----
  const int nt = omp_get_max_threads();
  std::vector<uint64_t> tcount(nt + 1, 0);
#pragma omp parallel for schedule(static, 1)
  for (int t = 0; t < nt; ++t) {  // chunk numbers, not thread numbers: any team size gives the same result
    const size_t lo = M * (size_t)t / nt, hi = M * (size_t)(t + 1) / nt;
    uint64_t c = 0;
    for (size_t p = lo; p < hi; ++p) c += fresh(0, p);
    tcount[t + 1] = c;
  }
  for (int t = 0; t < nt; ++t) tcount[t + 1] += tcount[t];
  const uint64_t S = tcount[nt];
  std::vector<uint32_t> sStart(S + 1);
#pragma omp parallel for schedule(static, 1)
  for (int t = 0; t < nt; ++t) {
    const size_t lo = M * (size_t)t / nt, hi = M * (size_t)(t + 1) / nt;
    uint64_t at = tcount[t];
    for (size_t p = lo; p < hi; ++p)
      if (fresh(0, p)) sStart[at++] = (uint32_t)p;
  }
  sStart[S] = (uint32_t)M;

  // ---- classify slices (Section V; Section VI-D) ----
  // Per slice (the paper's rule): one nonzero -> COO; every deepest-level fiber a singleton -> CSL; else CSF.
  // With hybrid_granularity = 1 the choice is made per fiber inside heavy slices: a slice of at least 2 L
  // nonzeros (it spans several runs, so its row is merged with atomic adds anyway) of which at least an eighth
  // sit in singleton deepest-level fibers is split: those nonzeros form a CSL-group slice of the same root index,
  // the others a CSF-group slice; both pieces are marked shared.
  const int NF = N - 2;  // fiber levels 1..NF
  const bool perFiber = opts.hybrid_granularity == 1 && cslOn;
  // a nonzero whose deepest-level fiber holds only itself
  auto single = [&](size_t p, size_t e) -> bool { return fresh(NF, p) && (p + 1 == e || fresh(NF, p + 1)); };
  constexpr uint8_t kSplit = 3;  // CSL piece + CSF piece
  std::vector<uint8_t> grp(S);
  std::vector<uint32_t> nSingle(perFiber ? S : 0);
  constexpr int kFL = HBCSF_MAX_FIBER_LEVELS;
  uint64_t fibNat[kFL] = {0, 0, 0};
  uint64_t fibNatCsf[kFL] = {0, 0, 0};
  {
    uint64_t f0 = 0, f1 = 0, f2 = 0, c0 = 0, c1 = 0, c2 = 0;
#pragma omp parallel for schedule(dynamic, 512) reduction(+ : f0, f1, f2, c0, c1, c2)
    for (int64_t s = 0; s < (int64_t)S; ++s) {
      const size_t b = sStart[s], e = sStart[s + 1];
      uint64_t nf[kFL] = {0, 0, 0};
      for (size_t p = b; p < e; ++p)
        for (int f = 0; f < NF; ++f) nf[f] += fresh(f + 1, p);
      const uint64_t n = e - b, deep = nf[NF - 1];
      uint8_t g;
      if (n == 1 && cooOn) g = kCoo;
      else if (deep == n && cslOn) g = kCsl;
      else g = kCsf;
      uint64_t kept[kFL] = {nf[0], nf[1], nf[2]};  // fibers that stay in the CSF group
      if (perFiber && g == kCsf && n >= 2ull * L) {
        uint64_t ns = 0;
        for (size_t p = b; p < e; ++p) ns += single(p, e);
        if (ns * 8 >= n) {
          g = kSplit;
          nSingle[s] = (uint32_t)ns;
          // fibers of the CSF piece: a fiber level counts once per run of kept nonzeros that share it
          kept[0] = kept[1] = kept[2] = 0;
          bool pend[kFL] = {false, false, false};
          for (size_t p = b; p < e; ++p) {
            for (int f = 0; f < NF; ++f) pend[f] = pend[f] || fresh(f + 1, p);
            if (single(p, e)) continue;
            for (int f = 0; f < NF; ++f) {
              kept[f] += pend[f];
              pend[f] = false;
            }
          }
        }
      }
      grp[s] = g;
      f0 += nf[0];
      f1 += nf[1];
      f2 += nf[2];
      if (g == kCsf || g == kSplit) { c0 += kept[0]; c1 += kept[1]; c2 += kept[2]; }
    }
    fibNat[0] = f0; fibNat[1] = f1; fibNat[2] = f2;
    fibNatCsf[0] = c0; fibNatCsf[1] = c1; fibNatCsf[2] = c2;
  }

  // ---- position of each slice (piece) inside its group ----
  // ord / off: the slice's entry and first nonzero in its group; a split slice's CSL piece is in ordL / offL
  std::vector<uint32_t> ord(S), off(S), ordL(perFiber ? S : 0), offL(perFiber ? S : 0);
  uint64_t gS[3] = {0, 0, 0}, gM[3] = {0, 0, 0};
  for (uint64_t s = 0; s < S; ++s) {
    const uint64_t n = sStart[s + 1] - sStart[s];
    if (grp[s] == kSplit) {
      ordL[s] = (uint32_t)gS[kCsl];
      offL[s] = (uint32_t)gM[kCsl];
      gS[kCsl] += 1;
      gM[kCsl] += nSingle[s];
      ord[s] = (uint32_t)gS[kCsf];
      off[s] = (uint32_t)gM[kCsf];
      gS[kCsf] += 1;
      gM[kCsf] += n - nSingle[s];
      continue;
    }
    const int g = grp[s];
    ord[s] = (uint32_t)gS[g];
    off[s] = (uint32_t)gM[g];
    gS[g] += 1;
    gM[g] += n;
  }

  // ---- count fiber segments of the CSF group (fbr-split on the run grid) ----
  // A segment starts at a kept nonzero that lies on the run grid or is the first kept one of its fiber.
  std::vector<uint32_t> segOff[kFL];
  uint64_t nSeg[kFL] = {0, 0, 0};
  for (int f = 0; f < NF; ++f) segOff[f].assign(S + 1, 0);
#pragma omp parallel for schedule(dynamic, 512)
  for (int64_t s = 0; s < (int64_t)S; ++s) {
    if (grp[s] != kCsf && grp[s] != kSplit) continue;
    const size_t b = sStart[s], e = sStart[s + 1];
    const bool split = grp[s] == kSplit;
    uint32_t c[kFL] = {0, 0, 0};
    uint32_t pos = off[s];
    bool pend[kFL] = {false, false, false};
    for (size_t p = b; p < e; ++p) {
      for (int f = 0; f < NF; ++f) pend[f] = pend[f] || fresh(f + 1, p);
      if (split && single(p, e)) continue;
      const bool cut = (pos % L) == 0;
      for (int f = 0; f < NF; ++f) {
        c[f] += cut || pend[f];
        pend[f] = false;
      }
      ++pos;
    }
    for (int f = 0; f < NF; ++f) segOff[f][s + 1] = c[f];
  }
  for (int f = 0; f < NF; ++f) {
    uint64_t run = 0;
    for (uint64_t s = 0; s < S; ++s) {
      const uint32_t c = segOff[f][s + 1];
      segOff[f][s] = (uint32_t)run;
      run += c;
    }
    segOff[f][S] = (uint32_t)run;
    nSeg[f] = run;
  }

  // ---- lay the arrays out in one blob ----
  layout_mode(out, N, gS, gM, nSeg);
  const uint64_t ownedWords = (out->rows + 31) / 32;
  void* mem = nullptr;
  if (posix_memalign(&mem, kAlign, (size_t)out->blobBytes) != 0 || !mem) {
    *err = "out of host memory for the format arrays";
    return HBCSF_ENOMEM;
  }
  out->blob = (uint8_t*)mem;
  auto U32 = [&](const ArrayRef& r) { return (uint32_t*)(out->blob + r.off); };
  uint32_t* owned = U32(out->ownedBits);
  std::memset(owned, 0, ownedWords * 4);
  uint32_t* cooBits = U32(out->cooBits);
  std::memset(cooBits, 0, ownedWords * 4);

  GroupFormat& Go = out->g[kCoo];
  GroupFormat& Gl = out->g[kCsl];
  GroupFormat& Gc = out->g[kCsf];
  uint32_t* cooInd[HBCSF_MAX_ORDER];
  uint32_t* cslInd[HBCSF_MAX_ORDER];
  uint32_t* csfInd[HBCSF_MAX_ORDER];
  uint32_t* csfPtr[HBCSF_MAX_ORDER];
  uint32_t* csfRun[HBCSF_MAX_ORDER];
  for (int l = 0; l < N; ++l) {
    cooInd[l] = U32(Go.ind[l]);
    cslInd[l] = U32(Gl.ind[l]);
    csfInd[l] = U32(Gc.ind[l]);
    csfPtr[l] = l < N - 1 ? U32(Gc.ptr[l]) : nullptr;
    csfRun[l] = l < N - 1 ? U32(Gc.runFirst[l]) : nullptr;
  }
  uint32_t* cooVal = U32(Go.val);
  uint32_t* cslVal = U32(Gl.val);
  uint32_t* csfVal = U32(Gc.val);
  uint32_t* cslPtr = U32(Gl.ptr[0]);
  uint32_t* cslRun = U32(Gl.runFirst[0]);

  uint64_t sharedSlices = 0;
#pragma omp parallel for schedule(dynamic, 512) reduction(+ : sharedSlices)
  for (int64_t s = 0; s < (int64_t)S; ++s) {
    const size_t b = sStart[s], e = sStart[s + 1];
    const uint32_t root = idx(0, b);
    const int g = grp[s];
    bool own = true;
    if (g == kCoo) {
      const uint32_t a = off[s];
      for (int l = out->cooRowFlags ? 1 : 0; l < N; ++l) cooInd[l][a] = idx(l, b);
      cooVal[a] = V[b];
      __atomic_fetch_or(&cooBits[root >> 5], 1u << (root & 31), __ATOMIC_RELAXED);
    } else {
      const bool split = g == kSplit;
      // the CSL piece (a whole CSL slice, or the singleton-fiber nonzeros of a split slice)
      if (g == kCsl || split) {
        const uint32_t a = split ? offL[s] : off[s], o = split ? ordL[s] : ord[s];
        const uint32_t n = split ? nSingle[s] : (uint32_t)(e - b);
        own = !split && bb == 0 && (a / L) == ((a + n - 1) / L);
        for (uint32_t r = (a + L - 1) / L; r <= (a + n - 1) / L; ++r) cslRun[r] = o;
        cslInd[0][o] = root | (own ? kOwnedBit : 0u);
        cslPtr[o] = a;
        uint32_t pos = a;
        for (size_t p = b; p < e; ++p) {
          if (split && !single(p, e)) continue;
          for (int l = 1; l < N; ++l) cslInd[l][pos] = idx(l, p);
          cslVal[pos] = V[p];
          ++pos;
        }
      }
      // the CSF piece
      if (g == kCsf || split) {
        const uint32_t a = off[s], o = ord[s];
        const uint32_t n = split ? (uint32_t)(e - b) - nSingle[s] : (uint32_t)(e - b);
        own = !split && bb == 0 && (a / L) == ((a + n - 1) / L);
        for (uint32_t r = (a + L - 1) / L; r <= (a + n - 1) / L; ++r) csfRun[0][r] = o;
        csfInd[0][o] = root | (own ? kOwnedBit : 0u);
        csfPtr[0][o] = a;
        uint32_t f[kFL] = {0, 0, 0};
        for (int q = 0; q < NF; ++q) f[q] = segOff[q][s];
        uint32_t pos = a;
        bool pend[kFL] = {false, false, false};
        for (size_t p = b; p < e; ++p) {
          for (int q = 0; q < NF; ++q) pend[q] = pend[q] || fresh(q + 1, p);
          if (split && single(p, e)) continue;
          const bool cut = (pos % L) == 0;
          for (int l = 1; l <= NF; ++l) {
            if (cut || pend[l - 1]) {
              csfInd[l][f[l - 1]] = idx(l, p);
              csfPtr[l][f[l - 1]] = pos;
              if (cut) csfRun[l][pos / L] = f[l - 1];
              ++f[l - 1];
            }
          }
          pend[0] = pend[1] = pend[2] = false;
          csfInd[N - 1][pos] = idx(N - 1, p);
          csfVal[pos] = V[p];
          ++pos;
        }
      }
      if (!own) ++sharedSlices;
    }
    if (own) __atomic_fetch_or(&owned[root >> 5], 1u << (root & 31), __ATOMIC_RELAXED);
  }
  {
    // COO-group nonzeros are stored in row order, so a running count over the bitmap locates them
    uint32_t* cooPtr = U32(out->cooPtr);
    uint32_t run = 0;
    for (uint64_t w = 0; w < ownedWords; ++w) {
      cooPtr[w] = run;
      run += (uint32_t)__builtin_popcount(cooBits[w]);
    }
    cooPtr[ownedWords] = run;
  }
  // sentinels and pads
  cslInd[0][Gl.n[0]] = 0;
  cslPtr[Gl.n[0]] = (uint32_t)Gl.nnz;
  cslRun[Gl.runs] = (uint32_t)Gl.n[0];
  for (int l = 0; l < N - 1; ++l) {
    csfInd[l][Gc.n[l]] = 0;
    csfPtr[l][Gc.n[l]] = (uint32_t)Gc.nnz;
    csfRun[l][Gc.runs] = (uint32_t)Gc.n[l];
  }

  // ---- statistics ----
  fill_count_stats(out, N, M, S, fibNat, fibNatCsf, nSeg, gS, gM, sharedSlices);
  hbcsf_stats& st = out->stats;
  {
    uint64_t cnt = 0;
#pragma omp parallel for schedule(static) reduction(+ : cnt)
    for (int64_t w = 0; w < (int64_t)ownedWords; ++w) cnt += (uint64_t)__builtin_popcount(owned[w]);
    st.owned_rows = cnt;
  }
  {
    // distinct factor rows each group gathers, per tree level
    std::vector<uint8_t> seen;
    for (int g = 0; g < 3; ++g) {
      const GroupFormat& G = out->g[g];
      for (int l = 1; l < N; ++l) {
        const uint32_t* a = U32(G.ind[l]);
        const uint64_t cnt = (g == kCsf && l < N - 1) ? G.n[l] : G.nnz;
        uint64_t d = 0;
        if (cnt == 0) {
          d = 0;
        } else if (cnt * 16 < dims[lv[l]]) {  // few indices in a long mode: sort and count
          std::vector<uint32_t> tmp(a, a + cnt);
          std::sort(tmp.begin(), tmp.end());
          d = (uint64_t)(std::unique(tmp.begin(), tmp.end()) - tmp.begin());
        } else {
          seen.assign(dims[lv[l]], 0);
          uint8_t* sp = seen.data();
#pragma omp parallel for schedule(static)
          for (int64_t t = 0; t < (int64_t)cnt; ++t) __atomic_store_n(&sp[a[t]], (uint8_t)1, __ATOMIC_RELAXED);
#pragma omp parallel for schedule(static) reduction(+ : d)
          for (int64_t t = 0; t < (int64_t)seen.size(); ++t) d += sp[t];
        }
        st.distinct_rows[g][l] = d;
      }
    }
  }
  st.build_seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t_begin).count();
  return HBCSF_OK;
}

}  // namespace

int build_mode(int order, const uint64_t* dims, uint64_t nnz, const uint32_t* const* inds,
               const float* vals, const hbcsf_opts& opts, int mode, ModeFormat* out,
               std::string* err) {
  int total = mid_block_bits(order, dims, opts, mode);
  for (int m = 0; m < order; ++m) total += bits_for(dims[m]);
  try {
    if (total <= 64)
      return build_mode_t<uint64_t>(order, dims, nnz, inds, vals, opts, mode, out, err);
    return build_mode_t<unsigned __int128>(order, dims, nnz, inds, vals, opts, mode, out, err);
  } catch (const std::bad_alloc&) {
    *err = "out of host memory while building the format";
    return HBCSF_ENOMEM;
  } catch (...) {
    *err = "unexpected failure while building the format";
    return HBCSF_EINVAL;
  }
}

}  // namespace hbcsf
