// Workgroup-level radix select for the Top-K sparsifier S_k (Sec. 4.3, Eq. 8), shared by the
// stand-alone Top-K kernel and the Top-K prologue of the fused projection kernel.
//
// The ordering key is the stored 16-bit pattern with the sign cleared (15 bits, unsigned), so
// the selection is pure integer work and identical for binary16 and bfloat16.  Lane t owns the
// contiguous elements [t*E, (t+1)*E) and keeps them in registers through all phases:
//   1. 256-bin histogram of the top 8 key bits.  Activations crowd into a few of these bins (for
//      bfloat16 the 8 bits are the exponent alone), and lanes of one wave that add to the same LDS
//      word are served one per clock; so there are kTopkCopies histograms (in different banks for one
//      bin) and a lane adds to copy (lane mod kTopkCopies): at most 64 / kTopkCopies lanes meet in a
//      word whatever the data.
//      Suffix sums from the top locate the bin holding the K-th largest key;
//   2. 128-bin histogram (same copies) of the low 7 bits inside that bin gives the threshold key T and
//      r = K - #{key > T}, the number of threshold ties to keep;
//   3. block prefix sums of the ">T" and "==T" counts give every lane the number of kept
//      elements before its own, so an index-ordered compaction keeps every key > T and the first
//      r keys == T: ascending indices and the lower-index tie rule with no sort.
#pragma once
#include <cstddef>

#include "numeric.hpp"

namespace larosa {

constexpr int kTopkCopies = 8;
constexpr int kTopkCopyStride = 260;   // words between copies: 16-byte aligned, and the copies of one bin fall in different LDS banks
constexpr int kTopkCopyStride2 = 132;  // the same for the 128-bin pass

template <int NW>
struct TopkShared {
  alignas(16) unsigned hist[kTopkCopyStride * kTopkCopies];   // pass 1: word copy * kTopkCopyStride + bin
  unsigned hist2[kTopkCopyStride2 * kTopkCopies];            // pass 2 (adjacent, so both are cleared in one step)
  unsigned wave_tot[NW];
  int bin, bin2;            // pass-1 / pass-2 bin holding the K-th largest key
  unsigned above, above2;   // counts strictly above those bins
};

// Selection state of one lane after block_select.
struct TopkLane {
  unsigned T;          // threshold key
  unsigned r;          // number of keys == T to keep (>= 1)
  unsigned gt_before;  // kept-by-magnitude elements before this lane's first element
  unsigned eq_before;  // threshold ties before this lane's first element
  unsigned n_gt, n_eq; // this lane's own counts of keys > T and == T
  unsigned long long m_gt, m_eq;   // bit q set: this lane's element q has key > T / == T
  // ranks [first, end) of the ascending kept list held by this lane
  __device__ __forceinline__ unsigned first_rank() const { return gt_before + min(eq_before, r); }
  __device__ __forceinline__ unsigned end_rank() const { return gt_before + n_gt + min(eq_before + n_eq, r); }
};

// Zero both histograms; every lane of the workgroup calls it.  No barrier: the caller's next barrier
// (it usually has one of its own while it builds the vector) makes the zeros visible.
template <int NW>
__device__ __forceinline__ void topk_clear(TopkShared<NW>& sm) {
  constexpr int kWords = (kTopkCopyStride + kTopkCopyStride2) * kTopkCopies;   // hist and hist2 are adjacent
  static_assert(offsetof(TopkShared<NW>, hist2) == sizeof(unsigned) * kTopkCopyStride * kTopkCopies,
                "histograms must be adjacent");
  static_assert(offsetof(TopkShared<NW>, hist) % 16 == 0 && kWords % 4 == 0, "cleared and read in 16-byte pieces");
  uint4* flat = reinterpret_cast<uint4*>(sm.hist);
  for (int i = threadIdx.x; i < kWords / 4; i += NW * 64) flat[i] = make_uint4(0u, 0u, 0u, 0u);
}

// raw[q] (q < nvalid) are this lane's stored 16-bit values; raw[q] for q >= nvalid (positions past
// the end of the vector) MUST be zero.  Such padding is counted like a zero at an index above every
// real element: it is never above the threshold, and among threshold ties the lower-index rule takes
// the real elements first (K is at most their number), so it is never kept -- and the three passes
// over the elements need no per-element predicate.  Every lane of the NW-wave workgroup must call
// this, after topk_clear and a workgroup barrier.  1 <= K <= total number of valid elements <= 32768.
template <int NW, int E>
__device__ __forceinline__ TopkLane block_select(const uint16_t (&raw)[E], int nvalid, int K, TopkShared<NW>& sm) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;

  // ---- pass 1: top 8 key bits
  unsigned* mine = sm.hist + (static_cast<unsigned>(lane) & (kTopkCopies - 1)) * kTopkCopyStride;
#pragma unroll
  for (int q = 0; q < E; ++q)
    atomicAdd(&mine[(raw[q] & 0x7FFFu) >> 7], 1u);
  __syncthreads();
  if (wave == 0) {
    // lane covers 4 bins counted from the top: position p = 4*lane + q is bin 255 - p; its four
    // counts of one copy are one aligned 16-byte read
    unsigned c[4] = {0u, 0u, 0u, 0u}, local = 0;
#pragma unroll
    for (int k = 0; k < kTopkCopies; ++k) {
      const uint4 v = *reinterpret_cast<const uint4*>(sm.hist + k * kTopkCopyStride + 252 - 4 * lane);
      c[0] += v.w; c[1] += v.z; c[2] += v.y; c[3] += v.x;
    }
    local = (c[0] + c[1]) + (c[2] + c[3]);
    const unsigned need = static_cast<unsigned>(K);
    unsigned run = wave_scan_inclusive(local, lane) - local;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const unsigned before = run;
      run += c[q];
      if (before < need && run >= need) {
        sm.bin = 255 - (lane * 4 + q);
        sm.above = before;
      }
    }
  }
  __syncthreads();
  const int bin1 = sm.bin;
  const unsigned above1 = sm.above;

  // ---- pass 2: low 7 bits inside bin1
  unsigned* mine2 = sm.hist2 + (static_cast<unsigned>(lane) & (kTopkCopies - 1)) * kTopkCopyStride2;
#pragma unroll
  for (int q = 0; q < E; ++q) {
    const unsigned key = raw[q] & 0x7FFFu;
    if (static_cast<int>(key >> 7) == bin1) atomicAdd(&mine2[key & 127u], 1u);
  }
  __syncthreads();
  if (wave == 0) {
    unsigned c[2] = {0u, 0u};
#pragma unroll
    for (int k = 0; k < kTopkCopies; ++k) {   // bins 127 - 2*lane (c[0]) and 126 - 2*lane (c[1]): one 8-byte read per copy
      const uint2 v = *reinterpret_cast<const uint2*>(sm.hist2 + k * kTopkCopyStride2 + 126 - 2 * lane);
      c[0] += v.y; c[1] += v.x;
    }
    const unsigned local = c[0] + c[1];
    const unsigned need = static_cast<unsigned>(K) - above1;
    unsigned run = wave_scan_inclusive(local, lane) - local;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const unsigned before = run;
      run += c[q];
      if (before < need && run >= need) {
        sm.bin2 = 127 - (lane * 2 + q);
        sm.above2 = before;
      }
    }
  }
  __syncthreads();
  TopkLane out;
  out.T = (static_cast<unsigned>(bin1) << 7) | static_cast<unsigned>(sm.bin2);
  out.r = static_cast<unsigned>(K) - (above1 + sm.above2);

  // per-lane bit masks of the two classes (independent compares: no chain from element to element)
  unsigned long long m_gt = 0, m_eq = 0;
#pragma unroll
  for (int q = 0; q < E; ++q) {
    const unsigned key = raw[q] & 0x7FFFu;
    m_gt |= static_cast<unsigned long long>(key > out.T ? 1u : 0u) << q;
    m_eq |= static_cast<unsigned long long>(key == out.T ? 1u : 0u) << q;
  }
  (void)nvalid;
  const unsigned n_gt = static_cast<unsigned>(__popcll(m_gt)), n_eq = static_cast<unsigned>(__popcll(m_eq));
  out.m_gt = m_gt;
  out.m_eq = m_eq;
  const unsigned packed = n_gt | (n_eq << 16);          // each total <= 32768: no carry between halves
  const unsigned incl = wave_scan_inclusive(packed, lane);
  if (lane == 63) sm.wave_tot[wave] = incl;
  __syncthreads();
  unsigned prefix = incl - packed;
#pragma unroll
  for (int w = 0; w < NW; ++w) {          // all totals are read at once; a loop to `wave` would chain the reads
    const unsigned t = sm.wave_tot[w];
    prefix += (w < wave) ? t : 0u;
  }
  out.gt_before = prefix & 0xFFFFu;
  out.eq_before = prefix >> 16;
  out.n_gt = n_gt;
  out.n_eq = n_eq;
  return out;
}

// Visit this lane's elements in index order; emit(q, pos, kept) is called for EVERY element q < E, with
// kept telling whether it is selected and, if so, pos its rank in the ascending kept list (callers
// fold `kept` into their store predicate: a branch per element costs more than the stores).  Kept = key > T, plus the first r threshold ties in index
// order; a kept element's rank is the lane's first rank plus the number of kept elements before it
// in the lane, so every element is handled independently of the others.
template <int E, typename F>
__device__ __forceinline__ void for_each_kept(const uint16_t (&raw)[E], int nvalid, const TopkLane& st, F emit) {
  (void)raw; (void)nvalid;
  // threshold ties of this lane that are kept: its first (r - eq_before) ones
  unsigned long long eq_keep = st.m_eq;
  const int want = static_cast<int>(st.r) - static_cast<int>(st.eq_before);
  if (want < static_cast<int>(st.n_eq)) {            // rare: the tie quota ends inside this lane
    unsigned long long m = st.m_eq;
    eq_keep = 0;
    for (int i = 0; i < want; ++i) {
      const unsigned long long low = m & (0ull - m);
      eq_keep |= low;
      m ^= low;
    }
  }
  const unsigned long long kept = st.m_gt | eq_keep;
  const unsigned first = st.first_rank();
#pragma unroll
  for (int q = 0; q < E; ++q)
    emit(q, first + static_cast<unsigned>(__popcll(kept & ((1ull << q) - 1ull))), ((kept >> q) & 1ull) != 0ull);
}

}  // namespace larosa
