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
//      word whatever the data.  After ONE barrier every wave sums the copies and walks the bins from
//      the top by itself (suffix sums on the data-parallel path), so the bin holding the K-th largest
//      key needs no broadcast through LDS and no second barrier;
//   2. 128-bin histogram of the low 7 bits inside that bin, one copy PER WAVE.  After one more barrier
//      every wave reads all copies: their sum gives the threshold key T and r = K - #{key > T}, the
//      number of threshold ties to keep, and the copies of the waves before it give the number of
//      kept elements of that bin in front of the wave -- the block prefix needs no barrier of its own.
//      (The counts of elements in higher bins travel as one total per wave with the same barrier.)
//   3. a wave-level prefix sum of the ">T" and "==T" counts then gives every lane the number of kept
//      elements before its own, so an index-ordered compaction keeps every key > T and the first
//      r keys == T: ascending indices and the lower-index tie rule with no sort.
// Two barriers in all (after the one that makes the cleared histograms and the vector visible).
#pragma once
#include <cstddef>

#include "kernels.hpp"
#include "numeric.hpp"

namespace larosa {

constexpr int kTopkCopies = 8;
// Pass 1's 256 bins times kTopkCopies are 8 KiB to read: one wave walks them and hands the bin on through
// LDS (one more barrier); every wave doing it by itself measured slower with two workgroups per compute unit.
#ifndef LAROSA_TOPK_ALL_WAVES_SCAN1
#define LAROSA_TOPK_ALL_WAVES_SCAN1 0
#endif
constexpr bool kTopkAllWavesScan1 = LAROSA_TOPK_ALL_WAVES_SCAN1 != 0;
constexpr int kTopkCopyStride = 260;   // words between copies: 16-byte aligned, and the copies of one bin fall in different LDS banks
constexpr int kTopkCopyStride2 = 132;  // the same for the 128-bin pass (one copy per wave)

// A workgroup that selects for a wide vector, or for bfloat16 (whose top 8 key bits are the exponent alone,
// so nearly every lane of a wave adds to the same few bins), is bound by those same-word additions: with
// kTopkCopiesWide copies (lane mod 32 picks the copy; stride 1 mod 32, so the 32 copies of one bin lie
// in 32 different banks) at most two lanes of a wave ever meet in a word.  The copies are then summed by
// the whole workgroup (one more barrier) before wave 0 walks the bins.
constexpr int kTopkCopiesWide = 32;
constexpr int kTopkCopyStrideWide = 257;
// words of the pass-1 histograms, padded to a multiple of 4 (they are cleared in 16-byte pieces)
template <int C> struct TopkHist1 { static constexpr int words = kTopkCopyStride * C; static constexpr int stride = kTopkCopyStride; };
template <> struct TopkHist1<kTopkCopiesWide> {
  static constexpr int words = (kTopkCopyStrideWide * kTopkCopiesWide + 3) / 4 * 4;
  static constexpr int stride = kTopkCopyStrideWide;
};

template <int NW, int C = kTopkCopies>
struct TopkShared {
  alignas(16) unsigned hist[TopkHist1<C>::words];             // pass 1: word copy * stride + bin
  unsigned hist2[kTopkCopyStride2 * NW];                      // pass 2: word wave * kTopkCopyStride2 + bin (adjacent: cleared in one step)
  alignas(16) unsigned part[C == kTopkCopiesWide ? 256 * (NW / 4) : 4];   // wide copies: sums over NW/4 groups of copies
  unsigned wave_tot[NW];                                      // per wave: elements in bins above the threshold bin
  int bin;                                                    // pass-1 bin holding the K-th largest key, and the
  unsigned above;                                             // count strictly above it (written by wave 0)
};

// one bit per element of a lane
template <int E> struct LaneMask { typedef unsigned long long type; };
template <> struct LaneMask<4> { typedef unsigned type; };
template <> struct LaneMask<8> { typedef unsigned type; };
template <> struct LaneMask<12> { typedef unsigned type; };
template <> struct LaneMask<16> { typedef unsigned type; };
template <> struct LaneMask<24> { typedef unsigned type; };
template <> struct LaneMask<32> { typedef unsigned type; };

__device__ __forceinline__ unsigned popc_mask(unsigned m) { return static_cast<unsigned>(__popc(m)); }
__device__ __forceinline__ unsigned popc_mask(unsigned long long m) { return static_cast<unsigned>(__popcll(m)); }

// Selection state of one lane after block_select.
template <typename Mask>
struct TopkLaneT {
  unsigned T;          // threshold key
  unsigned r;          // number of keys == T to keep (>= 1)
  unsigned gt_before;  // kept-by-magnitude elements before this lane's first element
  unsigned eq_before;  // threshold ties before this lane's first element
  unsigned n_gt, n_eq; // this lane's own counts of keys > T and == T
  Mask m_gt, m_eq;     // bit q set: this lane's element q has key > T / == T
  // ranks [first, end) of the ascending kept list held by this lane
  __device__ __forceinline__ unsigned first_rank() const { return gt_before + min(eq_before, r); }
  __device__ __forceinline__ unsigned end_rank() const { return gt_before + n_gt + min(eq_before + n_eq, r); }
};

// Zero both histograms; every lane of the workgroup calls it.  No barrier: the caller's next barrier
// (it usually has one of its own while it builds the vector) makes the zeros visible.
template <int NW, int C>
__device__ __forceinline__ void topk_clear(TopkShared<NW, C>& sm) {
  constexpr int kWords = TopkHist1<C>::words + kTopkCopyStride2 * NW;   // hist and hist2 are adjacent
  typedef TopkShared<NW, C> Sh;
  static_assert(offsetof(Sh, hist2) == sizeof(unsigned) * TopkHist1<C>::words, "histograms must be adjacent");
  static_assert(offsetof(Sh, hist) % 16 == 0 && kWords % 4 == 0, "cleared and read in 16-byte pieces");
  uint4* flat = reinterpret_cast<uint4*>(sm.hist);
  for (int i = threadIdx.x; i < kWords / 4; i += NW * 64) flat[i] = make_uint4(0u, 0u, 0u, 0u);
}

// Sum over the 64 lanes, the same value in every lane (and known to be uniform).
__device__ __forceinline__ unsigned wave_total(unsigned v, int lane) {
  return static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(wave_scan_inclusive(v, lane)), 63));
}

// raw[q] are this lane's stored 16-bit values; positions past the end of the vector MUST hold zero.
// Such padding is counted like a zero at an index above every real element: it is never above the
// threshold, and among threshold ties the lower-index rule takes the real elements first (K is at most
// their number), so it is never kept -- and the passes over the elements need no per-element predicate.
// Every lane of the NW-wave workgroup must call this, after topk_clear and a workgroup barrier.
// 1 <= K <= total number of valid elements <= 32768.
template <int NW, int E, int C>
__device__ __forceinline__ TopkLaneT<typename LaneMask<E>::type> block_select(const uint16_t (&raw)[E], int K,
                                                                              TopkShared<NW, C>& sm) {
  typedef typename LaneMask<E>::type Mask;
  constexpr bool kWide = C == kTopkCopiesWide;
  static_assert(!kWide || (NW % 4 == 0 && 32 % (NW / 4) == 0), "the copies are summed by NW/4 groups of 256 lanes");
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // ---- pass 1: top 8 key bits
  unsigned* mine = sm.hist + (static_cast<unsigned>(lane) & (C - 1)) * TopkHist1<C>::stride;
#pragma unroll
  for (int q = 0; q < E; ++q)
    atomicAdd(&mine[(raw[q] & 0x7FFFu) >> 7], 1u);
  __syncthreads();
  if constexpr (kWide) {
    // lane group g = tid / 256 sums its 32 / (NW/4) copies of bin tid % 256 (consecutive lanes, consecutive banks)
    constexpr int kGroups = NW / 4, kPer = kTopkCopiesWide / kGroups;
    const int bin = tid & 255, grp = tid >> 8;
    unsigned sum = 0;
#pragma unroll
    for (int k = 0; k < kPer; ++k) sum += sm.hist[(grp * kPer + k) * kTopkCopyStrideWide + bin];
    sm.part[grp * 256 + bin] = sum;
    __syncthreads();
  }
  int bin1;
  unsigned above1;
  if (kTopkAllWavesScan1 || wave == 0) {
    // lane covers 4 bins counted from the top: position p = 4*lane + q is bin 255 - p; its four
    // counts of one copy are one aligned 16-byte read
    unsigned c[4] = {0u, 0u, 0u, 0u};
    if constexpr (kWide) {
#pragma unroll
      for (int k = 0; k < NW / 4; ++k) {
        const uint4 v = *reinterpret_cast<const uint4*>(sm.part + k * 256 + 252 - 4 * lane);
        c[0] += v.w; c[1] += v.z; c[2] += v.y; c[3] += v.x;
      }
    } else {
#pragma unroll
      for (int k = 0; k < kTopkCopies; ++k) {
        const uint4 v = *reinterpret_cast<const uint4*>(sm.hist + k * kTopkCopyStride + 252 - 4 * lane);
        c[0] += v.w; c[1] += v.z; c[2] += v.y; c[3] += v.x;
      }
    }
    const unsigned local = (c[0] + c[1]) + (c[2] + c[3]);
    const unsigned need = static_cast<unsigned>(K);
    unsigned run = wave_scan_inclusive(local, lane) - local;
    int cand = -1;
    unsigned cand_above = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const unsigned before = run;
      run += c[q];
      if (before < need && run >= need) {
        cand = 255 - (lane * 4 + q);
        cand_above = before;
      }
    }
    // exactly one lane holds the bin (1 <= K <= number of counted elements)
    if (kTopkAllWavesScan1) {
      const unsigned long long found = __builtin_amdgcn_ballot_w64(cand >= 0);
      const int src = found ? __builtin_ctzll(found) : 0;
      bin1 = __builtin_amdgcn_readlane(cand, src);
      above1 = static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(cand_above), src));
    } else if (cand >= 0) {
      sm.bin = cand;
      sm.above = cand_above;
    }
  }
  if (!kTopkAllWavesScan1) {
    __syncthreads();
    bin1 = sm.bin;
    above1 = sm.above;
  }

  // ---- pass 2: low 7 bits inside bin1 (this wave's copy), and the wave's count of elements in higher bins
  unsigned* mine2 = sm.hist2 + wave * kTopkCopyStride2;
  Mask m_hi = 0;
#pragma unroll
  for (int q = 0; q < E; ++q) {
    const unsigned key = raw[q] & 0x7FFFu;
    const int cb = static_cast<int>(key >> 7);
    if (cb == bin1) atomicAdd(&mine2[key & 127u], 1u);
    m_hi |= static_cast<Mask>(cb > bin1 ? 1u : 0u) << q;
  }
  {
    const unsigned tot_hi = wave_total(popc_mask(m_hi), lane);
    if (lane == 0) sm.wave_tot[wave] = tot_hi;
  }
  __syncthreads();
  TopkLaneT<Mask> out;
  unsigned base_gt, base_eq;   // kept-by-magnitude elements / threshold ties in the waves before this one
  {
    // lane covers bins 127 - 2*lane (c[0]) and 126 - 2*lane (c[1]): one 8-byte read per wave copy;
    // p[] = the same two bins summed over the waves before this one
    unsigned c[2] = {0u, 0u}, p[2] = {0u, 0u};
#pragma unroll
    for (int k = 0; k < NW; ++k) {
      const uint2 v = *reinterpret_cast<const uint2*>(sm.hist2 + k * kTopkCopyStride2 + 126 - 2 * lane);
      c[0] += v.y; c[1] += v.x;
      if (k < wave) { p[0] += v.y; p[1] += v.x; }   // uniform condition
    }
    const unsigned local = c[0] + c[1];
    const unsigned need = static_cast<unsigned>(K) - above1;
    unsigned run = wave_scan_inclusive(local, lane) - local;
    int cand = -1;
    unsigned cand_above = 0;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const unsigned before = run;
      run += c[q];
      if (before < need && run >= need) {
        cand = 127 - (lane * 2 + q);
        cand_above = before;
      }
    }
    const unsigned long long found = __builtin_amdgcn_ballot_w64(cand >= 0);
    const int src = found ? __builtin_ctzll(found) : 0;
    const int bin2 = __builtin_amdgcn_readlane(cand, src);
    const unsigned above2 = static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(cand_above), src));
    out.T = (static_cast<unsigned>(bin1) << 7) | static_cast<unsigned>(bin2);
    out.r = static_cast<unsigned>(K) - (above1 + above2);
    // elements of the threshold bin above / at T in earlier waves, plus earlier waves' higher-bin totals
    // (lane k < wave adds wave_tot[k]); packed as gt | eq << 16, each at most 32768
    const int b0 = 127 - 2 * lane, b1 = 126 - 2 * lane;
    unsigned gt = (b0 > bin2 ? p[0] : 0u) + (b1 > bin2 ? p[1] : 0u);
    const unsigned eq = (b0 == bin2 ? p[0] : 0u) + (b1 == bin2 ? p[1] : 0u);
    if (lane < wave) gt += sm.wave_tot[lane];      // wave <= NW <= 16 < 64
    // the two sums are reduced separately: their packed total could carry (32768 + 32768 in one half)
    base_gt = wave_total(gt, lane);
    base_eq = wave_total(eq, lane);
  }

  // per-lane bit masks of the two classes (independent compares: no chain from element to element)
  Mask m_gt = 0, m_eq = 0;
#pragma unroll
  for (int q = 0; q < E; ++q) {
    const unsigned key = raw[q] & 0x7FFFu;
    m_gt |= static_cast<Mask>(key > out.T ? 1u : 0u) << q;
    m_eq |= static_cast<Mask>(key == out.T ? 1u : 0u) << q;
  }
  const unsigned n_gt = popc_mask(m_gt), n_eq = popc_mask(m_eq);
  out.m_gt = m_gt;
  out.m_eq = m_eq;
  // within the wave: one wave holds at most 64 * E <= 4096 elements, so both counts fit 16-bit halves
  const unsigned packed = n_gt | (n_eq << 16);
  const unsigned excl = wave_scan_inclusive(packed, lane) - packed;
  out.gt_before = base_gt + (excl & 0xFFFFu);
  out.eq_before = base_eq + (excl >> 16);
  out.n_gt = n_gt;
  out.n_eq = n_eq;
  return out;
}

// ---- selection from histograms that the producer of the vector has already built ------------------
//
// A vector that one of the library's own kernels writes (the MLP intermediate vector, a rotated block
// input) can arrive with the two histograms of its keys in device memory: hist[0 .. 256) counts the top
// 8 key bits, hist[256 + key] every 15-bit key (the workgroups that store the vector's strips add their
// elements with device atomics).  The threshold then costs two small dependent reads by one wave instead
// of two histogram passes over the vector in every workgroup.

// Threshold key T and tie quota r = K - #{key > T} from such histograms, in two steps so that the caller
// can issue the loads where it wants them (the second read depends on the first step's result); all 64
// lanes of one wave take part, results in every lane.  1 <= K <= number of counted elements.
// Lane's words: coarse bins 255 - 4 lane - q (q = 0..3) are hist[252 - 4 lane + (3 - q)], one 16-byte read.
__device__ __forceinline__ const uint4* hist_coarse_ptr(const unsigned* hist, int lane) {
  return reinterpret_cast<const uint4*>(hist + 252 - 4 * lane);
}
// fine bins 127 - 2 lane, 126 - 2 lane of coarse bin `bin1`: one 8-byte read
__device__ __forceinline__ const uint2* hist_fine_ptr(const unsigned* hist, int bin1, int lane) {
  return reinterpret_cast<const uint2*>(hist + kHistCoarse + bin1 * 128 + 126 - 2 * lane);
}
// step 1: the coarse bin that holds the K-th largest key, and the count above it
__device__ __forceinline__ void hist_coarse_step(const uint4& v, int K, int lane, int& bin1, unsigned& above1) {
  const unsigned c[4] = {v.w, v.z, v.y, v.x};
  const unsigned local = (c[0] + c[1]) + (c[2] + c[3]);
  const unsigned need = static_cast<unsigned>(K);
  unsigned run = wave_scan_inclusive(local, lane) - local;
  int cand = -1;
  unsigned cand_above = 0;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const unsigned before = run;
    run += c[q];
    if (before < need && run >= need) {
      cand = 255 - (lane * 4 + q);
      cand_above = before;
    }
  }
  const unsigned long long found = __builtin_amdgcn_ballot_w64(cand >= 0);
  const int src = found ? __builtin_ctzll(found) : 0;
  bin1 = max(0, __builtin_amdgcn_readlane(cand, src));
  above1 = static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(cand_above), src));
}
// step 2: the threshold key and the tie quota
__device__ __forceinline__ void hist_fine_step(const uint2& f, int K, int bin1, unsigned above1, int lane, unsigned& T,
                                               unsigned& r) {
  const unsigned c2[2] = {f.y, f.x};
  const unsigned need = static_cast<unsigned>(K) - above1;
  unsigned run = wave_scan_inclusive(c2[0] + c2[1], lane) - (c2[0] + c2[1]);
  int cand = -1;
  unsigned cand_above = 0;
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const unsigned before = run;
    run += c2[q];
    if (before < need && run >= need) {
      cand = 127 - (lane * 2 + q);
      cand_above = before;
    }
  }
  const unsigned long long found = __builtin_amdgcn_ballot_w64(cand >= 0);
  const int src = found ? __builtin_ctzll(found) : 0;
  const int bin2 = max(0, __builtin_amdgcn_readlane(cand, src));
  const unsigned above2 = static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(cand_above), src));
  T = (static_cast<unsigned>(bin1) << 7) | static_cast<unsigned>(bin2);
  r = static_cast<unsigned>(K) - (above1 + above2);
}

// Producer side: the eight stored 16-bit values of each lane of ONE wave (valid lanes only) are added to
// the histograms, each counting `weight` times.  The coarse counts are summed in `scratch` (256 words of
// LDS owned by this wave) first, so a bin that many strips fill costs one device atomic per strip and
// not one per element.  All 64 lanes must call it.
__device__ __forceinline__ void histograms_add_wave(const uint16_t (&bits)[8], bool valid, unsigned weight,
                                                    unsigned* __restrict__ hist, unsigned* scratch, int lane) {
  // Lanes of the wave exchange counts through `scratch`: every access to it is an atomic, and the three
  // steps are separated by wavefront-scope fences (no instructions on this hardware, where a wave's LDS
  // operations complete in order; they keep the compiler from forwarding a lane's own zeros to its read).
#pragma unroll
  for (int k = 0; k < 4; ++k)
    __hip_atomic_store(scratch + 4 * lane + k, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  if (valid) {
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const unsigned key = bits[k] & 0x7FFFu;
      __hip_atomic_fetch_add(scratch + (key >> 7), weight, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
      atomicAdd(&hist[kHistCoarse + key], weight);
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const unsigned c = __hip_atomic_load(scratch + 4 * lane + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
    if (c) atomicAdd(&hist[4 * lane + k], c);
  }
}

// Visit this lane's elements in index order; emit(q, pos, kept) is called for EVERY element q < E, with
// kept telling whether it is selected and, if so, pos its rank in the ascending kept list (callers
// fold `kept` into their store predicate: a branch per element costs more than the stores).  Kept = key > T, plus the first r threshold ties in index
// order; a kept element's rank is the lane's first rank plus the number of kept elements before it
// in the lane, so every element is handled independently of the others.
template <int E, typename Mask, typename F>
__device__ __forceinline__ void for_each_kept(const TopkLaneT<Mask>& st, F emit) {
  // threshold ties of this lane that are kept: its first (r - eq_before) ones
  Mask eq_keep = st.m_eq;
  const int want = static_cast<int>(st.r) - static_cast<int>(st.eq_before);
  if (want < static_cast<int>(st.n_eq)) {            // rare: the tie quota ends inside this lane
    Mask m = st.m_eq;
    eq_keep = 0;
    for (int i = 0; i < want; ++i) {
      const Mask low = m & (static_cast<Mask>(0) - m);
      eq_keep |= low;
      m ^= low;
    }
  }
  const Mask kept = st.m_gt | eq_keep;
  const unsigned first = st.first_rank();
#pragma unroll
  for (int q = 0; q < E; ++q)
    emit(q, first + popc_mask(static_cast<Mask>(kept & ((static_cast<Mask>(1) << q) - static_cast<Mask>(1)))),
         ((kept >> q) & static_cast<Mask>(1)) != 0);
}

}  // namespace larosa
