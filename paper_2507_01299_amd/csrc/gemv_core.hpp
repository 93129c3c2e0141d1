// Device-side building blocks of the row-streaming mat-vec (shared by the stand-alone kernel and
// the kernel with the Top-K prologue): the row loop, the LDS reduction across the row-waves of a
// workgroup, the cross-workgroup hand-off of partial strips and the epilogue.
//
// Geometry: a wave owns one strip of 512 output columns (64 lanes x 16 bytes, so one kept row
// is a 1 KiB coalesced burst) and a run of kept rows; each lane keeps 8 fp32 accumulators.
// A workgroup is RW such waves on the same strip.
#pragma once
#include "kernels.hpp"
#include "numeric.hpp"

namespace larosa {

constexpr int kStripCols = 512;
constexpr int kUnroll = 8;

// 16-byte load of weight data that is read once: the non-temporal hint keeps the stream from
// displacing the small reused vectors (h, indices, partial strips) in the caches.
__device__ __forceinline__ uint4 load_stream16(const uint16_t* p) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// Row source read from global memory: indexed (idx != nullptr) or the identity list.
template <typename T, bool INDEXED>
struct GlobalRows {
  const int32_t* idx;        // this token's kept indices (INDEXED) or unused
  const uint16_t* h;         // this token's activation vector
  const uint16_t* coef_scale;
  __device__ __forceinline__ int row(int t) const { return INDEXED ? idx[t] : t; }
  __device__ __forceinline__ float coef(int t, int j) const {
    float c = T::to_f32(h[j]);
    if (coef_scale) c *= T::to_f32(coef_scale[j]);
    return c;
  }
};

// Row source staged in LDS by the Top-K prologue: (row index, coefficient) pairs for the ranks
// [base, base + n) of this workgroup's segment.
struct LdsRows {
  const int* idx;
  const float* val;
  int base;                  // rank of entry 0
  __device__ __forceinline__ int row(int t) const { return __builtin_amdgcn_readfirstlane(idx[t - base]); }
  __device__ __forceinline__ float coef(int t, int) const { return val[t - base]; }
};

// The identity row list with its coefficients staged in LDS (dense mat-vec: row t is rank t).
struct LdsCoefs {
  const float* val;
  int base;                  // rank of entry 0
  __device__ __forceinline__ int row(int t) const { return t; }
  __device__ __forceinline__ float coef(int t, int) const { return val[t - base]; }
};

// acc[k] += sum over ranks t in [ra, re) of coef(t) * W[row(t), col + k]
template <typename T, typename Rows>
__device__ __forceinline__ void stream_rows(const uint16_t* __restrict__ wcol, int d_out, const Rows& rows, int ra,
                                            int re, float (&acc)[8]) {
  for (int t = ra; t < re; t += kUnroll) {
    int j[kUnroll];
    uint4 v[kUnroll];
    float c[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) j[u] = rows.row(min(t + u, re - 1));
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
      v[u] = load_stream16(wcol + static_cast<size_t>(j[u]) * d_out);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const float cc = rows.coef(min(t + u, re - 1), j[u]);
      c[u] = (t + u < re) ? cc : 0.f;
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      float w[8];
      unpack8<T>(v[u], w);
#pragma unroll
      for (int k = 0; k < 8; ++k) acc[k] = fmaf(c[u], w[k], acc[k]);
    }
  }
}

// Where a workgroup's share of the (strip, rank) space falls.
struct Segment {
  int s;        // strip
  int t0, t1;   // ranks [t0, t1) of the kept list
};

// Epilogue parameters of one launch (see GemvArgs).
struct Epilogue {
  uint16_t* y;
  const uint16_t* rms_src;
  float rms_eps;
  const uint16_t* residual;
  uint16_t* y_pre;
  int d_in, d_out;
  // Paired strips (gate|up): pair_cols = d_ff > 0 makes strip s cover the gate columns
  // [256 s, 256 s + 256) on lanes 0..31 and the up columns d_ff + [256 s, 256 s + 256) on lanes 32..63,
  // so the workgroup that finishes a strip holds both halves of 256 channels and also stores
  // pair_out[b, c] = R(SiLU(R(gate_c)) * R(up_c)).
  int pair_cols = 0;
  uint16_t* pair_out = nullptr;
};

// First output column of a lane in strip s (8 consecutive columns), and whether the lane has any.
__device__ __forceinline__ int strip_lane_col(int s, int lane, int d_out, int pair_cols, bool& valid) {
  if (pair_cols > 0) {
    const int c = s * 256 + (lane & 31) * 8;
    valid = c < pair_cols;
    return (lane >> 5) * pair_cols + c;
  }
  const int col = s * kStripCols + lane * 8;
  valid = col < d_out;
  return col;
}

template <int RW, int NA = 8>
struct GemvShared {
  float red[RW > 1 ? RW - 1 : 1][NA][64];
  float blockred[RW];
  int last;
};

// Sum the RW row-waves through LDS, hand the strip partial to the workspace, and -- in the
// workgroup that arrives last at the strip -- add all partials in workgroup order, apply the
// epilogue and store.  Must be called by every lane of the workgroup; ends with a barrier.
// NA = fp32 accumulators (consecutive output columns) per lane; a strip is 64 * NA columns wide.
//
// Partials travel as relaxed agent-scope 64-bit atomics: such accesses are coherent across the
// chip's L2 slices by themselves, so no cache write-back / invalidate is needed (a release/acquire
// fence pair per wave costs more than the whole mat-vec here).  Order: every lane waits for its
// stores to complete, the workgroup barrier joins the lanes, then one lane bumps the strip's
// arrival counter; the workgroup that observes the last arrival therefore reads completed stores.
// Slot layout [NA/2][64] of float pairs keeps each store instruction one contiguous 512-byte run.
template <typename T, int RW, int NA = 8>
__device__ __forceinline__ void reduce_and_finish(float (&acc)[NA], const Segment& sg, int seg_no, int b, int g, int G,
                                                  int K, int chunk, int nstrips, float* partial, unsigned* counters,
                                                  const Epilogue& ep, GemvShared<RW, NA>& sh, int lane, int rw) {
  constexpr int NT = RW * 64;
  constexpr int SC = 64 * NA;
  const int s = sg.s;
  bool lane_valid = true;
  const int col = (NA == 8 && ep.pair_cols > 0) ? strip_lane_col(s, lane, ep.d_out, ep.pair_cols, lane_valid)
                                                : s * SC + lane * NA;

  if (RW > 1) {
    if (rw > 0) {
#pragma unroll
      for (int k = 0; k < NA; ++k) sh.red[rw - 1][k][lane] = acc[k];
    }
    __syncthreads();
    if (rw == 0) {
      for (int r = 0; r < RW - 1; ++r) {
#pragma unroll
        for (int k = 0; k < NA; ++k) acc[k] += sh.red[r][k][lane];
      }
    }
  }

  // The residual a finishing workgroup adds is fetched now, by every workgroup, so that its latency
  // overlaps the hand-off below instead of following it (16 bytes per lane of one wave).
  // (only in the 8-accumulator geometry: the wide one has no registers to spare for it)
  constexpr bool kPrefetchResidual = NA == 8;
  uint4 res_pref[kPrefetchResidual ? NA / 8 : 1];
  if (kPrefetchResidual && ep.residual && rw == 0) {
#pragma unroll
    for (int c = 0; c < NA / 8; ++c) {
      res_pref[c] = make_uint4(0u, 0u, 0u, 0u);
      if (lane_valid && col + c * 8 < ep.d_out)
        res_pref[c] = *reinterpret_cast<const uint4*>(ep.residual + static_cast<size_t>(b) * ep.d_out + col + c * 8);
    }
  }

  const int g_first = (s * K) / chunk;
  const int g_last = ((s + 1) * K - 1) / chunk;
  const int n_s = g_last - g_first + 1;
  bool last = (n_s == 1);
  if (n_s > 1) {
    unsigned long long* slot = reinterpret_cast<unsigned long long*>(
        partial + ((static_cast<size_t>(b) * G + g) * 2 + seg_no) * SC);
    // one counter per 256 bytes: arrivals at different strips must not share a cache line
    unsigned* ctr = counters + (static_cast<size_t>(b) * nstrips + s) * kCounterStride;
    if (rw == 0) {
#pragma unroll
      for (int k = 0; k < NA / 2; ++k) {
        const unsigned long long v = static_cast<unsigned long long>(__float_as_uint(acc[2 * k])) |
                                     (static_cast<unsigned long long>(__float_as_uint(acc[2 * k + 1])) << 32);
        __hip_atomic_store(slot + k * 64 + lane, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
      const unsigned old = __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      sh.last = (old == static_cast<unsigned>(n_s - 1)) ? 1 : 0;
    }
    __syncthreads();
    last = (sh.last != 0);
    if (last) {
      // row-wave rw adds partials g_first+rw, g_first+rw+RW, ... (kBatch in flight at a time);
      // the RW sub-sums are then added in wave order through LDS: the order never changes.
      constexpr int kBatch = NA <= 8 ? 8 : 2;
#pragma unroll
      for (int k = 0; k < NA; ++k) acc[k] = 0.f;
      for (int gg = g_first + rw; gg <= g_last; gg += kBatch * RW) {
        unsigned long long v[kBatch][NA / 2];
#pragma unroll
        for (int q = 0; q < kBatch; ++q) {
          const int g2 = min(gg + q * RW, g_last);
          const int sgn = ((g2 * chunk) / K != s) ? 1 : 0;
          const unsigned long long* p = reinterpret_cast<const unsigned long long*>(
              partial + ((static_cast<size_t>(b) * G + g2) * 2 + sgn) * SC);
#pragma unroll
          for (int k = 0; k < NA / 2; ++k)
            v[q][k] = __hip_atomic_load(p + k * 64 + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int q = 0; q < kBatch; ++q) {
          if (gg + q * RW <= g_last) {
#pragma unroll
            for (int k = 0; k < NA / 2; ++k) {
              acc[2 * k] += __uint_as_float(static_cast<unsigned>(v[q][k] & 0xFFFFFFFFull));
              acc[2 * k + 1] += __uint_as_float(static_cast<unsigned>(v[q][k] >> 32));
            }
          }
        }
      }
      if (threadIdx.x == 0) __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (RW > 1) {
        if (rw > 0) {
#pragma unroll
          for (int k = 0; k < NA; ++k) sh.red[rw - 1][k][lane] = acc[k];
        }
        __syncthreads();
        if (rw == 0) {
          for (int r = 0; r < RW - 1; ++r) {
#pragma unroll
            for (int k = 0; k < NA; ++k) acc[k] += sh.red[r][k][lane];
          }
        }
      }
    }
  }

  if (last) {   // uniform over the workgroup
    float scale = 1.f;
    if (ep.rms_src) {
      const uint16_t* xs = ep.rms_src + static_cast<size_t>(b) * ep.d_in;
      float ss = 0.f;
      for (int i = threadIdx.x * 8; i < ep.d_in; i += NT * 8) {
        float w[8];
        unpack8<T>(*reinterpret_cast<const uint4*>(xs + i), w);
#pragma unroll
        for (int k = 0; k < 8; ++k) ss = fmaf(w[k], w[k], ss);
      }
      ss = wave_sum(ss);
      if (lane == 0) sh.blockred[rw] = ss;
      __syncthreads();
      float tot = 0.f;
      for (int w2 = 0; w2 < RW; ++w2) tot += sh.blockred[w2];
      scale = 1.0f / sqrtf(tot / static_cast<float>(ep.d_in) + ep.rms_eps);
    }
    if (rw == 0) {
#pragma unroll
      for (int c = 0; c < NA / 8; ++c) {
        const bool ok = lane_valid && col + c * 8 < ep.d_out;   // d_out % 8 == 0: the eight are valid together
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = acc[c * 8 + k] * scale;
        const size_t off = static_cast<size_t>(b) * ep.d_out + col + c * 8;
        if (ok) {
          if (ep.residual) {
            if (ep.y_pre) *reinterpret_cast<uint4*>(ep.y_pre + off) = pack8<T>(v);
            float r[8];
            unpack8<T>(kPrefetchResidual ? res_pref[kPrefetchResidual ? c : 0]
                                         : *reinterpret_cast<const uint4*>(ep.residual + off), r);
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = r[k] + round_store<T>(v[k]);
          }
          *reinterpret_cast<uint4*>(ep.y + off) = pack8<T>(v);
        }
        if (NA == 8 && ep.pair_cols > 0 && ep.pair_out) {
          // lanes 0..31 hold gate, lanes 32..63 the up values of the same channels (all 64 lanes take part
          // in the exchange; the product is formed from the stored, i.e. rounded, values)
          float h[8];
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            const float mine = round_store<T>(v[k]);
            const float up = __shfl(mine, (lane & 31) + 32, kWave);
            h[k] = silu_f32(mine) * up;
          }
          if (ok && lane < 32)
            *reinterpret_cast<uint4*>(ep.pair_out + static_cast<size_t>(b) * ep.pair_cols + (col + c * 8)) = pack8<T>(h);
        }
      }
    }
  }
  __syncthreads();   // LDS is reused by a following segment
}

constexpr int kRowListMax = 2048;   // (strip, rank) pairs of a workgroup whose rows are staged in LDS

// Copy the (row, coefficient) pairs of a workgroup's `count` consecutive (strip, rank) pairs, starting
// at rank t0 of its first strip, into LDS: entries [0, nA) are ranks t0 + e of the first strip,
// entries [nA, count) ranks e - nA of the next one (nA = min(K - t0, count)).  Returns false (and
// copies nothing) when the list does not fit; ends with a barrier otherwise.  Uniform over the workgroup.
template <int NT, int CAP = kRowListMax, typename Rows>
__device__ __forceinline__ bool stage_row_list(const Rows& rows, int t0, int count, int K, int* lst_idx,
                                               float* lst_val) {
  if (count > CAP) return false;
  const int nA = min(K - t0, count);
  for (int e = threadIdx.x; e < count; e += NT) {
    const int t = e < nA ? t0 + e : e - nA;
    const int j = rows.row(t);
    if (lst_idx) lst_idx[e] = j;          // the identity list needs no indices
    lst_val[e] = rows.coef(t, j);
  }
  __syncthreads();
  return true;
}

// The row-streaming mat-vec of workgroup g for token b: its share of the (strip, kept row) pairs,
// at most two segments, each reduced and handed over by reduce_and_finish.  The workgroup first
// copies its ranks' (row, coefficient) pairs into LDS (coalesced; lst_idx / lst_val hold kRowListMax
// entries, the dense form uses only lst_val), so the row loop has no dependent index -> activation
// -> address chain through global memory, and no per-row activation load that the compiler would
// wait for row by row.
template <typename T, int RW, bool INDEXED>
__device__ __forceinline__ void gemv_rows_body(const GemvArgs& a, int g, int b, GemvShared<RW>& sh, int* lst_idx,
                                               float* lst_val) {
  const int lane = threadIdx.x & 63;
  const int rw = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
  const int K = a.K;

  GlobalRows<T, INDEXED> rows;
  rows.idx = INDEXED ? a.idx + static_cast<size_t>(b) * K : nullptr;
  rows.h = a.h + static_cast<size_t>(b) * a.d_in;
  rows.coef_scale = a.coef_scale;
  const Epilogue ep{a.y, a.rms_src, a.rms_eps, a.residual, a.y_pre, a.d_in, a.d_out, 0, nullptr};

  int f0 = g * a.chunk;
  const int f1 = min(f0 + a.chunk, a.nstrips * K);
  Segment sg{f0 / K, 0, 0};
  sg.t0 = f0 - sg.s * K;
  const bool staged = stage_row_list<RW * 64>(rows, sg.t0, f1 - f0, K, INDEXED ? lst_idx : nullptr, lst_val);
  int seg_no = 0;
  int list_base = 0;
  while (f0 < f1) {
    sg.t1 = min(K, sg.t0 + (f1 - f0));
    const int col = sg.s * kStripCols + lane * 8;
    float acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = 0.f;
    // this wave's run of kept rows
    const int n = sg.t1 - sg.t0;
    const int per = (n + RW - 1) / RW;
    const int ra = sg.t0 + rw * per;
    const int re = min(sg.t1, ra + per);
    if (col < a.d_out) {
      if (staged && INDEXED) {
        LdsRows lr;
        lr.idx = lst_idx + list_base;
        lr.val = lst_val + list_base;
        lr.base = sg.t0;
        stream_rows<T>(a.W + col, a.d_out, lr, ra, re, acc);
      } else if (staged) {
        LdsCoefs lc;
        lc.val = lst_val + list_base;
        lc.base = sg.t0;
        stream_rows<T>(a.W + col, a.d_out, lc, ra, re, acc);
      } else {
        stream_rows<T>(a.W + col, a.d_out, rows, ra, re, acc);
      }
    }
    reduce_and_finish<T, RW>(acc, sg, seg_no, b, g, a.G, K, a.chunk, a.nstrips, a.partial, a.counters, ep, sh, lane,
                             rw);
    list_base += n;
    f0 += sg.t1 - sg.t0;
    sg.s += 1;
    sg.t0 = 0;
    seg_no += 1;
  }
}

}  // namespace larosa
