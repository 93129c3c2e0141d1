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
#include "topk_core.hpp"

namespace larosa {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kStripCols = 512;
constexpr int kUnroll = 8;

// 16-byte load of weight data that is read once: the non-temporal hint keeps the stream from
// displacing the small reused vectors (h, indices, partial strips) in the caches.
__device__ __forceinline__ uint4 load_stream16(const uint16_t* p) {
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// Row sources.  batch(t, re, lane, j, c) gives the rows and coefficients of the kUnroll ranks
// t .. t + kUnroll - 1 of the kept list (ranks >= re: any valid row with coefficient zero).

// Read from global memory: indexed (idx != nullptr) or the identity list.
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
  __device__ __forceinline__ void batch(int t, int re, int /*lane*/, int (&j)[kUnroll], float (&c)[kUnroll]) const {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) j[u] = row(min(t + u, re - 1));
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const float cc = coef(min(t + u, re - 1), j[u]);
      c[u] = (t + u < re) ? cc : 0.f;
    }
  }
};

// (row index, coefficient) pairs staged in LDS for the ranks [base, base + n) of a workgroup's segment.
// Lane u of every group of kUnroll lanes reads entry t + u (one LDS instruction each for the indices and
// the coefficients of a whole batch); the values then move to scalar registers, so the row addresses are
// formed on the scalar unit and the row loop has no per-row LDS round trip.
struct LdsRows {
  const int* idx;
  const float* val;
  int base;                  // rank of entry 0
  // one entry at a time (the 4-bit kernels' row loops)
  __device__ __forceinline__ int row(int t) const { return __builtin_amdgcn_readfirstlane(idx[t - base]); }
  __device__ __forceinline__ float coef(int t, int) const { return val[t - base]; }
  __device__ __forceinline__ void batch(int t, int re, int lane, int (&j)[kUnroll], float (&c)[kUnroll]) const {
    const int u0 = lane & (kUnroll - 1);
    const int e = min(t + u0, re - 1) - base;
    const int myj = idx[e];
    const float myc = (t + u0 < re) ? val[e] : 0.f;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      j[u] = __builtin_amdgcn_readlane(myj, u);
      c[u] = __uint_as_float(static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(__float_as_uint(myc)), u)));
    }
  }
};

// The identity row list with its coefficients staged in LDS (dense mat-vec: row t is rank t).
struct LdsCoefs {
  const float* val;
  int base;                  // rank of entry 0
  __device__ __forceinline__ void batch(int t, int re, int lane, int (&j)[kUnroll], float (&c)[kUnroll]) const {
    const int u0 = lane & (kUnroll - 1);
    const float myc = (t + u0 < re) ? val[min(t + u0, re - 1) - base] : 0.f;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      j[u] = min(t + u, re - 1);
      c[u] = __uint_as_float(static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(__float_as_uint(myc)), u)));
    }
  }
};

// acc[k] += sum over ranks t in [ra, re) of coef(t) * W[row(t), col + k]
// kUnroll rows in flight per wave; with two 8-wave workgroups per compute unit other waves' loads cover
// the time a wave spends on its multiply-adds (issuing the next batch before consuming the current one
// costs 32 more registers per lane and measured no faster).
// Every lane of the wave must call this (the row sources exchange values between lanes); lanes without
// output columns in the strip pass active = false and load nothing.
template <typename T, typename Rows>
__device__ __forceinline__ void stream_rows(const uint16_t* __restrict__ wcol, int d_out, const Rows& rows, int ra,
                                            int re, float (&acc)[8], bool active) {
  const int lane = threadIdx.x & 63;
  for (int t = ra; t < re; t += kUnroll) {
    int j[kUnroll];
    float c[kUnroll];
    uint4 v[kUnroll];
    rows.batch(t, re, lane, j, c);
    if (active) {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) v[u] = load_stream16(wcol + static_cast<size_t>(j[u]) * d_out);
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        float w[8];
        unpack8<T>(v[u], w);
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] = fmaf(c[u], w[k], acc[k]);
      }
    }
  }
}

// A workgroup's share of the work: ranks [t0, t1) of the kept list, on strip s.  Workgroup g of a
// launch with `wps` workgroups per strip and `per` ranks per workgroup takes strip g / wps and the
// ranks [j * per, min(K, (j + 1) * per)), j = g mod wps (the planner makes all of them non-empty).
// A workgroup therefore meets exactly one strip, and hands over exactly one partial.
struct Segment {
  int s;        // strip
  int t0, t1;   // ranks [t0, t1) of the kept list
};

__device__ __forceinline__ Segment segment_of(int g, int wps, int per, int K) {
  Segment sg;
  sg.s = g / wps;
  sg.t0 = (g - sg.s * wps) * per;
  sg.t1 = min(K, sg.t0 + per);
  return sg;
}

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
  // Histograms of what the next Top-K will select on (topk_core.hpp, histograms_add_wave): hist_out != nullptr
  // makes the finishing workgroups add the keys of the values they store -- of pair_out when the strips
  // are paired, else of the y columns in [hist_col0, hist_col1) -- each counting hist_weight times.
  unsigned* hist_out = nullptr;
  int hist_col0 = 0, hist_col1 = 0;
  unsigned hist_weight = 1;
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
  alignas(16) float red[RW > 1 ? RW - 1 : 1][NA][64];
  float blockred[RW];
  int last;
};

// Sum the RW row-waves through LDS, hand the strip partial to the workspace, and -- in the
// workgroup that arrives last at the strip -- add all partials in workgroup order, apply the
// epilogue and store.  Must be called by every lane of the workgroup.
// NA = fp32 accumulators (consecutive output columns) per lane; a strip is 64 * NA columns wide.
//
// Partials travel as 16-byte accesses with the sc1 cache policy (what a relaxed agent-scope atomic
// compiles to, four times as wide): such accesses are coherent across the
// chip's L2 slices by themselves, so no cache write-back / invalidate is needed (a release/acquire
// fence pair per wave costs more than the whole mat-vec here).  Order: wave 0, which alone writes the
// partial, waits for its stores to complete, then its lane 0 bumps the strip's arrival counter; the
// workgroup that observes the last arrival therefore reads completed stores.
template <typename T, int RW, int NA = 8>
__device__ __forceinline__ void reduce_and_finish(float (&acc)[NA], int s, int b, int g, int G, int wps,
                                                  float* partial, unsigned* counters, int nstrips,
                                                  const Epilogue& ep, GemvShared<RW, NA>& sh, int lane, int rw) {
  constexpr int NT = RW * 64;
  constexpr int SC = 64 * NA;
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

  LAROSA_STAMP(7);
  const int g_first = s * wps;
  const int g_last = g_first + wps - 1;
  const int n_s = wps;
  bool last = (n_s == 1);
  if (n_s > 1) {
    // the strip's partials as one buffer: partial i (workgroup g_first + i) at byte i * SC * 4, lane's
    // accumulators 4 k4 .. 4 k4 + 3 at (k4 * 64 + lane) * 16 within it (every instruction moves one
    // contiguous KiB); 16-byte accesses that are coherent across the chip (sc1)
    const __amdgpu_buffer_rsrc_t strip_buf = __builtin_amdgcn_make_buffer_rsrc(
        partial + (static_cast<size_t>(b) * G + g_first) * SC, 0, wps * SC * 4, 0x00027000);
    constexpr int kCoherent = 16;   // cache policy: sc1
    // one counter per 256 bytes: arrivals at different strips must not share a cache line
    unsigned* ctr = counters + (static_cast<size_t>(b) * nstrips + s) * kCounterStride;
    if (rw == 0) {
      const int mine = (g - g_first) * SC * 4 + lane * 16;
#pragma unroll
      for (int k4 = 0; k4 < NA / 4; ++k4) {
        const u32x4 v = {__float_as_uint(acc[4 * k4]), __float_as_uint(acc[4 * k4 + 1]), __float_as_uint(acc[4 * k4 + 2]),
                         __float_as_uint(acc[4 * k4 + 3])};
        __builtin_amdgcn_raw_buffer_store_b128(v, strip_buf, mine + k4 * 1024, 0, kCoherent);
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      LAROSA_STAMP(8);
      if (lane == 0) {
        const unsigned old = __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sh.last = (old == static_cast<unsigned>(n_s - 1)) ? 1 : 0;
      }
    }
    __syncthreads();
    LAROSA_STAMP(9);
    last = (sh.last != 0);
    if (last) {
      // row-wave rw adds partials g_first+rw, g_first+rw+RW, ... (kBatch in flight at a time, none read
      // twice); the RW sub-sums are then added in wave order through LDS: the order never changes.
      constexpr int kBatch = NA <= 8 ? 8 : 2;
#pragma unroll
      for (int k = 0; k < NA; ++k) acc[k] = 0.f;
      for (int i0 = rw; i0 < n_s; i0 += kBatch * RW) {
        u32x4 v[kBatch][NA / 4];
#pragma unroll
        for (int q = 0; q < kBatch; ++q) {
          if (i0 + q * RW < n_s) {            // uniform over the wave
#pragma unroll
            for (int k4 = 0; k4 < NA / 4; ++k4)
              v[q][k4] = __builtin_amdgcn_raw_buffer_load_b128(strip_buf, (i0 + q * RW) * SC * 4 + lane * 16 + k4 * 1024, 0,
                                                               kCoherent);
          }
        }
#pragma unroll
        for (int q = 0; q < kBatch; ++q) {
          if (i0 + q * RW < n_s) {
#pragma unroll
            for (int k4 = 0; k4 < NA / 4; ++k4) {
              acc[4 * k4] += __uint_as_float(v[q][k4].x);
              acc[4 * k4 + 1] += __uint_as_float(v[q][k4].y);
              acc[4 * k4 + 2] += __uint_as_float(v[q][k4].z);
              acc[4 * k4 + 3] += __uint_as_float(v[q][k4].w);
            }
          }
        }
      }
      if (threadIdx.x == 0) __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      LAROSA_STAMP(10);
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
  (void)g_last;

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
          const uint4 hp = pack8<T>(h);
          if (ok && lane < 32)
            *reinterpret_cast<uint4*>(ep.pair_out + static_cast<size_t>(b) * ep.pair_cols + (col + c * 8)) = hp;
          if (ep.hist_out) {
            static_assert(sizeof(sh.red) >= 256 * sizeof(unsigned), "the histogram scratch lives in the reduction buffer");
            const uint16_t bits[8] = {static_cast<uint16_t>(hp.x & 0xFFFFu), static_cast<uint16_t>(hp.x >> 16),
                                      static_cast<uint16_t>(hp.y & 0xFFFFu), static_cast<uint16_t>(hp.y >> 16),
                                      static_cast<uint16_t>(hp.z & 0xFFFFu), static_cast<uint16_t>(hp.z >> 16),
                                      static_cast<uint16_t>(hp.w & 0xFFFFu), static_cast<uint16_t>(hp.w >> 16)};
            histograms_add_wave(bits, ok && lane < 32, ep.hist_weight, ep.hist_out + static_cast<size_t>(b) * kHistWords,
                                reinterpret_cast<unsigned*>(&sh.red[0][0][0]), lane);
          }
        } else if (NA == 8 && ep.hist_out) {
          const uint4 yp = pack8<T>(v);     // what was stored to y
          const uint16_t bits[8] = {static_cast<uint16_t>(yp.x & 0xFFFFu), static_cast<uint16_t>(yp.x >> 16),
                                    static_cast<uint16_t>(yp.y & 0xFFFFu), static_cast<uint16_t>(yp.y >> 16),
                                    static_cast<uint16_t>(yp.z & 0xFFFFu), static_cast<uint16_t>(yp.z >> 16),
                                    static_cast<uint16_t>(yp.w & 0xFFFFu), static_cast<uint16_t>(yp.w >> 16)};
          const int c0 = col + c * 8;
          histograms_add_wave(bits, ok && c0 >= ep.hist_col0 && c0 < ep.hist_col1, ep.hist_weight,
                              ep.hist_out + static_cast<size_t>(b) * kHistWords,
                              reinterpret_cast<unsigned*>(&sh.red[0][0][0]), lane);
        }
      }
    }
  }
}

// Copy the (row, coefficient) pairs of the ranks [t0, t0 + count) into LDS (entry e = rank t0 + e).
// Returns false (and copies nothing) when the list does not fit; ends with a barrier otherwise.
// Uniform over the workgroup.
template <int NT, int CAP = kRowListMax, typename Rows>
__device__ __forceinline__ bool stage_row_list(const Rows& rows, int t0, int count, int* lst_idx, float* lst_val) {
  if (count > CAP) return false;
  for (int e = threadIdx.x; e < count; e += NT) {
    const int j = rows.row(t0 + e);
    if (lst_idx) lst_idx[e] = j;          // the identity list needs no indices
    lst_val[e] = rows.coef(t0 + e, j);
  }
  __syncthreads();
  return true;
}

// The RW row-waves of a workgroup share its ranks [t0, t1) in contiguous runs: wave rw takes [ra, re).
template <int RW>
__device__ __forceinline__ void wave_run(int t0, int t1, int rw, int& ra, int& re) {
  const int per = (t1 - t0 + RW - 1) / RW;
  ra = t0 + rw * per;
  re = min(t1, ra + per);
}

// The row-streaming mat-vec of workgroup g for token b: its ranks of its strip, reduced and handed
// over by reduce_and_finish.  The workgroup first copies its ranks' (row, coefficient) pairs into LDS
// (coalesced; lst_idx / lst_val hold kRowListMax entries, the dense form uses only lst_val), so the
// row loop has no dependent index -> activation -> address chain through global memory, and no
// per-row activation load that the compiler would wait for row by row.
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

  const Segment sg = segment_of(g, a.wps, a.chunk, K);
  const bool staged = stage_row_list<RW * 64>(rows, sg.t0, sg.t1 - sg.t0, INDEXED ? lst_idx : nullptr, lst_val);
  const int col = sg.s * kStripCols + lane * 8;
  float acc[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) acc[k] = 0.f;
  int ra, re;
  wave_run<RW>(sg.t0, sg.t1, rw, ra, re);
  const bool active = col < a.d_out;
  if (staged && INDEXED) {
    LdsRows lr;
    lr.idx = lst_idx;
    lr.val = lst_val;
    lr.base = sg.t0;
    stream_rows<T>(a.W + col, a.d_out, lr, ra, re, acc, active);
  } else if (staged) {
    LdsCoefs lc;
    lc.val = lst_val;
    lc.base = sg.t0;
    stream_rows<T>(a.W + col, a.d_out, lc, ra, re, acc, active);
  } else {
    stream_rows<T>(a.W + col, a.d_out, rows, ra, re, acc, active);
  }
  reduce_and_finish<T, RW>(acc, sg.s, b, g, a.G, a.wps, a.partial, a.counters, a.nstrips, ep, sh, lane, rw);
}

}  // namespace larosa
