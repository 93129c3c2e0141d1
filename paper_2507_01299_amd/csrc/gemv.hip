// Row-streaming mat-vec for gfx950: the column-sparse projection of LaRoSA (Sec. 4.3 Eq. 10,
// Sec. 4.4) and, with the identity row list, the dense rotation / adapter / baseline.
//
// The weight is input-channel-major, so a kept input channel is one contiguous run of d_out
// 16-bit values.  A wave owns 512 consecutive output columns (64 lanes x 16 bytes: one kept
// row is a 1 KiB coalesced burst per wave) and a run of kept rows; each lane keeps 8 fp32
// accumulators.  Work is the set of (column strip, kept row) pairs, cut into equal contiguous
// chunks over all workgroups so every workgroup moves the same number of bytes whatever the
// shape.  Inside a workgroup the RW row-waves of a strip are summed through LDS; across
// workgroups, fp32 partial strips go to the workspace and the workgroup that arrives last at
// a strip (agent-scope counter) adds them in workgroup order, which fixes the summation order
// and makes the result run-to-run bit-stable.  The epilogue (pre-norm factor, residual add,
// rounding) runs in that last workgroup.
#include "kernels.hpp"
#include "numeric.hpp"

namespace larosa {

namespace {

constexpr int kUnroll = 8;

template <typename T, int CW, int RW, bool INDEXED>
__global__ __launch_bounds__(CW* RW * 64) void gemv_rows_kernel(GemvArgs a) {
  constexpr int SC = CW * 512;
  constexpr int NT = CW * RW * 64;
  constexpr int NW = CW * RW;
  __shared__ float red[RW > 1 ? RW - 1 : 1][8][CW * 64];
  __shared__ float blockred[NW];
  __shared__ int s_last;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
  const int cw = wave % CW;
  const int rw = wave / CW;
  const int b = blockIdx.y;
  const int g = blockIdx.x;
  const int K = a.K;
  const int d_out = a.d_out;
  const int chunk = a.chunk;

  const uint16_t* hb = a.h + static_cast<size_t>(b) * a.d_in;
  const int32_t* idxb = INDEXED ? a.idx + static_cast<size_t>(b) * K : nullptr;

  int f0 = g * chunk;
  const int f1 = min(f0 + chunk, a.nstrips * K);
  int s = f0 / K;
  int t0 = f0 - s * K;
  int seg = 0;

  while (f0 < f1) {
    const int t1 = min(K, t0 + (f1 - f0));
    const int col = s * SC + cw * 512 + lane * 8;
    const bool colv = col < d_out;
    float acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = 0.f;

    // this wave's run of kept rows
    const int n = t1 - t0;
    const int per = (n + RW - 1) / RW;
    const int ra = t0 + rw * per;
    const int re = min(t1, ra + per);

    if (colv) {
      const uint16_t* wcol = a.W + col;
      for (int t = ra; t < re; t += kUnroll) {
        int j[kUnroll];
        uint4 v[kUnroll];
        float c[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
          const int tt = min(t + u, re - 1);
          j[u] = INDEXED ? idxb[tt] : tt;
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
          v[u] = *reinterpret_cast<const uint4*>(wcol + static_cast<size_t>(j[u]) * d_out);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
          float cc = T::to_f32(hb[j[u]]);
          if (a.coef_scale) cc *= T::to_f32(a.coef_scale[j[u]]);
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

    // sum the RW row-waves of each strip column through LDS
    if (RW > 1) {
      if (rw > 0) {
#pragma unroll
        for (int k = 0; k < 8; ++k) red[rw - 1][k][cw * 64 + lane] = acc[k];
      }
      __syncthreads();
      if (rw == 0) {
        for (int r = 0; r < RW - 1; ++r) {
#pragma unroll
          for (int k = 0; k < 8; ++k) acc[k] += red[r][k][cw * 64 + lane];
        }
      }
    }

    // cross-workgroup sum: the last workgroup to arrive at strip s adds all partials in a fixed order
    const int g_first = (s * K) / chunk;
    const int g_last = ((s + 1) * K - 1) / chunk;
    const int n_s = g_last - g_first + 1;
    bool last = (n_s == 1);
    if (n_s > 1) {
      // Partials travel as relaxed agent-scope 64-bit atomics: such accesses are coherent across
      // the chip's L2 slices by themselves, so no cache write-back / invalidate is needed (a
      // release/acquire fence pair per workgroup costs far more than the whole mat-vec here).
      // Order: every lane waits for its stores to complete, the workgroup barrier joins the lanes,
      // then one lane bumps the strip's arrival counter; the workgroup that observes the last
      // arrival therefore reads completed stores.  Slot layout [4][CW*64] of float pairs keeps
      // each store instruction one contiguous 512-byte run per wave.
      unsigned long long* slot =
          reinterpret_cast<unsigned long long*>(a.partial + ((static_cast<size_t>(b) * a.G + g) * 2 + seg) * SC);
      // one counter per 256 bytes: arrivals at different strips must not share a cache line
      unsigned* ctr = a.counters + (static_cast<size_t>(b) * a.nstrips + s) * kCounterStride;
      if (rw == 0) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const unsigned long long v = static_cast<unsigned long long>(__float_as_uint(acc[2 * k])) |
                                       (static_cast<unsigned long long>(__float_as_uint(acc[2 * k + 1])) << 32);
          __hip_atomic_store(slot + k * (CW * 64) + cw * 64 + lane, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (threadIdx.x == 0) {
        const unsigned old = __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = (old == static_cast<unsigned>(n_s - 1)) ? 1 : 0;
      }
      __syncthreads();
      last = (s_last != 0);
      if (last) {
        // row-wave rw adds partials g_first+rw, g_first+rw+RW, ... (kBatch in flight at a time);
        // the RW sub-sums are then added in wave order through LDS: the order never changes.
        constexpr int kBatch = 8;
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] = 0.f;
        for (int gg = g_first + rw; gg <= g_last; gg += kBatch * RW) {
          unsigned long long v[kBatch][4];
#pragma unroll
          for (int q = 0; q < kBatch; ++q) {
            const int g2 = min(gg + q * RW, g_last);
            const int sg = ((g2 * chunk) / K != s) ? 1 : 0;
            const unsigned long long* p = reinterpret_cast<const unsigned long long*>(
                a.partial + ((static_cast<size_t>(b) * a.G + g2) * 2 + sg) * SC);
#pragma unroll
            for (int k = 0; k < 4; ++k)
              v[q][k] = __hip_atomic_load(p + k * (CW * 64) + cw * 64 + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
#pragma unroll
          for (int q = 0; q < kBatch; ++q) {
            if (gg + q * RW <= g_last) {
#pragma unroll
              for (int k = 0; k < 4; ++k) {
                acc[2 * k] += __uint_as_float(static_cast<unsigned>(v[q][k] & 0xFFFFFFFFull));
                acc[2 * k + 1] += __uint_as_float(static_cast<unsigned>(v[q][k] >> 32));
              }
            }
          }
        }
        if (threadIdx.x == 0) __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (RW > 1) {
          __syncthreads();                 // the first LDS reduction has been consumed by every wave
          if (rw > 0) {
#pragma unroll
            for (int k = 0; k < 8; ++k) red[rw - 1][k][cw * 64 + lane] = acc[k];
          }
          __syncthreads();
          if (rw == 0) {
            for (int r = 0; r < RW - 1; ++r) {
#pragma unroll
              for (int k = 0; k < 8; ++k) acc[k] += red[r][k][cw * 64 + lane];
            }
          }
        }
      }
    }

    if (last) {   // uniform over the workgroup
      float scale = 1.f;
      if (a.rms_src) {
        const uint16_t* xs = a.rms_src + static_cast<size_t>(b) * a.d_in;
        float ss = 0.f;
        for (int i = threadIdx.x * 8; i < a.d_in; i += NT * 8) {
          float w[8];
          unpack8<T>(*reinterpret_cast<const uint4*>(xs + i), w);
#pragma unroll
          for (int k = 0; k < 8; ++k) ss = fmaf(w[k], w[k], ss);
        }
        ss = wave_sum(ss);
        if (lane == 0) blockred[wave] = ss;
        __syncthreads();
        float tot = 0.f;
        for (int w2 = 0; w2 < NW; ++w2) tot += blockred[w2];
        scale = 1.0f / sqrtf(tot / static_cast<float>(a.d_in) + a.rms_eps);
      }
      if (rw == 0 && colv) {
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = acc[k] * scale;
        const size_t off = static_cast<size_t>(b) * d_out + col;
        if (a.residual) {
          if (a.y_pre) *reinterpret_cast<uint4*>(a.y_pre + off) = pack8<T>(v);
          float r[8];
          unpack8<T>(*reinterpret_cast<const uint4*>(a.residual + off), r);
#pragma unroll
          for (int k = 0; k < 8; ++k) v[k] = r[k] + round_store<T>(v[k]);
        }
        *reinterpret_cast<uint4*>(a.y + off) = pack8<T>(v);
      }
    }
    __syncthreads();   // red / s_last / blockred are reused by a second segment

    f0 += t1 - t0;
    s += 1;
    t0 = 0;
    seg += 1;
  }
}

template <typename T, int CW, int RW>
hipError_t launch_shape(const GemvArgs& a, hipStream_t st) {
  dim3 grid(a.G, a.B), block(CW * RW * 64);
  if (a.idx)
    hipLaunchKernelGGL((gemv_rows_kernel<T, CW, RW, true>), grid, block, 0, st, a);
  else
    hipLaunchKernelGGL((gemv_rows_kernel<T, CW, RW, false>), grid, block, 0, st, a);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_variant(const GemvArgs& a, hipStream_t st) {
  switch (tuning().variant) {
    case 1: return launch_shape<T, 1, 16>(a, st);
    case 2: return launch_shape<T, 2, 4>(a, st);
    case 3: return launch_shape<T, 4, 4>(a, st);
    case 4: return launch_shape<T, 1, 4>(a, st);
    case 5: return launch_shape<T, 2, 8>(a, st);
    default: return launch_shape<T, 1, 8>(a, st);
  }
}

}  // namespace

Tuning& tuning() {
  static Tuning t;
  return t;
}

int gemv_strip_cols() {
  switch (tuning().variant) {
    case 2: case 5: return 1024;
    case 3: return 2048;
    default: return 512;
  }
}

GemvPlan plan_gemv(int d_out, int K) {
  GemvPlan p;
  p.strip_cols = gemv_strip_cols();
  p.nstrips = (d_out + p.strip_cols - 1) / p.strip_cols;
  const long T = static_cast<long>(p.nstrips) * K;
  long G = T / tuning().min_rows;
  if (G > tuning().g_target) G = tuning().g_target;
  if (G < p.nstrips) G = p.nstrips;
  p.chunk = static_cast<int>((T + G - 1) / G);
  p.G = static_cast<int>((T + p.chunk - 1) / p.chunk);
  p.partial_floats = static_cast<size_t>(p.G) * 2 * p.strip_cols;
  return p;
}

hipError_t launch_gemv(const GemvArgs& a, bool bf16, hipStream_t s) {
  return bf16 ? launch_variant<BF16>(a, s) : launch_variant<F16>(a, s);
}

}  // namespace larosa
