// Stand-alone Top-K sparsifier kernel (Sec. 4.3, Eq. 8): one workgroup of 1024 lanes per token;
// the selection itself is in topk_core.hpp.
#include "kernels.hpp"
#include "topk_core.hpp"

namespace larosa {

namespace {

#ifndef LAROSA_TOPK_KERNEL_COPIES
#define LAROSA_TOPK_KERNEL_COPIES kTopkCopiesWide
#endif
constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / 64;

// Where the selected vector comes from (batched decoder layer): the plain vector, the context-length-1
// attention output read straight from q|k|v (value head of the query head's group), or
// R(SiLU(gate) * up) computed from gate|up.  The vector itself can be written out as well.
template <typename T, int E>   // E elements per lane, multiple of 4
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(const uint16_t* __restrict__ h, int d, int K,
                                                            int32_t* __restrict__ idx,
                                                            uint16_t* __restrict__ vals,
                                                            uint16_t* __restrict__ masked, TopkSource sc) {
  __shared__ TopkShared<kTopkWaves, LAROSA_TOPK_KERNEL_COPIES> sm;
  const int b = blockIdx.x;
  const uint16_t* hb = h + static_cast<size_t>(b) * d;
  const int base = threadIdx.x * E;

  LAROSA_STAMP(0);
  topk_clear<kTopkWaves>(sm);             // made visible by the first barrier below
  // All of the lane's loads are issued first, unconditionally and from addresses clamped into the
  // vector (d % 4 == 0: a group of four is all valid or all past the end; groups past the end re-read
  // the last group and are ignored).  Loads under a lane or mode condition sit in branches of their
  // own, and each is then waited for before the next is issued: one memory round trip per group.
  uint2 ld0[E / 4], ld1[E / 4];
  if (sc.mode == kSrcGqa) {
#pragma unroll
    for (int q = 0; q < E / 4; ++q) {
      const int i = min(base + q * 4, d - 4);
      const int head = i / sc.head_dim;
      const int src = (head / sc.group) * sc.head_dim + (i - head * sc.head_dim);
      ld0[q] = *reinterpret_cast<const uint2*>(sc.src + static_cast<size_t>(b) * (sc.d_q + 2 * sc.d_kv) + sc.d_q +
                                               sc.d_kv + src);
      ld1[q] = make_uint2(0u, 0u);
    }
  } else if (sc.mode == kSrcSilu) {
    const uint16_t* gb = sc.src + static_cast<size_t>(b) * 2 * d;
#pragma unroll
    for (int q = 0; q < E / 4; ++q) {
      const int i = min(base + q * 4, d - 4);
      ld0[q] = *reinterpret_cast<const uint2*>(gb + i);
      ld1[q] = *reinterpret_cast<const uint2*>(gb + d + i);
    }
  } else {
#pragma unroll
    for (int q = 0; q < E / 4; ++q) {
      ld0[q] = *reinterpret_cast<const uint2*>(hb + min(base + q * 4, d - 4));
      ld1[q] = make_uint2(0u, 0u);
    }
  }
  uint16_t raw[E];
#pragma unroll
  for (int q = 0; q < E / 4; ++q) {
    const int i = base + q * 4;
    uint2 v = ld0[q];
    if (sc.mode == kSrcSilu) {
      float g[4], u[4];
      T::unpack2(ld0[q].x, g[0], g[1]);
      T::unpack2(ld0[q].y, g[2], g[3]);
      T::unpack2(ld1[q].x, u[0], u[1]);
      T::unpack2(ld1[q].y, u[2], u[3]);
      uint16_t o[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) o[k] = T::from_f32(silu_f32(g[k]) * u[k]);
      v.x = o[0] | (static_cast<uint32_t>(o[1]) << 16);
      v.y = o[2] | (static_cast<uint32_t>(o[3]) << 16);
    }
    if (i >= d) v = make_uint2(0u, 0u);
    if (i < d && sc.h_out && sc.mode != kSrcNorm) *reinterpret_cast<uint2*>(sc.h_out + static_cast<size_t>(b) * d + i) = v;
    raw[q * 4 + 0] = static_cast<uint16_t>(v.x & 0xFFFFu);
    raw[q * 4 + 1] = static_cast<uint16_t>(v.x >> 16);
    raw[q * 4 + 2] = static_cast<uint16_t>(v.y & 0xFFFFu);
    raw[q * 4 + 3] = static_cast<uint16_t>(v.y >> 16);
  }
  const int nvalid = max(0, min(E, d - base));
  if (sc.mode == kSrcNorm) {
    // h = R(x * rsqrt(mean(x^2) + eps) * scale): the pre-norm of a block whose rotation is absorbed
    // the lane's slice of the learned scale, fetched up front (loads at each use would each wait for memory)
    uint2 sc2[E / 4];
#pragma unroll
    for (int q = 0; q < E / 4; ++q) {
      const int i = base + q * 4;
      sc2[q] = (sc.norm_scale && i < d) ? *reinterpret_cast<const uint2*>(sc.norm_scale + i) : make_uint2(0u, 0u);
    }
    float ss = 0.f;
#pragma unroll
    for (int q = 0; q < E; ++q) {
      const float xv = (q < nvalid) ? T::to_f32(raw[q]) : 0.f;
      ss = fmaf(xv, xv, ss);
    }
    ss = wave_sum(ss);
    float* tot_w = reinterpret_cast<float*>(sm.wave_tot);
    if ((threadIdx.x & 63) == 0) tot_w[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
    for (int w2 = 0; w2 < kTopkWaves; ++w2) tot += tot_w[w2];   // the select writes wave_tot only after further barriers
    const float rinv = 1.0f / sqrtf(tot / static_cast<float>(d) + sc.norm_eps);
#pragma unroll
    for (int q = 0; q < E; ++q) {
      float xv = T::to_f32(raw[q]) * rinv;
      const uint32_t w = (q & 2) ? sc2[q >> 2].y : sc2[q >> 2].x;
      if (sc.norm_scale) xv *= T::to_f32(static_cast<uint16_t>((q & 1) ? (w >> 16) : (w & 0xFFFFu)));
      raw[q] = (q < nvalid) ? T::from_f32(xv) : static_cast<uint16_t>(0);   // padding stays zero
    }
    if (sc.h_out) {
#pragma unroll
      for (int q = 0; q < E / 4; ++q) {
        const int i = base + q * 4;
        if (i < d) {
          uint2 v;
          v.x = raw[q * 4 + 0] | (static_cast<uint32_t>(raw[q * 4 + 1]) << 16);
          v.y = raw[q * 4 + 2] | (static_cast<uint32_t>(raw[q * 4 + 3]) << 16);
          *reinterpret_cast<uint2*>(sc.h_out + static_cast<size_t>(b) * d + i) = v;
        }
      }
    }
  }
  if (sc.mode != kSrcNorm) __syncthreads();
  LAROSA_STAMP(1);
  const auto st = block_select<kTopkWaves, E>(raw, K, sm);
  LAROSA_STAMP(2);

  int32_t* idxb = idx ? idx + static_cast<size_t>(b) * K : nullptr;   // the index list is optional
  uint16_t* valb = vals ? vals + static_cast<size_t>(b) * K : nullptr;
  uint16_t mk[E];
#pragma unroll
  for (int q = 0; q < E; ++q) mk[q] = 0;
  for_each_kept<E>(st, [&](int q, unsigned pos, bool kept) {
    if (kept) {
      if (idxb) idxb[pos] = base + q;
      if (valb) valb[pos] = raw[q];
    }
    mk[q] = kept ? raw[q] : static_cast<uint16_t>(0);
  });
  LAROSA_STAMP(3);
  if (masked) {
    uint16_t* mb = masked + static_cast<size_t>(b) * d;
#pragma unroll
    for (int q = 0; q < E / 4; ++q) {
      const int i = base + q * 4;
      if (i < d) {
        uint2 v;
        v.x = mk[q * 4 + 0] | (static_cast<uint32_t>(mk[q * 4 + 1]) << 16);
        v.y = mk[q * 4 + 2] | (static_cast<uint32_t>(mk[q * 4 + 3]) << 16);
        *reinterpret_cast<uint2*>(mb + i) = v;
      }
    }
  }
  LAROSA_STAMP(4);
}

// Magnitude-threshold sparsifier (Eq. 4-5), the comparison method with a data-dependent kept count:
// lane t owns elements [tE, (t+1)E); kept positions come from a block prefix sum of the lanes' counts.
template <typename T, int E>
__global__ __launch_bounds__(kTopkThreads) void threshold_kernel(const uint16_t* __restrict__ h, int d, float eps,
                                                                 int32_t* __restrict__ idx,
                                                                 int32_t* __restrict__ count) {
  __shared__ unsigned wave_total[kTopkWaves];
  const int b = blockIdx.x;
  const uint16_t* hb = h + static_cast<size_t>(b) * d;
  const int base = threadIdx.x * E;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  unsigned keep = 0;     // bit q: element base + q is kept
  unsigned n = 0;
#pragma unroll
  for (int q = 0; q < E / 4; ++q) {
    const int i = base + q * 4;
    if (i < d) {
      const uint2 v = *reinterpret_cast<const uint2*>(hb + i);
      const uint16_t r[4] = {static_cast<uint16_t>(v.x & 0xFFFFu), static_cast<uint16_t>(v.x >> 16),
                             static_cast<uint16_t>(v.y & 0xFFFFu), static_cast<uint16_t>(v.y >> 16)};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (T::to_f32(r[k] & 0x7FFFu) > eps) {
          keep |= 1u << (q * 4 + k);
          n += 1;
        }
      }
    }
  }
  const unsigned incl = wave_scan_inclusive(n, lane);
  if (lane == 63) wave_total[wv] = incl;
  __syncthreads();
  unsigned before = incl - n, total = 0;
#pragma unroll
  for (int w2 = 0; w2 < kTopkWaves; ++w2) {
    const unsigned tw = wave_total[w2];
    if (w2 < wv) before += tw;
    total += tw;
  }
  int32_t* idxb = idx + static_cast<size_t>(b) * d;
#pragma unroll
  for (int q = 0; q < E; ++q) {
    if (keep & (1u << q)) idxb[before++] = base + q;
  }
  if (threadIdx.x == 0) count[b] = static_cast<int32_t>(total);
}

template <typename T>
hipError_t launch_threshold_t(const uint16_t* h, int B, int d, float eps, int32_t* idx, int32_t* count, hipStream_t s) {
  dim3 grid(B), block(kTopkThreads);
  const int e = (d + kTopkThreads - 1) / kTopkThreads;
  if (e <= 4)
    hipLaunchKernelGGL((threshold_kernel<T, 4>), grid, block, 0, s, h, d, eps, idx, count);
  else if (e <= 8)
    hipLaunchKernelGGL((threshold_kernel<T, 8>), grid, block, 0, s, h, d, eps, idx, count);
  else if (e <= 16)
    hipLaunchKernelGGL((threshold_kernel<T, 16>), grid, block, 0, s, h, d, eps, idx, count);
  else if (e <= 32)
    hipLaunchKernelGGL((threshold_kernel<T, 32>), grid, block, 0, s, h, d, eps, idx, count);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace

hipError_t launch_threshold_select(const uint16_t* h, int B, int d, float eps, int32_t* idx, int32_t* count, bool bf16,
                                   hipStream_t s) {
  return bf16 ? launch_threshold_t<BF16>(h, B, d, eps, idx, count, s) : launch_threshold_t<F16>(h, B, d, eps, idx, count, s);
}

template <typename T>
hipError_t launch_topk_t(const uint16_t* h, int B, int d, int K, int32_t* idx, uint16_t* vals, uint16_t* masked,
                         const TopkSource& sc, hipStream_t s) {
  dim3 grid(B), block(kTopkThreads);
  const int e = (d + kTopkThreads - 1) / kTopkThreads;
  if (e <= 4)
    hipLaunchKernelGGL((topk_kernel<T, 4>), grid, block, 0, s, h, d, K, idx, vals, masked, sc);
  else if (e <= 8)
    hipLaunchKernelGGL((topk_kernel<T, 8>), grid, block, 0, s, h, d, K, idx, vals, masked, sc);
  else if (e <= 16)
    hipLaunchKernelGGL((topk_kernel<T, 16>), grid, block, 0, s, h, d, K, idx, vals, masked, sc);
  else if (e <= 24)
    hipLaunchKernelGGL((topk_kernel<T, 24>), grid, block, 0, s, h, d, K, idx, vals, masked, sc);
  else if (e <= 32)
    hipLaunchKernelGGL((topk_kernel<T, 32>), grid, block, 0, s, h, d, K, idx, vals, masked, sc);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_topk(const uint16_t* h, int B, int d, int K, int32_t* idx, uint16_t* vals, uint16_t* masked,
                       hipStream_t s) {
  TopkSource sc{};
  sc.mode = kSrcPlain;
  return launch_topk_t<F16>(h, B, d, K, idx, vals, masked, sc, s);   // the type matters for kSrcSilu only
}

hipError_t launch_topk_from(const TopkSource& sc, int B, int d, int K, int32_t* idx, uint16_t* masked, bool bf16,
                            hipStream_t s) {
  return bf16 ? launch_topk_t<BF16>(sc.src, B, d, K, idx, nullptr, masked, sc, s)
              : launch_topk_t<F16>(sc.src, B, d, K, idx, nullptr, masked, sc, s);
}

}  // namespace larosa
