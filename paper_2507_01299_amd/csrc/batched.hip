// Batched variant of the column-sparse projection for gfx950: B tokens with independent per-token
// index sets.  The union of the tokens' kept rows is what has to be read; at the sparsities of
// interest it is nearly every row once B >= 4 (1 - p^B of them), so the weight is streamed once
// over all rows and each token's dropped channels simply carry a zero coefficient:
//     y[b,:] = sum_j C[b,j] * W[j,:],   C[b,j] = h[b,j] if j in idx_b else 0.
// The same kernels serve the batched rotation / adapter / dense baseline (C = x).
//
//   * the product is a skinny dense contraction (all rows x B tokens), so it runs on the matrix
//     cores (v_mfma_f32_16x16x16 f16/bf16): M = 16 output columns, N = 16 tokens, K = 16 rows,
//     token blocks padded to 16.  A lane loads 8 consecutive columns of 4 rows (16 lanes x 16 bytes
//     = 256 contiguous bytes per row), and a byte permute regroups those registers into the K-runs
//     the instruction wants; the weight never passes through LDS.  Measured on MI355X this kernel is
//     the fastest for every B >= 2 (the fp32-FMA kernel needed 205 us per LLaMA3-8B layer at B = 4 where
//     this one needed 160 us), because the kernel is HBM-bound and the FMA variant spends its issue slots
//     on B x 8 multiply-adds and coefficient reads per 16 bytes loaded;
//   * an fp32-FMA kernel (2 or 4 tokens per workgroup) remains for the one case the 16-bit B
//     operand cannot express: a per-channel coefficient scale applied in fp32 (learned pre-norm
//     scale in front of an explicit rotation).
// Work split (one strip per workgroup, equal runs of rows), cross-workgroup hand-off (16-byte coherent
// stores and loads, arrival counter, the last arrival finishes) and epilogue follow the single-token
// kernel (gemv_core.hpp), with one arrival per workgroup for all its tokens.
#include "gemv_core.hpp"

namespace larosa {

namespace {

constexpr int kBRW = 8;                 // row-waves of the FMA kernel
constexpr int kBThreads = 512;

// ------------------------------------------------------------------------------------------------
// masked coefficient matrix from (h, idx): C[b,:] = 0, then C[b, idx[b,t]] = h[b, idx[b,t]]
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(512) void batch_prep_kernel(const uint16_t* __restrict__ h, const int32_t* __restrict__ idx,
                                                         uint16_t* __restrict__ C, int d_in, int K) {
  const int b = blockIdx.x;
  uint16_t* cb = C + static_cast<size_t>(b) * d_in;
  for (int i = threadIdx.x * 8; i < d_in; i += 512 * 8) *reinterpret_cast<uint4*>(cb + i) = make_uint4(0u, 0u, 0u, 0u);
  __syncthreads();   // this workgroup wrote the whole row itself
  const uint16_t* hb = h + static_cast<size_t>(b) * d_in;
  const int32_t* ib = idx + static_cast<size_t>(b) * K;
  for (int t = threadIdx.x; t < K; t += 512) {
    const int j = ib[t];
    cb[j] = hb[j];
  }
}

struct Geometry {
  int s, t0, t1;          // strip and row range of a segment
  int g_first, g_last;    // workgroups that contribute to the strip
};

// Workgroup g works on strip g / wps only, rows [(g % wps) * chunk, + chunk) of it (plan_batched: every
// workgroup of a strip has rows, all but the last one `chunk` of them).
__device__ __forceinline__ Geometry strip_geometry(int g, int wps, int K, int chunk) {
  const int s = g / wps;
  const int t0 = (g - s * wps) * chunk;
  Geometry q{s, t0, min(K, t0 + chunk), s * wps, s * wps + wps - 1};
  return q;
}

// per-token pre-norm factor 1/sqrt(mean(x^2)+eps): wave w handles tokens w, w+NW, ...
template <typename T, int NW>
__device__ __forceinline__ void token_scales(const BatchArgs& a, int b0, int ntok, float* scale_s, int lane, int wave) {
  for (int bb = wave; bb < ntok; bb += NW) {
    float sc = 1.f;
    const int tok = b0 + bb;
    if (a.rms_src && tok < a.B) {
      const uint16_t* xs = a.rms_src + static_cast<size_t>(tok) * a.d_in;
      float ss = 0.f;
      for (int i = lane * 8; i < a.d_in; i += 64 * 8) {
        float w[8];
        unpack8<T>(*reinterpret_cast<const uint4*>(xs + i), w);
#pragma unroll
        for (int k = 0; k < 8; ++k) ss = fmaf(w[k], w[k], ss);
      }
      ss = wave_sum(ss);
      sc = 1.0f / sqrtf(ss / static_cast<float>(a.d_in) + a.rms_eps);
    }
    if (lane == 0) scale_s[bb] = sc;
  }
}

// epilogue for 8 consecutive columns of one token
template <typename T>
__device__ __forceinline__ void store_out8(const BatchArgs& a, int tok, int col, float (&v)[8], float scale) {
#pragma unroll
  for (int k = 0; k < 8; ++k) v[k] *= scale;
  const size_t off = static_cast<size_t>(tok) * a.d_out + col;
  if (a.residual) {
    if (a.y_pre) *reinterpret_cast<uint4*>(a.y_pre + off) = pack8<T>(v);
    float r[8];
    unpack8<T>(*reinterpret_cast<const uint4*>(a.residual + off), r);
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = r[k] + round_store<T>(v[k]);
  }
  *reinterpret_cast<uint4*>(a.y + off) = pack8<T>(v);
}

// ------------------------------------------------------------------------------------------------
// FMA kernel, NB <= 4 tokens per workgroup
// ------------------------------------------------------------------------------------------------
// Geometry: a workgroup is 8 waves on ONE strip of 128 columns.  Lane (kgrp, m) = (lane / 16,
// lane % 16) owns columns 8m..8m+7 of the strip; one load instruction of a wave covers 4 rows (one
// per kgrp), 256 contiguous bytes each, and 8 such loads are in flight.  The four row groups of a
// wave are summed by two lane exchanges, the 8 waves through LDS, workgroups through the workspace.
// Narrow strips keep the number of workgroups per strip, and so the partial-sum traffic, small.
constexpr int kFStrip = 128;

template <typename T, int NB>
__global__ __launch_bounds__(kBThreads) void skinny_fma_kernel(BatchArgs a) {
  __shared__ float coef[NB][kBatchChunkMax];
  __shared__ float red[kBRW - 1][NB][8][16];
  __shared__ float scale_s[NB];
  __shared__ int s_last;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int rw = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kgrp = lane >> 4;
  const int m = lane & 15;
  const int g = blockIdx.x;
  const int grp = blockIdx.y;
  const int b0 = grp * NB;
  const int K = a.d_in;
  const int chunk = a.chunk;

  {
    const Geometry ge = strip_geometry(g, a.wps, K, chunk);
    const int s = ge.s, t0 = ge.t0, t1 = ge.t1;
    const int n = t1 - t0;
    const int col = s * kFStrip + m * 8;
    const bool colv = col < a.d_out;

    // this segment's coefficients, as floats, for the NB tokens
    for (int e = tid; e < NB * n; e += kBThreads) {
      const int bb = e / n;
      const int t = e - bb * n;
      const int tok = b0 + bb;
      float c = 0.f;
      if (tok < a.B) {
        c = T::to_f32(a.C[static_cast<size_t>(tok) * K + t0 + t]);
        if (a.coef_scale) c *= T::to_f32(a.coef_scale[t0 + t]);
      }
      coef[bb][t] = c;
    }
    __syncthreads();

    float acc[NB][8];
#pragma unroll
    for (int bb = 0; bb < NB; ++bb)
#pragma unroll
      for (int k = 0; k < 8; ++k) acc[bb][k] = 0.f;
    const int per = (n + kBRW - 1) / kBRW;
    const int ra = t0 + rw * per;
    const int re = min(t1, ra + per);
    if (colv) {
      const uint16_t* wcol = a.W + col;
      for (int t = ra; t < re; t += 4 * kUnroll) {
        uint4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
          v[u] = load_stream16(wcol + static_cast<size_t>(min(t + 4 * u + kgrp, re - 1)) * a.d_out);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
          float w[8];
          unpack8<T>(v[u], w);
          const int r = t + 4 * u + kgrp;
          const bool ok = r < re;
          const int ti = min(r, re - 1) - t0;
#pragma unroll
          for (int bb = 0; bb < NB; ++bb) {
            const float c = ok ? coef[bb][ti] : 0.f;
#pragma unroll
            for (int k = 0; k < 8; ++k) acc[bb][k] = fmaf(c, w[k], acc[bb][k]);
          }
        }
      }
    }
    // the four row groups of the wave (fixed order), then the 8 waves through LDS
#pragma unroll
    for (int bb = 0; bb < NB; ++bb)
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        acc[bb][k] += __shfl_xor(acc[bb][k], 16, kWave);
        acc[bb][k] += __shfl_xor(acc[bb][k], 32, kWave);
      }
    if (rw > 0 && kgrp == 0) {
#pragma unroll
      for (int bb = 0; bb < NB; ++bb)
#pragma unroll
        for (int k = 0; k < 8; ++k) red[rw - 1][bb][k][m] = acc[bb][k];
    }
    __syncthreads();
    if (rw == 0 && kgrp == 0) {
      for (int r = 0; r < kBRW - 1; ++r)
#pragma unroll
        for (int bb = 0; bb < NB; ++bb)
#pragma unroll
          for (int k = 0; k < 8; ++k) acc[bb][k] += red[r][bb][k][m];
    }
    __syncthreads();

    const int n_s = ge.g_last - ge.g_first + 1;
    bool last = (n_s == 1);
    if (n_s > 1) {
      // slot: [NB][4][16] float pairs; lane m of the first wave holds columns 8m..8m+7
      const size_t slot_floats = static_cast<size_t>(NB) * kFStrip;
      unsigned long long* slot = reinterpret_cast<unsigned long long*>(
          a.partial + (static_cast<size_t>(grp) * a.G + g) * slot_floats);
      unsigned* ctr = a.counters + (static_cast<size_t>(grp) * a.nstrips + s) * kCounterStride;
      if (rw == 0 && kgrp == 0) {
#pragma unroll
        for (int bb = 0; bb < NB; ++bb)
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const unsigned long long v = static_cast<unsigned long long>(__float_as_uint(acc[bb][2 * k])) |
                                         (static_cast<unsigned long long>(__float_as_uint(acc[bb][2 * k + 1])) << 32);
            __hip_atomic_store(slot + bb * 64 + k * 16 + m, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (tid == 0) {
        const unsigned old = __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = (old == static_cast<unsigned>(n_s - 1)) ? 1 : 0;
      }
      __syncthreads();
      last = (s_last != 0);
      if (last) {
        if (tid == 0) __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // lane group kgrp of wave rw adds partials g_first + 4*rw + kgrp, + 32, ...: 32 partials per pass
#pragma unroll
        for (int bb = 0; bb < NB; ++bb)
#pragma unroll
          for (int k = 0; k < 8; ++k) acc[bb][k] = 0.f;
        for (int gg = ge.g_first + 4 * rw + kgrp; gg <= ge.g_last; gg += 4 * kBRW) {
          const unsigned long long* p = reinterpret_cast<const unsigned long long*>(
              a.partial + (static_cast<size_t>(grp) * a.G + gg) * slot_floats);
          unsigned long long v[NB][4];
#pragma unroll
          for (int bb = 0; bb < NB; ++bb)
#pragma unroll
            for (int k = 0; k < 4; ++k)
              v[bb][k] = __hip_atomic_load(p + bb * 64 + k * 16 + m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
          for (int bb = 0; bb < NB; ++bb)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              acc[bb][2 * k] += __uint_as_float(static_cast<unsigned>(v[bb][k] & 0xFFFFFFFFull));
              acc[bb][2 * k + 1] += __uint_as_float(static_cast<unsigned>(v[bb][k] >> 32));
            }
        }
#pragma unroll
        for (int bb = 0; bb < NB; ++bb)
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            acc[bb][k] += __shfl_xor(acc[bb][k], 16, kWave);
            acc[bb][k] += __shfl_xor(acc[bb][k], 32, kWave);
          }
        if (rw > 0 && kgrp == 0) {
#pragma unroll
          for (int bb = 0; bb < NB; ++bb)
#pragma unroll
            for (int k = 0; k < 8; ++k) red[rw - 1][bb][k][m] = acc[bb][k];
        }
        __syncthreads();
        if (rw == 0 && kgrp == 0) {
          for (int r = 0; r < kBRW - 1; ++r)
#pragma unroll
            for (int bb = 0; bb < NB; ++bb)
#pragma unroll
              for (int k = 0; k < 8; ++k) acc[bb][k] += red[r][bb][k][m];
        }
        __syncthreads();
      }
    }
    if (last) {   // uniform over the workgroup
      token_scales<T, kBRW>(a, b0, NB, scale_s, lane, rw);
      __syncthreads();
      if (rw == 0 && kgrp == 0 && colv) {
#pragma unroll
        for (int bb = 0; bb < NB; ++bb)
          if (b0 + bb < a.B) store_out8<T>(a, b0 + bb, col, acc[bb], scale_s[bb]);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// matrix-core kernel, NTB blocks of 16 tokens per workgroup
// ------------------------------------------------------------------------------------------------
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));

template <typename T>
__device__ __forceinline__ float4_t mfma16(uint2 a, uint2 b, float4_t c);
template <>
__device__ __forceinline__ float4_t mfma16<F16>(uint2 a, uint2 b, float4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(half4_t, a), __builtin_bit_cast(half4_t, b), c, 0, 0, 0);
}
template <>
__device__ __forceinline__ float4_t mfma16<BF16>(uint2 a, uint2 b, float4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(short4_t, a), __builtin_bit_cast(short4_t, b), c, 0,
                                                   0, 0);
}

constexpr int kMStrip = 128;        // output columns per workgroup of the matrix-core kernel
constexpr int kMRW = 8;             // its row-waves
constexpr int kMTileStride = 130;   // floats per token row of an LDS tile (8-byte aligned, spreads tokens over banks)

// Geometry: a workgroup is 8 waves on ONE strip of 128 columns (256 contiguous bytes per row), each
// wave taking its own run of 16-row tiles, two tiles (8 row loads of 16 bytes per lane) in flight.
// Narrow strips keep the number of workgroups that share a strip -- and with it the partial-sum
// traffic, which grows with the token count -- small.
template <typename T, int NTB>
__device__ __forceinline__ void skinny_mfma_body(const BatchArgs& a, int g, int grp) {
  __shared__ float tile[4][16][kMTileStride];
  __shared__ float scale_s[NTB * 16];
  __shared__ int s_last;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int rw = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kgrp = lane >> 4;    // K-run of 4 rows inside a 16-row tile
  const int m = lane & 15;       // column group (A operand) / token (B operand)
  const int b0 = grp * NTB * 16;
  const int K = a.d_in;
  const int chunk = a.chunk;

  LAROSA_STAMP(0);
  {
    const Geometry ge = strip_geometry(g, a.wps, K, chunk);
    const int s = ge.s, t0 = ge.t0, t1 = ge.t1;
    const int n = t1 - t0;
    const int colbase = s * kMStrip + 8 * m;   // this lane's 8 columns (A operand)
    const bool colv = colbase < a.d_out;

    float4_t acc[NTB][8];
#pragma unroll
    for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[tb][i] = float4_t{0.f, 0.f, 0.f, 0.f};

    const int ntiles = (n + 15) / 16;
    const int per = (ntiles + kMRW - 1) / kMRW;
    const int tl0 = rw * per;
    const int tl1 = min(ntiles, tl0 + per);
    for (int tl = tl0; tl < tl1; tl += 2) {
      uint4 v[2][4];
      uint2 bf[2][NTB];
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        // first of this lane's 4 rows; t0 % 8 == 0, so j0 % 4 == 0.  A tile past this wave's run
        // starts at t1: its rows clamp to a valid address and its B operand is zero.
        const int j0 = (tl + h2 < tl1) ? t0 + (tl + h2) * 16 + 4 * kgrp : t1;
        // Every load is unconditional, from an address clamped into the operand (columns past d_out
        // read the strip's first column, tokens past B the last token, rows past t1 a valid row), and
        // what must not count is zeroed afterwards: a load under a lane condition sits in a branch of
        // its own, and the compiler then waits for the earlier loads half-way through issuing them.
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int r = min(j0 + q, t1 - 1);
          v[h2][q] = load_stream16(a.W + static_cast<size_t>(r) * a.d_out + (colv ? colbase : s * kMStrip));
        }
        // B operand: 4 consecutive rows of token (b0 + tb*16 + m); rows at or past t1 belong to
        // another workgroup (or do not exist) and must contribute nothing
#pragma unroll
        for (int tb = 0; tb < NTB; ++tb) {
          const int tok = b0 + tb * 16 + m;
          // j0 % 4 == 0 and K % 8 == 0, so min(j0, K - 4) keeps the four rows inside the token's vector
          uint2 c = *reinterpret_cast<const uint2*>(a.C + static_cast<size_t>(min(tok, a.B - 1)) * K + min(j0, K - 4));
          if (j0 + 1 >= t1) c.x &= 0x0000FFFFu;
          if (j0 + 2 >= t1) c.y = 0u;
          if (j0 + 3 >= t1) c.y &= 0x0000FFFFu;
          if (j0 >= t1 || tok >= a.B) c.x = 0u;
          if (tok >= a.B) c.y = 0u;
          bf[h2][tb] = c;
        }
      }
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        // A operand for column offset i: element i of each of the 4 row registers
        const uint32_t* vw0 = reinterpret_cast<const uint32_t*>(&v[h2][0]);
        const uint32_t* vw1 = reinterpret_cast<const uint32_t*>(&v[h2][1]);
        const uint32_t* vw2 = reinterpret_cast<const uint32_t*>(&v[h2][2]);
        const uint32_t* vw3 = reinterpret_cast<const uint32_t*>(&v[h2][3]);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
          uint2 af;
          af.x = __builtin_amdgcn_perm(vw1[i >> 1], vw0[i >> 1], sel);
          af.y = __builtin_amdgcn_perm(vw3[i >> 1], vw2[i >> 1], sel);
#pragma unroll
          for (int tb = 0; tb < NTB; ++tb) acc[tb][i] = mfma16<T>(af, bf[h2][tb], acc[tb][i]);
        }
      }
    }

    LAROSA_STAMP(1);
    const int n_s = ge.g_last - ge.g_first + 1;
    const size_t slot_floats = static_cast<size_t>(NTB) * 16 * kMStrip;
    unsigned* ctr = a.counters + (static_cast<size_t>(grp) * a.nstrips + s) * kCounterStride;
    // every partial of this token group as one buffer (slot of workgroup w at byte w * slot bytes; a thread's 16 bytes of token block tb at tb * 8 KiB + tid * 16 within it);
    // 16-byte accesses with the sc1 cache policy are coherent across the chip, see gemv_core.hpp
    const int slot_bytes = NTB * 8192;
    const __amdgpu_buffer_rsrc_t slots = __builtin_amdgcn_make_buffer_rsrc(
        a.partial + static_cast<size_t>(grp) * a.G * slot_floats, 0, a.G * slot_bytes, 0x00027000);
    constexpr int kCoherent = 16;
    const int my_slot = g * slot_bytes;

    // Sum the 8 row-waves of token block tb: waves 0-3 write their tiles, waves 4-7 add theirs on
    // top, then every thread adds the four tiles for its two float pairs (pair q: token q / 64,
    // columns 2*(q % 64), +1).  D element e of MFMA i in lane (kgrp, m) is column 32*kgrp + 8*e + i
    // of token m.  The order of the additions is fixed.
    auto reduce_tb = [&](int tb, float2 (&sm)[2]) {
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        if ((rw >> 2) == r) {
#pragma unroll
          for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              float* p = &tile[rw & 3][m][32 * kgrp + 8 * e + i];
              *p = (r == 0) ? acc[tb][i][e] : *p + acc[tb][i][e];
            }
        }
        __syncthreads();
      }
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int q = tid + k * kBThreads;
        float2 t = *reinterpret_cast<const float2*>(&tile[0][q >> 6][(q & 63) * 2]);
#pragma unroll
        for (int w = 1; w < 4; ++w) {
          const float2 u = *reinterpret_cast<const float2*>(&tile[w][q >> 6][(q & 63) * 2]);
          t.x += u.x;
          t.y += u.y;
        }
        sm[k] = t;
      }
      __syncthreads();
    };
    // epilogue of one token block: its 16 x 128 sums (pairs held as in reduce_tb) go through tile[0]
    auto tile_out = [&](int tb, const float2 (&sm)[2]) {
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int q = tid + k * kBThreads;
        *reinterpret_cast<float2*>(&tile[0][q >> 6][(q & 63) * 2]) = sm[k];
      }
      __syncthreads();
      if (tid < 256) {
        const int tok = b0 + tb * 16 + (tid >> 4);
        const int col = s * kMStrip + (tid & 15) * 8;
        if (tok < a.B && col < a.d_out) {
          float v[8];
          const float* p = &tile[0][tid >> 4][(tid & 15) * 8];
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = p[e];
          store_out8<T>(a, tok, col, v, scale_s[tb * 16 + (tid >> 4)]);
        }
      }
      __syncthreads();
    };

    if (n_s == 1) {
      token_scales<T, kMRW>(a, b0, NTB * 16, scale_s, lane, rw);
      __syncthreads();
#pragma unroll
      for (int tb = 0; tb < NTB; ++tb) {
        float2 sm[2];
        reduce_tb(tb, sm);
        tile_out(tb, sm);
      }
    } else {
#pragma unroll
      for (int tb = 0; tb < NTB; ++tb) {
        float2 sm[2];
        reduce_tb(tb, sm);
        // the thread's two float pairs of the block as one 16-byte chip-coherent store
        const u32x4 v = {__float_as_uint(sm[0].x), __float_as_uint(sm[0].y), __float_as_uint(sm[1].x), __float_as_uint(sm[1].y)};
        __builtin_amdgcn_raw_buffer_store_b128(v, slots, my_slot + tb * 8192 + tid * 16, 0, kCoherent);
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      LAROSA_STAMP(2);
      if (tid == 0) {
        const unsigned old = __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = (old == static_cast<unsigned>(n_s - 1)) ? 1 : 0;
      }
      __syncthreads();
      LAROSA_STAMP(3);
      if (s_last != 0) {   // uniform over the workgroup
        if (tid == 0) __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        token_scales<T, kMRW>(a, b0, NTB * 16, scale_s, lane, rw);
        for (int tb = 0; tb < NTB; ++tb) {
          // each thread owns 2 float pairs of the block and adds the partials in workgroup order
          float2 sum[2];
          sum[0] = sum[1] = make_float2(0.f, 0.f);
          for (int gg = ge.g_first; gg <= ge.g_last; gg += 8) {
            u32x4 v[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
              if (gg + q <= ge.g_last) {          // uniform over the workgroup: no partial is read twice
                v[q] = __builtin_amdgcn_raw_buffer_load_b128(slots, (gg + q) * slot_bytes + tb * 8192 + tid * 16, 0, kCoherent);
              }
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) {
              if (gg + q <= ge.g_last) {
                sum[0].x += __uint_as_float(v[q].x);
                sum[0].y += __uint_as_float(v[q].y);
                sum[1].x += __uint_as_float(v[q].z);
                sum[1].y += __uint_as_float(v[q].w);
              }
            }
          }
          tile_out(tb, sum);
        }
      }
    }
  }
  LAROSA_STAMP(5);
}


// One launch, up to two independent products: workgroups [0, side_G) of the grid run the side product
// (a residual adapter on a block's shortcut, which needs only the block's input), the others the main
// one.  Both use the same token grouping (blockIdx.y).
template <typename T, int NTB>
__global__ __launch_bounds__(kBThreads) void skinny_mfma_kernel(BatchPair p) {
  const int g = blockIdx.x;
  const bool side = g < p.side_G;                       // uniform over the workgroup
  skinny_mfma_body<T, NTB>(side ? p.side : p.main, side ? g : g - p.side_G, blockIdx.y);
}

}  // namespace
bool batched_uses_mfma(int B, bool coef_scale);
namespace {

template <typename T>
hipError_t launch_batched_t(const BatchPair& p, hipStream_t st) {
  const BatchArgs& a = p.main;
  const dim3 block(kBThreads);
  if (!batched_uses_mfma(a.B, a.coef_scale != nullptr)) {
    if (p.side_G > 0) return hipErrorInvalidValue;   // the FMA kernel carries no side product
    // (a per-channel coefficient scale is applied in fp32, which only the FMA kernel does)
    if (a.B <= 2) {
      hipLaunchKernelGGL((skinny_fma_kernel<T, 2>), dim3(a.G, (a.B + 1) / 2), block, 0, st, a);
    } else {
      hipLaunchKernelGGL((skinny_fma_kernel<T, 4>), dim3(a.G, (a.B + 3) / 4), block, 0, st, a);
    }
  } else if (a.B <= 16) {
    hipLaunchKernelGGL((skinny_mfma_kernel<T, 1>), dim3(a.G + p.side_G, 1), block, 0, st, p);
  } else {
    hipLaunchKernelGGL((skinny_mfma_kernel<T, 2>), dim3(a.G + p.side_G, (a.B + 31) / 32), block, 0, st, p);
  }
  return hipGetLastError();
}

}  // namespace

bool batched_uses_mfma(int B, bool coef_scale) { return B >= 2 && !coef_scale; }

int batched_g_total() { return tuning().g_target > 0 ? tuning().g_target : 256; }

int batched_tokens_per_group(int B, bool coef_scale) {
  if (batched_uses_mfma(B, coef_scale)) return B <= 16 ? 16 : 32;
  return B <= 2 ? 2 : 4;
}

GemvPlan plan_batched(int d_in, int d_out, bool mfma, int g_hint) {
  GemvPlan p;
  p.strip_cols = 128;   // both batched kernels work on 128-column strips
  p.nstrips = (d_out + p.strip_cols - 1) / p.strip_cols;
  // one workgroup per compute unit: each strip gets the same number of workgroups, each of those an equal run
  // of whole 16-row tiles (keeps row starts 8-aligned), so a workgroup never works on two strips
  long G = g_hint > 0 ? g_hint : batched_g_total();
  long wps = G / p.nstrips;
  if (wps < 1) wps = 1;
  long chunk = (d_in + wps - 1) / wps;
  chunk = (chunk + 15) / 16 * 16;
  if (!mfma && chunk > kBatchChunkMax) chunk = kBatchChunkMax;   // LDS staging of the coefficients
  wps = (d_in + chunk - 1) / chunk;
  p.chunk = static_cast<int>(chunk);
  p.wps = static_cast<int>(wps);
  p.G = static_cast<int>(p.nstrips * wps);
  p.partial_floats = static_cast<size_t>(p.G) * p.strip_cols;  // per token
  return p;
}

hipError_t launch_batch_prep(const uint16_t* h, const int32_t* idx, uint16_t* C, int B, int d_in, int K, hipStream_t s) {
  hipLaunchKernelGGL(batch_prep_kernel, dim3(B), dim3(512), 0, s, h, idx, C, d_in, K);
  return hipGetLastError();
}

hipError_t launch_batched(const BatchArgs& a, bool bf16, hipStream_t s) {
  BatchPair p{};
  p.main = a;
  return bf16 ? launch_batched_t<BF16>(p, s) : launch_batched_t<F16>(p, s);
}

hipError_t launch_batched_pair(const BatchPair& p, bool bf16, hipStream_t s) {
  return bf16 ? launch_batched_t<BF16>(p, s) : launch_batched_t<F16>(p, s);
}

}  // namespace larosa
