// Column-sparse projection over 4-bit weights (W4A16): the row-streaming mat-vec of gemv.hip with
// the kept rows read as packed 4-bit codes and dequantised in registers.  The paper shows that the
// method keeps its accuracy on 4-bit weights (Sec. 5.4, Table 9) and leaves a kernel that does
// both to future work; the storage format below is this library's own.
//
// Format.  Row j of the input-channel-major weight [d_in, d_out] is d_out / 8 dwords; nibble k
// (bits 4k .. 4k+3) of dword m holds the code q of column 8 m + k, and the weight is
// (q - 8) * s[j, (8 m + k) / 128] with one 16-bit scale per row and per group of 128 output columns
// (round-to-nearest codes, symmetric).  Groups run along a row, so the scale folds into the
// row's coefficient: y[o] = sum_t (h_t s_t,g(o)) (q_t,o - 8).
//
// Two geometries.  Wide (rows of at least 32768 columns, a multiple of 32): a wave owns 2048 output
// columns, a lane 32 of them (16 bytes per kept row, 1 KiB bursts, one scale), 8 rows in flight, 32
// accumulators per lane.  Narrow (anything else): the 16-bit kernel's 512-column strips, one dword
// per lane and row, 16 rows in flight.  The -8 offset is applied once per lane as -8 * sum of
// coefficients.  Reductions, cross-workgroup hand-off and epilogue are shared with the 16-bit kernel.
#include "gemv_core.hpp"

namespace larosa {

namespace {

constexpr int kW4Unroll = 16;
constexpr int kW4Group = 128;

__device__ __forceinline__ uint32_t load_stream4(const uint32_t* p) { return __builtin_nontemporal_load(p); }

// acc[k] += c * q_k for the 8 codes of one dword.  (v >> 4k) & 0x000F000F leaves codes k and k + 4 in
// the two 16-bit halves of a register; read as binary16 each half is the subnormal q * 2^-24 exactly,
// and the mixed-precision FMA takes it straight from the register half with the coefficient (scaled
// by 2^24, exact unless |coefficient| exceeds 2^104, far beyond any activation times scale) and the sum in
// fp32: two instructions per code instead of extract + convert + FMA.  Needs binary16 subnormals kept
// (the default float mode of a HIP kernel), which the parity tests would show at once if it were off.
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
constexpr float kW4CodeScale = 16777216.0f;   // 2^24

__device__ __forceinline__ void fma_codes8(uint32_t v, float c_scaled, float* acc) {
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const f16x2 p = __builtin_bit_cast(f16x2, (v >> (4 * k)) & 0x000F000Fu);
    acc[k] = fmaf(static_cast<float>(p.x), c_scaled, acc[k]);
    acc[k + 4] = fmaf(static_cast<float>(p.y), c_scaled, acc[k + 4]);
  }
}

template <typename T, typename Rows>
__device__ __forceinline__ void stream_rows_w4(const uint32_t* __restrict__ wcol, int row_dwords,
                                               const uint16_t* __restrict__ scol, int ng, const Rows& rows, int ra,
                                               int re, float (&acc)[8]) {
  float csum = 0.f;
  for (int t = ra; t < re; t += kW4Unroll) {
    int j[kW4Unroll];
    uint32_t v[kW4Unroll];
    uint16_t s[kW4Unroll];
#pragma unroll
    for (int u = 0; u < kW4Unroll; ++u) j[u] = rows.row(min(t + u, re - 1));
#pragma unroll
    for (int u = 0; u < kW4Unroll; ++u) {
      v[u] = load_stream4(wcol + static_cast<size_t>(j[u]) * row_dwords);
      s[u] = scol[static_cast<size_t>(j[u]) * ng];
    }
#pragma unroll
    for (int u = 0; u < kW4Unroll; ++u) {
      float c = rows.coef(min(t + u, re - 1), j[u]) * T::to_f32(s[u]);
      c = (t + u < re) ? c : 0.f;
      csum += c;
      fma_codes8(v[u], c * kW4CodeScale, acc);
    }
  }
#pragma unroll
  for (int k = 0; k < 8; ++k) acc[k] = fmaf(-8.0f, csum, acc[k]);
}

// Wide geometry: a lane reads 16 bytes (32 codes, one scale group) per kept row, a wave 2048 columns.
constexpr int kW4WideAcc = 32;
constexpr int kW4WideCols = 64 * kW4WideAcc;
constexpr int kW4WideUnroll = 8;
constexpr int kW4WideList = 512;

template <typename T, typename Rows>
__device__ __forceinline__ void stream_rows_w4_wide(const uint32_t* __restrict__ wcol, int row_dwords,
                                                    const uint16_t* __restrict__ scol, int ng, const Rows& rows,
                                                    int ra, int re, float (&acc)[kW4WideAcc]) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  float csum = 0.f;
  for (int t = ra; t < re; t += kW4WideUnroll) {
    int j[kW4WideUnroll];
    u32x4 v[kW4WideUnroll];
    uint32_t s[kW4WideUnroll];
#pragma unroll
    for (int u = 0; u < kW4WideUnroll; ++u) j[u] = rows.row(min(t + u, re - 1));
#pragma unroll
    for (int u = 0; u < kW4WideUnroll; ++u) s[u] = scol[static_cast<size_t>(j[u]) * ng];
#pragma unroll
    for (int u = 0; u < kW4WideUnroll; ++u)
      v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(wcol + static_cast<size_t>(j[u]) * row_dwords));
    // All scales must be in registers here.  Without this the compiler sinks each scale load to its
    // use and waits for it there: one memory round trip per row instead of one per batch of rows.
#pragma unroll
    for (int u = 0; u < kW4WideUnroll; ++u) asm volatile("" : "+v"(s[u]));
#pragma unroll
    for (int u = 0; u < kW4WideUnroll; ++u) {
      float c = rows.coef(min(t + u, re - 1), j[u]) * T::to_f32(static_cast<uint16_t>(s[u]));
      c = (t + u < re) ? c : 0.f;
      csum += c;
      const float cs = c * kW4CodeScale;
#pragma unroll
      for (int m = 0; m < 4; ++m) fma_codes8(v[u][m], cs, acc + m * 8);
    }
  }
#pragma unroll
  for (int k = 0; k < kW4WideAcc; ++k) acc[k] = fmaf(-8.0f, csum, acc[k]);
}

template <typename T, int RW, bool INDEXED>
__global__ __launch_bounds__(RW * 64, 2) void gemv_rows_w4_wide_kernel(W4Args w) {   // two workgroups per CU
  __shared__ GemvShared<RW, kW4WideAcc> sh;
  // a short list: this kernel's reduction buffers already take 57 KB of LDS per workgroup
  __shared__ int lst_idx[INDEXED ? kW4WideList : 1];
  __shared__ float lst_val[INDEXED ? kW4WideList : 1];
  const GemvArgs& a = w.g;
  const int lane = threadIdx.x & 63;
  const int rw = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
  const int b = blockIdx.y;
  const int g = blockIdx.x;
  const int K = a.K;

  GlobalRows<T, INDEXED> rows;
  rows.idx = INDEXED ? a.idx + static_cast<size_t>(b) * K : nullptr;
  rows.h = a.h + static_cast<size_t>(b) * a.d_in;
  rows.coef_scale = a.coef_scale;
  const Epilogue ep{a.y, a.rms_src, a.rms_eps, a.residual, a.y_pre, a.d_in, a.d_out, 0, nullptr};
  const int row_dwords = a.d_out / 8;

  const Segment sg = segment_of(g, a.wps, a.chunk, K);
  const bool staged = INDEXED && stage_row_list<RW * 64, kW4WideList>(rows, sg.t0, sg.t1 - sg.t0, lst_idx, lst_val);
  const int col = sg.s * kW4WideCols + lane * kW4WideAcc;
  float acc[kW4WideAcc];
#pragma unroll
  for (int k = 0; k < kW4WideAcc; ++k) acc[k] = 0.f;
  int ra, re;
  wave_run<RW>(sg.t0, sg.t1, rw, ra, re);
  if (col < a.d_out) {
    if (staged) {
      LdsRows lr;
      lr.idx = lst_idx;
      lr.val = lst_val;
      lr.base = sg.t0;
      stream_rows_w4_wide<T>(w.Wq + col / 8, row_dwords, w.scales + col / kW4Group, w.ng, lr, ra, re, acc);
    } else {
      stream_rows_w4_wide<T>(w.Wq + col / 8, row_dwords, w.scales + col / kW4Group, w.ng, rows, ra, re, acc);
    }
  }
  reduce_and_finish<T, RW, kW4WideAcc>(acc, sg.s, b, g, a.G, a.wps, a.partial, a.counters, a.nstrips, ep, sh, lane, rw);
}

template <typename T, int RW, bool INDEXED>
__global__ __launch_bounds__(RW * 64) void gemv_rows_w4_kernel(W4Args w) {
  __shared__ GemvShared<RW> sh;
  __shared__ int lst_idx[INDEXED ? kRowListMax : 1];
  __shared__ float lst_val[INDEXED ? kRowListMax : 1];
  const GemvArgs& a = w.g;
  const int lane = threadIdx.x & 63;
  const int rw = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
  const int b = blockIdx.y;
  const int g = blockIdx.x;
  const int K = a.K;

  GlobalRows<T, INDEXED> rows;
  rows.idx = INDEXED ? a.idx + static_cast<size_t>(b) * K : nullptr;
  rows.h = a.h + static_cast<size_t>(b) * a.d_in;
  rows.coef_scale = a.coef_scale;
  const Epilogue ep{a.y, a.rms_src, a.rms_eps, a.residual, a.y_pre, a.d_in, a.d_out, 0, nullptr};
  const int row_dwords = a.d_out / 8;

  const Segment sg = segment_of(g, a.wps, a.chunk, K);
  const bool staged = INDEXED && stage_row_list<RW * 64>(rows, sg.t0, sg.t1 - sg.t0, lst_idx, lst_val);
  const int col = sg.s * kStripCols + lane * 8;
  float acc[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) acc[k] = 0.f;
  int ra, re;
  wave_run<RW>(sg.t0, sg.t1, rw, ra, re);
  if (col < a.d_out) {
    if (staged) {
      LdsRows lr;
      lr.idx = lst_idx;
      lr.val = lst_val;
      lr.base = sg.t0;
      stream_rows_w4<T>(w.Wq + col / 8, row_dwords, w.scales + col / kW4Group, w.ng, lr, ra, re, acc);
    } else {
      stream_rows_w4<T>(w.Wq + col / 8, row_dwords, w.scales + col / kW4Group, w.ng, rows, ra, re, acc);
    }
  }
  reduce_and_finish<T, RW>(acc, sg.s, b, g, a.G, a.wps, a.partial, a.counters, a.nstrips, ep, sh, lane, rw);
}

// Round-to-nearest quantiser: one wave per row and 512 columns, a lane holds 8 columns, 16 lanes
// share a group.  s = max|w| / 7 rounded to 16 bits, q = clip(rint(w / s), -8, 7) + 8.
template <typename T>
__global__ __launch_bounds__(64) void quantize_w4_kernel(const uint16_t* __restrict__ W, int d_out, int ng,
                                                         uint32_t* __restrict__ Wq, uint16_t* __restrict__ scales) {
  const int lane = threadIdx.x;
  const int row = blockIdx.y;
  const int col = blockIdx.x * kStripCols + lane * 8;
  float w[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) w[k] = 0.f;
  if (col < d_out) unpack8<T>(*reinterpret_cast<const uint4*>(W + static_cast<size_t>(row) * d_out + col), w);
  float m = 0.f;
#pragma unroll
  for (int k = 0; k < 8; ++k) m = fmaxf(m, fabsf(w[k]));
#pragma unroll
  for (int o = 1; o < 16; o <<= 1) m = fmaxf(m, __shfl_xor(m, o, kWave));
  const uint16_t sb = T::from_f32(m / 7.0f);
  const float s = T::to_f32(sb);
  uint32_t packed = 0;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    float q = 0.f;
    if (s > 0.f) q = fminf(fmaxf(rintf(w[k] / s), -8.f), 7.f);
    packed |= static_cast<uint32_t>(static_cast<int>(q) + 8) << (4 * k);
  }
  if (col < d_out) {
    Wq[static_cast<size_t>(row) * (d_out / 8) + col / 8] = packed;
    if ((lane & 15) == 0) scales[static_cast<size_t>(row) * ng + col / kW4Group] = sb;
  }
}

template <typename T>
hipError_t launch_w4_t(const W4Args& w, hipStream_t st) {
  constexpr int RW = 8;
  dim3 grid(w.g.G, w.g.B), block(RW * 64);
  if (w4_strip_cols(w.g.d_out) == kW4WideCols) {
    if (w.g.idx)
      hipLaunchKernelGGL((gemv_rows_w4_wide_kernel<T, RW, true>), grid, block, 0, st, w);
    else
      hipLaunchKernelGGL((gemv_rows_w4_wide_kernel<T, RW, false>), grid, block, 0, st, w);
    return hipGetLastError();
  }
  if (w.g.idx)
    hipLaunchKernelGGL((gemv_rows_w4_kernel<T, RW, true>), grid, block, 0, st, w);
  else
    hipLaunchKernelGGL((gemv_rows_w4_kernel<T, RW, false>), grid, block, 0, st, w);
  return hipGetLastError();
}

}  // namespace

int w4_strip_cols(int d_out) {
  // A strip's finisher reads one partial per contributing workgroup, and a wide partial is 8 KiB: with
  // few strips (narrow outputs) that read-back outweighs the cheaper row loop (measured: 4096 columns
  // 30 vs 14 us, 22016 columns 27 vs 23 us, 57344 columns 54 vs 73 us).
  return (d_out % 32 == 0 && d_out >= tuning().w4_wide_min_cols) ? kW4WideCols : kStripCols;
}

hipError_t launch_quantize_w4(const uint16_t* W, int d_in, int d_out, uint32_t* Wq, uint16_t* scales, bool bf16,
                              hipStream_t s) {
  const int ng = (d_out + kW4Group - 1) / kW4Group;
  dim3 grid((d_out + kStripCols - 1) / kStripCols, d_in), block(64);
  if (bf16)
    hipLaunchKernelGGL(quantize_w4_kernel<BF16>, grid, block, 0, s, W, d_out, ng, Wq, scales);
  else
    hipLaunchKernelGGL(quantize_w4_kernel<F16>, grid, block, 0, s, W, d_out, ng, Wq, scales);
  return hipGetLastError();
}

hipError_t launch_gemv_w4(const W4Args& w, bool bf16, hipStream_t s) {
  return bf16 ? launch_w4_t<BF16>(w, s) : launch_w4_t<F16>(w, s);
}

}  // namespace larosa
