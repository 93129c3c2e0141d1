// Row-streaming mat-vec for gfx950: the column-sparse projection of LaRoSA (Sec. 4.3 Eq. 10,
// Sec. 4.4) with indices read from memory and, with the identity row list, the dense rotation /
// adapter / baseline.
//
// The weight is input-channel-major, so a kept input channel is one contiguous run of d_out
// 16-bit values.  Work is the set of (column strip, kept row) pairs; every strip's kept rows are cut
// into equal runs over the same number of workgroups, so every workgroup moves the same number of
// bytes and hands over exactly one partial strip.  The shared pieces (row loop, reductions, epilogue)
// are in gemv_core.hpp.
#include "gemv_core.hpp"

namespace larosa {

namespace {

template <typename T, int RW, bool INDEXED>
__global__ __launch_bounds__(RW * 64) void gemv_rows_kernel(GemvArgs a) {
  __shared__ GemvShared<RW> sh;
  __shared__ int lst_idx[INDEXED ? kRowListMax : 1];
  __shared__ float lst_val[kRowListMax];
  gemv_rows_body<T, RW, INDEXED>(a, blockIdx.x, blockIdx.y, sh, lst_idx, lst_val);
}

template <typename T, int RW>
hipError_t launch_shape(const GemvArgs& a, hipStream_t st) {
  dim3 grid(a.G, a.B), block(RW * 64);
  if (a.idx)
    hipLaunchKernelGGL((gemv_rows_kernel<T, RW, true>), grid, block, 0, st, a);
  else
    hipLaunchKernelGGL((gemv_rows_kernel<T, RW, false>), grid, block, 0, st, a);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_variant(const GemvArgs& a, hipStream_t st) {
  switch (tuning().variant) {
    case 1: return launch_shape<T, 16>(a, st);
    case 2: return launch_shape<T, 4>(a, st);
    default: return launch_shape<T, 8>(a, st);
  }
}

}  // namespace

Tuning& tuning() {
  static Tuning t;
  return t;
}

GemvPlan plan_gemv(int d_out, int K, int g_hint, int strip_cols, int max_ranks) {
  GemvPlan p;
  p.strip_cols = strip_cols;
  p.nstrips = (d_out + strip_cols - 1) / strip_cols;
  const long T = static_cast<long>(p.nstrips) * K;
  // 256 compute units, one workgroup each (a second one per unit does not raise the row-streaming rate
  // and doubles the per-unit cost of everything the workgroups do redundantly); every workgroup works
  // on one strip, so the count is a multiple of the number of strips (rounded down: what is left idle
  // is a few compute units, not bandwidth)
  long G = g_hint > 0 ? g_hint : tuning().g_target > 0 ? tuning().g_target : 256;
  (void)T;
  long wps = G / p.nstrips;
  if (wps > K / tuning().min_rows) wps = K / tuning().min_rows;
  if (wps < 1) wps = 1;
  long per = (K + wps - 1) / wps;
  if (max_ranks > 0 && per > max_ranks) {
    // The workgroup's rank list must fit its LDS arrays, so a strip needs more workgroups than one per
    // compute unit allows.  Between one and two per unit some units carry twice the load of others: go to
    // (at most) two per unit instead (70B gate|up alone: 121 us with 336 workgroups).
    long need = (K + max_ranks - 1) / max_ranks;
    if (g_hint == 0 && tuning().g_target == 0 && 512 / p.nstrips > need) need = 512 / p.nstrips;
    per = (K + need - 1) / need;
  }
  p.chunk = static_cast<int>(per);
  p.wps = static_cast<int>((K + per - 1) / per);           // every workgroup of a strip has ranks
  p.G = p.nstrips * p.wps;
  p.partial_floats = static_cast<size_t>(p.G) * strip_cols;
  return p;
}

hipError_t launch_gemv(const GemvArgs& a, bool bf16, hipStream_t s) {
  return bf16 ? launch_variant<BF16>(a, s) : launch_variant<F16>(a, s);
}

}  // namespace larosa
