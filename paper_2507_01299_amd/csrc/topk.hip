// Top-K sparsifier S_k of LaRoSA (Sec. 4.3, Eq. 8) for gfx950: per token, the K indices of
// largest magnitude, ties to the larger magnitude and then the lower index, ascending.
//
// The ordering key is the stored 16-bit pattern with the sign cleared (15 bits, unsigned), so
// the selection is pure integer work and identical for binary16 and bfloat16.  One workgroup
// of 1024 lanes handles one token.  Lane t owns the contiguous elements [t*E, (t+1)*E) and
// keeps their keys in registers for all three phases:
//   1. 256-bin histogram of the top 8 key bits (one LDS copy per wave to spread atomics),
//      suffix sums from the top locate the bin holding the K-th largest key;
//   2. 128-bin histogram of the low 7 bits inside that bin gives the threshold key T and
//      r = K - #{key > T}, the number of threshold ties to keep;
//   3. an index-ordered compaction (block prefix sums of the ">T" and "==T" counts) writes
//      every key > T and the first r keys == T, which yields ascending indices and the
//      lower-index tie rule with no sort.
#include "kernels.hpp"
#include "numeric.hpp"

namespace larosa {

namespace {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / 64;

// Find, over bins visited from the highest down, the first bin at which the running count
// reaches `need`.  Executed by wave 0; hist has NB bins; each lane covers NB/64 bins.
// Writes the bin and the count strictly above it.
template <int NB>
__device__ __forceinline__ void locate_bin(const unsigned* hist, unsigned need, int lane, int* out_bin,
                                           unsigned* out_above) {
  constexpr int PER = NB / 64;
  unsigned c[PER];
  unsigned local = 0;
#pragma unroll
  for (int q = 0; q < PER; ++q) {
    c[q] = hist[NB - 1 - (lane * PER + q)];   // position p = lane*PER+q counts from the top bin
    local += c[q];
  }
  const unsigned incl = wave_scan_inclusive(local, lane);
  unsigned run = incl - local;                // count in positions before this lane's first
#pragma unroll
  for (int q = 0; q < PER; ++q) {
    const unsigned before = run;
    run += c[q];
    if (before < need && run >= need) {
      *out_bin = NB - 1 - (lane * PER + q);
      *out_above = before;
    }
  }
}

template <int E>   // elements per lane, multiple of 4
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(const uint16_t* __restrict__ h, int d, int K,
                                                            int32_t* __restrict__ idx,
                                                            uint16_t* __restrict__ vals) {
  __shared__ unsigned hist_w[kTopkWaves][256];
  __shared__ unsigned hist[256];
  __shared__ unsigned wave_tot[kTopkWaves];
  __shared__ int s_bin;
  __shared__ unsigned s_above;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int b = blockIdx.x;
  const uint16_t* hb = h + static_cast<size_t>(b) * d;
  const int base = tid * E;

  // load this lane's elements (raw bits kept for vals)
  uint16_t raw[E];
#pragma unroll
  for (int q = 0; q < E / 4; ++q) {
    const int i = base + q * 4;
    uint2 v = make_uint2(0u, 0u);
    if (i < d) v = *reinterpret_cast<const uint2*>(hb + i);     // d % 4 == 0: all four valid or none
    raw[q * 4 + 0] = static_cast<uint16_t>(v.x & 0xFFFFu);
    raw[q * 4 + 1] = static_cast<uint16_t>(v.x >> 16);
    raw[q * 4 + 2] = static_cast<uint16_t>(v.y & 0xFFFFu);
    raw[q * 4 + 3] = static_cast<uint16_t>(v.y >> 16);
  }
  const int nvalid = max(0, min(E, d - base));

  // ---- phase 1: histogram of key >> 7
  for (int i = tid; i < kTopkWaves * 256; i += kTopkThreads) (&hist_w[0][0])[i] = 0u;
  __syncthreads();
#pragma unroll
  for (int q = 0; q < E; ++q)
    if (q < nvalid) atomicAdd(&hist_w[wave][(raw[q] & 0x7FFFu) >> 7], 1u);
  __syncthreads();
  if (tid < 256) {
    unsigned s = 0;
#pragma unroll
    for (int w = 0; w < kTopkWaves; ++w) s += hist_w[w][tid];
    hist[tid] = s;
  }
  __syncthreads();
  if (wave == 0) locate_bin<256>(hist, static_cast<unsigned>(K), lane, &s_bin, &s_above);
  __syncthreads();
  const int bin1 = s_bin;
  const unsigned above1 = s_above;
  __syncthreads();

  // ---- phase 2: histogram of key & 127 inside bin1
  for (int i = tid; i < kTopkWaves * 128; i += kTopkThreads) (&hist_w[0][0])[i] = 0u;
  __syncthreads();
#pragma unroll
  for (int q = 0; q < E; ++q) {
    const unsigned key = raw[q] & 0x7FFFu;
    if (q < nvalid && static_cast<int>(key >> 7) == bin1) atomicAdd(&(&hist_w[0][0])[wave * 128 + (key & 127u)], 1u);
  }
  __syncthreads();
  if (tid < 128) {
    unsigned s = 0;
#pragma unroll
    for (int w = 0; w < kTopkWaves; ++w) s += (&hist_w[0][0])[w * 128 + tid];
    hist[tid] = s;
  }
  __syncthreads();
  if (wave == 0) locate_bin<128>(hist, static_cast<unsigned>(K) - above1, lane, &s_bin, &s_above);
  __syncthreads();
  const unsigned T = (static_cast<unsigned>(bin1) << 7) | static_cast<unsigned>(s_bin);
  const unsigned r = static_cast<unsigned>(K) - (above1 + s_above);   // threshold ties to keep, >= 1

  // ---- phase 3: ordered compaction
  unsigned n_gt = 0, n_eq = 0;
#pragma unroll
  for (int q = 0; q < E; ++q) {
    const unsigned key = raw[q] & 0x7FFFu;
    if (q < nvalid) {
      n_gt += (key > T) ? 1u : 0u;
      n_eq += (key == T) ? 1u : 0u;
    }
  }
  const unsigned packed = n_gt | (n_eq << 16);          // each total <= 32768, no carry between halves
  const unsigned incl = wave_scan_inclusive(packed, lane);
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  unsigned prefix = incl - packed;
  for (int w = 0; w < wave; ++w) prefix += wave_tot[w];
  unsigned gt_before = prefix & 0xFFFFu;
  unsigned eq_before = prefix >> 16;
  int32_t* idxb = idx + static_cast<size_t>(b) * K;
  uint16_t* valb = vals ? vals + static_cast<size_t>(b) * K : nullptr;
#pragma unroll
  for (int q = 0; q < E; ++q) {
    if (q < nvalid) {
      const unsigned key = raw[q] & 0x7FFFu;
      const bool gt = key > T;
      const bool eq = key == T;
      if (gt || (eq && eq_before < r)) {
        const unsigned pos = gt_before + min(eq_before, r);
        if (pos < static_cast<unsigned>(K)) {   // always true; keeps a stray position inside the row
          idxb[pos] = base + q;
          if (valb) valb[pos] = raw[q];
        }
      }
      gt_before += gt ? 1u : 0u;
      eq_before += eq ? 1u : 0u;
    }
  }
}

}  // namespace

hipError_t launch_topk(const uint16_t* h, int B, int d, int K, int32_t* idx, uint16_t* vals, hipStream_t s) {
  dim3 grid(B), block(kTopkThreads);
  const int e = (d + kTopkThreads - 1) / kTopkThreads;
  if (e <= 4)
    hipLaunchKernelGGL(topk_kernel<4>, grid, block, 0, s, h, d, K, idx, vals);
  else if (e <= 8)
    hipLaunchKernelGGL(topk_kernel<8>, grid, block, 0, s, h, d, K, idx, vals);
  else if (e <= 16)
    hipLaunchKernelGGL(topk_kernel<16>, grid, block, 0, s, h, d, K, idx, vals);
  else if (e <= 24)
    hipLaunchKernelGGL(topk_kernel<24>, grid, block, 0, s, h, d, K, idx, vals);
  else if (e <= 32)
    hipLaunchKernelGGL(topk_kernel<32>, grid, block, 0, s, h, d, K, idx, vals);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace larosa
