// Column-sparse projection with the Top-K sparsifier fused into its prologue (Sec. 4.4 point 2
// of the paper: selection and mat-vec in one kernel), for gfx950.
//
// Every workgroup rebuilds the block's input vector from its producer (a plain vector, the
// value heads of q|k|v broadcast to their query heads, SiLU(gate)*up, or the RMS-normed residual
// stream), runs the exact radix select on it (topk_core.hpp) and keeps, in LDS, only the (row,
// coefficient) pairs of the ranks it will stream.  The vector is at most 64 KiB and comes from
// L2, so the redundant selection costs about a microsecond per workgroup and removes three
// dependent kernels (copy/activation, Top-K, and the index/value gathers of the mat-vec) per
// projection.  Workgroup 0 also writes the vector and the index list for callers that ask.
#include "gemv_core.hpp"
#include "topk_core.hpp"

namespace larosa {

namespace {

constexpr int kFusedRW = 8;
constexpr int kFusedThreads = kFusedRW * 64;

template <typename T, int NV>   // NV 16-byte groups (8 elements each) per lane
__global__ __launch_bounds__(kFusedThreads) void fused_topk_gemv_kernel(FusedArgs a) {
  constexpr int E = NV * 8;
  __shared__ TopkShared<kFusedRW> tk;
  __shared__ GemvShared<kFusedRW> sh;
  __shared__ int lst_idx[kFusedChunkMax];
  __shared__ float lst_val[kFusedChunkMax];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int rw = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int b = blockIdx.y;
  const int g = blockIdx.x;
  const int d_in = a.g.d_in;
  const int K = a.g.K;
  const int base = tid * E;
  const int nvalid = max(0, min(E, d_in - base));

  // ---- the block's input vector, this lane's E elements as stored 16-bit values
  uint16_t raw[E];
#pragma unroll
  for (int q = 0; q < NV; ++q) {
    const int i = base + q * 8;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (i < d_in) {
      if (a.src_mode == kSrcGqa) {
        // context-length-1 attention: query head i/head_dim outputs the value head of its group
        const int head = i / a.head_dim;
        const int src = (head / a.group) * a.head_dim + (i - head * a.head_dim);
        v = *reinterpret_cast<const uint4*>(a.src + static_cast<size_t>(b) * (a.d_q + 2 * a.d_kv) + a.d_q + a.d_kv + src);
      } else if (a.src_mode == kSrcSilu) {
        const uint16_t* row = a.src + static_cast<size_t>(b) * 2 * d_in;
        float gt[8], up[8], o[8];
        unpack8<T>(*reinterpret_cast<const uint4*>(row + i), gt);
        unpack8<T>(*reinterpret_cast<const uint4*>(row + d_in + i), up);
#pragma unroll
        for (int k = 0; k < 8; ++k) o[k] = (gt[k] / (1.0f + expf(-gt[k]))) * up[k];
        v = pack8<T>(o);
      } else {
        v = *reinterpret_cast<const uint4*>(a.src + static_cast<size_t>(b) * d_in + i);
      }
    }
    raw[q * 8 + 0] = static_cast<uint16_t>(v.x & 0xFFFFu); raw[q * 8 + 1] = static_cast<uint16_t>(v.x >> 16);
    raw[q * 8 + 2] = static_cast<uint16_t>(v.y & 0xFFFFu); raw[q * 8 + 3] = static_cast<uint16_t>(v.y >> 16);
    raw[q * 8 + 4] = static_cast<uint16_t>(v.z & 0xFFFFu); raw[q * 8 + 5] = static_cast<uint16_t>(v.z >> 16);
    raw[q * 8 + 6] = static_cast<uint16_t>(v.w & 0xFFFFu); raw[q * 8 + 7] = static_cast<uint16_t>(v.w >> 16);
  }
  if (a.src_mode == kSrcNorm) {
    // h = R(x * rsqrt(mean(x^2) + eps) * scale)
    float ss = 0.f;
#pragma unroll
    for (int q = 0; q < E; ++q) {
      const float xv = (q < nvalid) ? T::to_f32(raw[q]) : 0.f;
      ss = fmaf(xv, xv, ss);
    }
    ss = wave_sum(ss);
    if (lane == 0) sh.blockred[rw] = ss;
    __syncthreads();
    float tot = 0.f;
    for (int w2 = 0; w2 < kFusedRW; ++w2) tot += sh.blockred[w2];
    const float rinv = 1.0f / sqrtf(tot / static_cast<float>(d_in) + a.norm_eps);
#pragma unroll
    for (int q = 0; q < E; ++q) {
      if (q < nvalid) {
        float xv = T::to_f32(raw[q]) * rinv;
        if (a.norm_scale) xv *= T::to_f32(a.norm_scale[base + q]);
        raw[q] = T::from_f32(xv);
      }
    }
    __syncthreads();
  }
  if (a.h_out && g == 0) {
#pragma unroll
    for (int q = 0; q < NV; ++q) {
      const int i = base + q * 8;
      if (i < d_in) {
        uint4 v;
        v.x = raw[q * 8 + 0] | (static_cast<uint32_t>(raw[q * 8 + 1]) << 16);
        v.y = raw[q * 8 + 2] | (static_cast<uint32_t>(raw[q * 8 + 3]) << 16);
        v.z = raw[q * 8 + 4] | (static_cast<uint32_t>(raw[q * 8 + 5]) << 16);
        v.w = raw[q * 8 + 6] | (static_cast<uint32_t>(raw[q * 8 + 7]) << 16);
        *reinterpret_cast<uint4*>(a.h_out + static_cast<size_t>(b) * d_in + i) = v;
      }
    }
  }

  // ---- Top-K select; keep the (row, coefficient) pairs of this workgroup's ranks in LDS
  const TopkLane st = block_select<kFusedRW, E>(raw, nvalid, K, tk);
  const int f0 = g * a.g.chunk;
  const int f1 = min(f0 + a.g.chunk, a.g.nstrips * K);
  const int sA = f0 / K;
  const int tA0 = f0 - sA * K;
  const int nA = min(K - tA0, f1 - f0);   // ranks [tA0, tA0+nA) of strip sA
  const int nB = (f1 - f0) - nA;          // ranks [0, nB) of strip sA+1; nB <= tA0, so the two never overlap
  int32_t* idx_out = (a.idx_out && g == 0) ? a.idx_out + static_cast<size_t>(b) * K : nullptr;
  for_each_kept<E>(raw, nvalid, st, [&](int q, unsigned upos) {
    const int pos = static_cast<int>(upos);
    if (pos >= K) return;                 // never taken; keeps a stray rank out of the lists
    if (idx_out) idx_out[pos] = base + q;
    int e = -1;
    if (pos >= tA0 && pos < tA0 + nA) e = pos - tA0;
    else if (pos < nB) e = nA + pos;
    if (e >= 0) {
      lst_idx[e] = base + q;
      lst_val[e] = T::to_f32(raw[q]);
    }
  });
  __syncthreads();

  // ---- stream the kept rows of the (at most two) segments
  const Epilogue ep{a.g.y, a.g.rms_src, a.g.rms_eps, a.g.residual, a.g.y_pre, d_in, a.g.d_out};
#pragma unroll 1
  for (int seg_no = 0; seg_no < 2; ++seg_no) {
    const int n = seg_no == 0 ? nA : nB;
    if (n <= 0) break;                    // uniform over the workgroup
    Segment sg;
    sg.s = sA + seg_no;
    sg.t0 = seg_no == 0 ? tA0 : 0;
    sg.t1 = sg.t0 + n;
    LdsRows rows;
    rows.idx = lst_idx + (seg_no == 0 ? 0 : nA);
    rows.val = lst_val + (seg_no == 0 ? 0 : nA);
    rows.base = sg.t0;
    const int col = sg.s * kStripCols + lane * 8;
    float acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = 0.f;
    const int per = (n + kFusedRW - 1) / kFusedRW;
    const int ra = sg.t0 + rw * per;
    const int re = min(sg.t1, ra + per);
    if (col < a.g.d_out) stream_rows<T>(a.g.W + col, a.g.d_out, rows, ra, re, acc);
    reduce_and_finish<T, kFusedRW>(acc, sg, seg_no, b, g, a.g.G, K, a.g.chunk, a.g.nstrips, a.g.partial,
                                   a.g.counters, ep, sh, lane, rw);
  }
}

template <typename T>
hipError_t launch_nv(const FusedArgs& a, hipStream_t st) {
  dim3 grid(a.g.G, a.g.B), block(kFusedThreads);
  const int nv = (a.g.d_in + kFusedThreads * 8 - 1) / (kFusedThreads * 8);
  if (nv <= 1) hipLaunchKernelGGL((fused_topk_gemv_kernel<T, 1>), grid, block, 0, st, a);
  else if (nv <= 2) hipLaunchKernelGGL((fused_topk_gemv_kernel<T, 2>), grid, block, 0, st, a);
  else if (nv <= 3) hipLaunchKernelGGL((fused_topk_gemv_kernel<T, 3>), grid, block, 0, st, a);
  else if (nv <= 4) hipLaunchKernelGGL((fused_topk_gemv_kernel<T, 4>), grid, block, 0, st, a);
  else if (nv <= 6) hipLaunchKernelGGL((fused_topk_gemv_kernel<T, 6>), grid, block, 0, st, a);
  else if (nv <= 8) hipLaunchKernelGGL((fused_topk_gemv_kernel<T, 8>), grid, block, 0, st, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace

GemvPlan plan_fused(int d_out, int K) {
  GemvPlan p = plan_gemv(d_out, K);
  if (p.chunk > kFusedChunkMax) {       // the workgroup's rank list must fit its LDS arrays
    const long T = static_cast<long>(p.nstrips) * K;
    p.chunk = kFusedChunkMax;
    p.G = static_cast<int>((T + p.chunk - 1) / p.chunk);
    p.partial_floats = static_cast<size_t>(p.G) * 2 * kStripCols;
  }
  return p;
}

hipError_t launch_fused(const FusedArgs& a, bool bf16, hipStream_t s) {
  return bf16 ? launch_nv<BF16>(a, s) : launch_nv<F16>(a, s);
}

}  // namespace larosa
