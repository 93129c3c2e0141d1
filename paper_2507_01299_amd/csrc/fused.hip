// Column-sparse projection with the Top-K sparsifier fused into its prologue (Sec. 4.4 point 2
// of the paper: selection and mat-vec in one kernel), for gfx950.
//
// Every workgroup rebuilds the block's input vector from its producer (a plain vector, the
// value heads of q|k|v broadcast to their query heads, or the RMS-normed residual stream; the
// SiLU(gate)*up vector is stored by the gate|up launch itself, see paired strips below), runs the exact radix select on it (topk_core.hpp) and keeps, in LDS, only the (row,
// coefficient) pairs of the ranks it will stream.  The vector is at most 64 KiB and comes from
// L2, so the redundant selection costs about a microsecond per workgroup and removes three
// dependent kernels (copy/activation, Top-K, and the index/value gathers of the mat-vec) per
// projection.  Workgroup 0 also writes the vector and the index list for callers that ask.
//
// A launch can carry a dense side job (FusedArgs::side): the residual adapter on the block's
// shortcut, x (Q_in^T Q_out), needs only the block's input, so its workgroups stream their rows
// while the projection's workgroups are still selecting, and the adapter leaves the layer's
// critical path.
#include "gemv_core.hpp"
#include "topk_core.hpp"

namespace larosa {

namespace {

template <typename T, int RW, int NV>   // RW row-waves; NV 8-byte groups (4 elements each) per lane
__global__ __launch_bounds__(RW * 64) void fused_topk_gemv_kernel(FusedArgs a) {
  constexpr int E = NV * 4;
  constexpr int kFusedRW = RW;
  __shared__ TopkShared<RW> tk;
  __shared__ GemvShared<RW> sh;
  __shared__ int lst_idx[kFusedChunkMax];
  __shared__ float lst_val[kFusedChunkMax];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int rw = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int b = blockIdx.y;
  int g = blockIdx.x;
  if (a.side_G > 0) {                     // uniform over the workgroup
    if (g < a.side_G) {
      static_assert(kFusedChunkMax >= kRowListMax, "the side job stages its coefficients in lst_val");
      gemv_rows_body<T, RW, false>(a.side, g, b, sh, nullptr, lst_val);
      return;
    }
    g -= a.side_G;
  }
  const int d_in = a.g.d_in;
  const int K = a.g.K;
  const int base = tid * E;
  const int nvalid = max(0, min(E, d_in - base));
  topk_clear<kFusedRW>(tk);               // made visible by the first barrier below, while the loads are in flight

  // ---- the block's input vector, this lane's E elements as stored 16-bit values
  uint16_t raw[E];
#pragma unroll
  for (int q = 0; q < NV; ++q) {
    const int i = base + q * 4;
    uint2 v = make_uint2(0u, 0u);
    if (i < d_in) {
      if (a.src_mode == kSrcGqa) {
        // context-length-1 attention: query head i/head_dim outputs the value head of its group
        const int head = i / a.head_dim;
        const int src = (head / a.group) * a.head_dim + (i - head * a.head_dim);
        v = *reinterpret_cast<const uint2*>(a.src + static_cast<size_t>(b) * (a.d_q + 2 * a.d_kv) + a.d_q + a.d_kv + src);
      } else {
        v = *reinterpret_cast<const uint2*>(a.src + static_cast<size_t>(b) * d_in + i);
      }
    }
    raw[q * 4 + 0] = static_cast<uint16_t>(v.x & 0xFFFFu); raw[q * 4 + 1] = static_cast<uint16_t>(v.x >> 16);
    raw[q * 4 + 2] = static_cast<uint16_t>(v.y & 0xFFFFu); raw[q * 4 + 3] = static_cast<uint16_t>(v.y >> 16);
  }
  if (a.src_mode == kSrcNorm) {
    // h = R(x * rsqrt(mean(x^2) + eps) * scale)
    // the lane's slice of the learned scale, fetched with x (loads at each use would each wait for memory)
    uint2 sc2[NV];
#pragma unroll
    for (int q = 0; q < NV; ++q) {
      const int i = base + q * 4;
      sc2[q] = (a.norm_scale && i < d_in) ? *reinterpret_cast<const uint2*>(a.norm_scale + i) : make_uint2(0u, 0u);
    }
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
      float xv = T::to_f32(raw[q]) * rinv;
      const uint32_t w = (q & 2) ? sc2[q >> 2].y : sc2[q >> 2].x;
      if (a.norm_scale) xv *= T::to_f32(static_cast<uint16_t>((q & 1) ? (w >> 16) : (w & 0xFFFFu)));
      raw[q] = (q < nvalid) ? T::from_f32(xv) : static_cast<uint16_t>(0);   // padding stays zero
    }
  } else {
    __syncthreads();
  }
  if (a.h_out && g == 0) {
#pragma unroll
    for (int q = 0; q < NV; ++q) {
      const int i = base + q * 4;
      if (i < d_in) {
        uint2 v;
        v.x = raw[q * 4 + 0] | (static_cast<uint32_t>(raw[q * 4 + 1]) << 16);
        v.y = raw[q * 4 + 2] | (static_cast<uint32_t>(raw[q * 4 + 3]) << 16);
        *reinterpret_cast<uint2*>(a.h_out + static_cast<size_t>(b) * d_in + i) = v;
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
  // only lanes whose ranks meet this workgroup's two rank ranges (a few percent) walk their elements
  const int p0 = static_cast<int>(st.first_rank()), p1 = static_cast<int>(st.end_rank());
  if (idx_out || (p0 < tA0 + nA && p1 > tA0) || p0 < nB) {
    for_each_kept<E>(raw, nvalid, st, [&](int q, unsigned upos, bool kept) {
      const int pos = static_cast<int>(upos);
      if (idx_out && kept) idx_out[pos] = base + q;          // idx_out is uniform over the workgroup
      // entry of the rank in this workgroup's list: segment A holds ranks [tA0, tA0 + nA), segment B
      // ranks [0, nB); e < nA + nB <= the list capacity by construction
      const int eA = pos - tA0;
      const bool inA = static_cast<unsigned>(eA) < static_cast<unsigned>(nA);
      const bool inB = pos < nB;
      const int e = inA ? eA : nA + pos;
      if (kept && (inA || inB)) {
        lst_idx[e] = base + q;
        lst_val[e] = T::to_f32(raw[q]);
      }
    });
  }
  __syncthreads();

  // ---- stream the kept rows of the (at most two) segments
  const Epilogue ep{a.g.y, a.g.rms_src, a.g.rms_eps, a.g.residual, a.g.y_pre, d_in, a.g.d_out, a.pair_cols, a.pair_out};
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
    bool col_valid;
    const int col = strip_lane_col(sg.s, lane, a.g.d_out, a.pair_cols, col_valid);
    float acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = 0.f;
    const int per = (n + kFusedRW - 1) / kFusedRW;
    const int ra = sg.t0 + rw * per;
    const int re = min(sg.t1, ra + per);
    if (col_valid) stream_rows<T>(a.g.W + col, a.g.d_out, rows, ra, re, acc);
    reduce_and_finish<T, kFusedRW>(acc, sg, seg_no, b, g, a.g.G, K, a.g.chunk, a.g.nstrips, a.g.partial,
                                   a.g.counters, ep, sh, lane, rw);
  }
}

template <typename T, int RW>
hipError_t launch_nv(const FusedArgs& a, hipStream_t st) {
  dim3 grid(a.g.G + a.side_G, a.g.B), block(RW * 64);
  const int nv = (a.g.d_in + RW * 64 * 4 - 1) / (RW * 64 * 4);
#define LAROSA_FUSED_CASE(N) \
  if (nv <= N) { hipLaunchKernelGGL((fused_topk_gemv_kernel<T, RW, N>), grid, block, 0, st, a); return hipGetLastError(); }
  LAROSA_FUSED_CASE(1)
  LAROSA_FUSED_CASE(2)
  LAROSA_FUSED_CASE(3)
  LAROSA_FUSED_CASE(4)
  LAROSA_FUSED_CASE(6)
  LAROSA_FUSED_CASE(8)
  if (RW == 8) {
    LAROSA_FUSED_CASE(12)
    LAROSA_FUSED_CASE(16)
  }
#undef LAROSA_FUSED_CASE
  return hipErrorInvalidValue;
}

template <typename T>
hipError_t launch_rw(const FusedArgs& a, hipStream_t st) {
  return fused_row_waves() == 16 ? launch_nv<T, 16>(a, st) : launch_nv<T, 8>(a, st);
}

}  // namespace

int fused_row_waves() { return tuning().fused_rw == 16 ? 16 : 8; }

GemvPlan plan_fused(int d_out, int K, int g_hint, int pair_cols) {
  // paired strips: ceil(d_ff / 256) strips of 512 columns (256 gate + 256 up); plan_gemv only needs the count
  GemvPlan p = plan_gemv(pair_cols > 0 ? (pair_cols + 255) / 256 * kStripCols : d_out, K, g_hint);
  if (fused_row_waves() == 16 && tuning().g_target == 0 && g_hint == 0 && p.G > 256) {
    // 1024-lane workgroups: one per compute unit, so the redundant prologue runs once per CU
    const long T = static_cast<long>(p.nstrips) * K;
    long G = 256 > p.nstrips ? 256 : p.nstrips;
    p.chunk = static_cast<int>((T + G - 1) / G);
    p.G = static_cast<int>((T + p.chunk - 1) / p.chunk);
    p.partial_floats = static_cast<size_t>(p.G) * 2 * kStripCols;
  }
  if (p.chunk > kFusedChunkMax) {       // the workgroup's rank list must fit its LDS arrays
    const long T = static_cast<long>(p.nstrips) * K;
    p.chunk = kFusedChunkMax;
    p.G = static_cast<int>((T + p.chunk - 1) / p.chunk);
    p.partial_floats = static_cast<size_t>(p.G) * 2 * kStripCols;
  }
  return p;
}

hipError_t launch_fused(const FusedArgs& a, bool bf16, hipStream_t s) {
  return bf16 ? launch_rw<BF16>(a, s) : launch_rw<F16>(a, s);
}

}  // namespace larosa
