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

// This launch's share of the words it has to clear for a later launch (workgroup g of a.g.G).
template <int NT>
__device__ __forceinline__ void clear_words(const FusedArgs& a, int g) {
  if (a.zero_ptr) {
    for (int i = g * NT + static_cast<int>(threadIdx.x); i < a.zero_words; i += a.g.G * NT) a.zero_ptr[i] = 0u;
  }
}

// The block's input vector, four elements at a time: element group i / 4 of token b.
__device__ __forceinline__ uint2 load_source4(const FusedArgs& a, int b, int i) {
  if (a.src_mode == kSrcGqa) {
    // context-length-1 attention: query head i/head_dim outputs the value head of its group
    const int head = i / a.head_dim;
    const int src = (head / a.group) * a.head_dim + (i - head * a.head_dim);
    return *reinterpret_cast<const uint2*>(a.src + static_cast<size_t>(b) * (a.d_q + 2 * a.d_kv) + a.d_q + a.d_kv + src);
  }
  return *reinterpret_cast<const uint2*>(a.src + static_cast<size_t>(b) * a.g.d_in + i);
}

// Projection whose input vector arrives with its key histograms (FusedArgs::hist_in): the threshold
// comes from two small reads by wave 0; every workgroup then only classifies the vector's elements
// against it, ranks them and keeps its own ranks' rows.
//
// The vector sits in LDS in its natural order (one instantiation serves every width up to kHintMaxWidth),
// and lane t owns the groups of four elements t, t + NT, t + 2 NT, ...: "slab" q4 is the NT * 4
// consecutive elements whose groups the lanes hold at step q4.  A kept element's rank is the number of
// kept elements in earlier slabs, plus those of earlier waves in its slab, plus those of earlier lanes
// in its wave (a wave-level prefix sum per slab), plus those before it in its group.  A workgroup's
// contiguous rank range therefore falls on many consecutive lanes, a few elements each: building the
// row list is parallel work, not a long walk by a few lanes.
constexpr int kHintSlabs = kHintMaxWidth / (8 * 64 * 4);   // 16 slabs of 2048 elements

struct HintShared {
  uint2 vec[kHintMaxWidth / 4];          // group i / 4 of the vector
  unsigned tot[kHintSlabs * 8];          // per (slab, wave): kept-by-magnitude count | threshold ties << 16
  unsigned T, r;
};

// The rows of a workgroup's ranks as indices in LDS, their coefficients read from the vector in LDS.
template <typename T>
struct LdsRowsOfVector {
  const int* idx;
  const uint16_t* vec;
  int base;                  // rank of entry 0
  __device__ __forceinline__ void batch(int t, int re, int lane, int (&j)[kUnroll], float (&c)[kUnroll]) const {
    const int u0 = lane & (kUnroll - 1);
    const int myj = idx[min(t + u0, re - 1) - base];
    const float myc = (t + u0 < re) ? T::to_f32(vec[myj]) : 0.f;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      j[u] = __builtin_amdgcn_readlane(myj, u);
      c[u] = __uint_as_float(static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(__float_as_uint(myc)), u)));
    }
  }
};

template <typename T, int NS>   // NS slabs (2048 elements each) cover the vector
__global__ __launch_bounds__(512) void fused_hinted_gemv_kernel(FusedArgs a) {
  constexpr int RW = 8, NT = RW * 64;
  __shared__ HintShared hs;
  __shared__ GemvShared<RW> sh;
  __shared__ int lst_idx[kFusedChunkMax];

  LAROSA_STAMP(0);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int rw = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int b = blockIdx.y;
  const int g = blockIdx.x;
  clear_words<NT>(a, g);
  const int d_in = a.g.d_in;
  const int K = a.g.K;

  // ---- wave 0 reads the threshold off the histograms (two dependent reads, the first issued before
  // anything else); every lane's groups of the vector are loaded at once, kept in registers for the
  // classification and copied to LDS for the row loop (padding of the last slab: zeros)
  const unsigned* hist = a.hist_in + static_cast<size_t>(b) * kHistWords;
  uint4 coarse = make_uint4(0u, 0u, 0u, 0u);
  if (rw == 0) coarse = *hist_coarse_ptr(hist, lane);
  uint2 vq[NS];
#pragma unroll
  for (int q4 = 0; q4 < NS; ++q4) {
    vq[q4] = make_uint2(0u, 0u);
    const int i = (q4 * NT + tid) * 4;
    if (i < d_in) vq[q4] = load_source4(a, b, i);
  }
  int bin1 = 0;
  unsigned above1 = 0;
  uint2 fine = make_uint2(0u, 0u);
  if (rw == 0) {
    hist_coarse_step(coarse, K, lane, bin1, above1);
    fine = *hist_fine_ptr(hist, bin1, lane);
  }
#pragma unroll
  for (int q4 = 0; q4 < NS; ++q4) {
    {
      hs.vec[q4 * NT + tid] = vq[q4];
      const int i = (q4 * NT + tid) * 4;
      if (a.h_out && g == 0 && i < d_in) *reinterpret_cast<uint2*>(a.h_out + static_cast<size_t>(b) * d_in + i) = vq[q4];
    }
  }
  if (rw == 0) {
    unsigned Tk, r;
    hist_fine_step(fine, K, bin1, above1, lane, Tk, r);
    if (lane == 0) {
      hs.T = Tk;
      hs.r = r;
    }
  }
  __syncthreads();
  LAROSA_STAMP(1);
  const unsigned Tk = hs.T, r = hs.r;

  // ---- classify: per slab a 4-bit mask of keys > T and of keys == T, then the wave-level prefix of their counts
  unsigned cls[NS];      // gt mask | eq mask << 4, later also the exclusive wave prefix: gt << 8 | eq << 16
  unsigned cnt[NS];
#pragma unroll
  for (int q4 = 0; q4 < NS; ++q4) {
    const uint2 v = vq[q4];
    const unsigned k0 = v.x & 0x7FFFu, k1 = (v.x >> 16) & 0x7FFFu, k2 = v.y & 0x7FFFu, k3 = (v.y >> 16) & 0x7FFFu;
    const unsigned gt = (k0 > Tk ? 1u : 0u) | (k1 > Tk ? 2u : 0u) | (k2 > Tk ? 4u : 0u) | (k3 > Tk ? 8u : 0u);
    const unsigned eq = (k0 == Tk ? 1u : 0u) | (k1 == Tk ? 2u : 0u) | (k2 == Tk ? 4u : 0u) | (k3 == Tk ? 8u : 0u);
    cls[q4] = gt | (eq << 4);
    cnt[q4] = static_cast<unsigned>(__popc(gt)) | (static_cast<unsigned>(__popc(eq)) << 16);   // a wave: <= 256 each
  }
#pragma unroll
  for (int q4 = 0; q4 < NS; ++q4) {
    {
      const unsigned incl = wave_scan_inclusive(cnt[q4], lane);
      if (lane == 63) hs.tot[q4 * RW + rw] = incl;
      const unsigned excl = incl - cnt[q4];
      cls[q4] |= ((excl & 0xFFu) << 8) | ((excl >> 16) << 16);   // below 256: 8 bits each
    }
  }
  __syncthreads();
  // every wave: exclusive prefix of the (slab, wave) totals in that order; entry e = slab * 8 + wave sits in
  // lane e / 2, half e % 2 (at most 128 entries)
  unsigned pre_gt[2], pre_eq[2], tot2[2] = {0u, 0u};
  {
    if (2 * lane < NS * RW) {
      const uint2 tt = *reinterpret_cast<const uint2*>(&hs.tot[2 * lane]);
      tot2[0] = tt.x;
      tot2[1] = tt.y;
    }
    const unsigned g0 = tot2[0] & 0xFFFFu, g1 = tot2[1] & 0xFFFFu, e0 = tot2[0] >> 16, e1 = tot2[1] >> 16;
    const unsigned sg_ = wave_scan_inclusive(g0 + g1, lane) - (g0 + g1);
    const unsigned se_ = wave_scan_inclusive(e0 + e1, lane) - (e0 + e1);
    pre_gt[0] = sg_; pre_gt[1] = sg_ + g0;
    pre_eq[0] = se_; pre_eq[1] = se_ + e0;
  }
  LAROSA_STAMP(2);

  // ---- this workgroup's ranks: row indices into LDS; workgroup 0 also writes the whole index list.
  // A wave's share of a slab holds a contiguous run of ranks: waves whose run misses the workgroup's
  // range skip the slab (all but one or two of the wave-slab pairs).
  const Segment sg = segment_of(g, a.g.wps, a.g.chunk, K);
  const int n = sg.t1 - sg.t0;
  int32_t* idx_out = (a.idx_out && g == 0) ? a.idx_out + static_cast<size_t>(b) * K : nullptr;
#pragma unroll
  for (int q4 = 0; q4 < NS; ++q4) {
    {
      const int ent = q4 * RW + rw;
      // the kept elements before this wave's share of the slab, from the lane that holds the entry
      const unsigned bg = static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>((ent & 1) ? pre_gt[1] : pre_gt[0]), ent >> 1));
      const unsigned be = static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>((ent & 1) ? pre_eq[1] : pre_eq[0]), ent >> 1));
      const unsigned tw = static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>((ent & 1) ? tot2[1] : tot2[0]), ent >> 1));
      const int first = static_cast<int>(bg + min(be, r));                                     // rank of the wave's first kept element
      const int end = static_cast<int>(bg + (tw & 0xFFFFu) + min(be + (tw >> 16), r));         // one past its last
      if (idx_out || (first < sg.t1 && end > sg.t0)) {   // uniform over the wave
        const unsigned c = cls[q4];
        const unsigned gt = c & 0xFu, eq = (c >> 4) & 0xFu;
        unsigned gt_before = bg + ((c >> 8) & 0xFFu), eq_before = be + (c >> 16);
        const int i0 = (q4 * NT + tid) * 4;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bool is_gt = (gt >> j) & 1u, is_eq = (eq >> j) & 1u;
          const bool kept = is_gt || (is_eq && eq_before < r);       // ties: the first r in index order
          const int pos = static_cast<int>(gt_before + min(eq_before, r));
          if (kept) {
            if (idx_out) idx_out[pos] = i0 + j;
            const int e = pos - sg.t0;
            if (static_cast<unsigned>(e) < static_cast<unsigned>(n)) lst_idx[e] = i0 + j;
          }
          gt_before += is_gt ? 1u : 0u;
          eq_before += is_eq ? 1u : 0u;
        }
      }
    }
  }
  LAROSA_STAMP(3);
  __syncthreads();
  LAROSA_STAMP(4);

  // ---- stream the kept rows of this workgroup's ranks
  const Epilogue ep{a.g.y, a.g.rms_src, a.g.rms_eps, a.g.residual, a.g.y_pre, d_in, a.g.d_out, a.pair_cols, a.pair_out,
                    a.hist_out, a.hist_col0, a.hist_col1, a.hist_weight};
  LdsRowsOfVector<T> rows;
  rows.idx = lst_idx;
  rows.vec = reinterpret_cast<const uint16_t*>(hs.vec);
  rows.base = sg.t0;
  bool col_valid;
  const int col = strip_lane_col(sg.s, lane, a.g.d_out, a.pair_cols, col_valid);
  float acc[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) acc[k] = 0.f;
  int ra, re;
  wave_run<RW>(sg.t0, sg.t1, rw, ra, re);
  stream_rows<T>(a.g.W + col, a.g.d_out, rows, ra, re, acc, col_valid);
  LAROSA_STAMP(5);
  reduce_and_finish<T, RW>(acc, sg.s, b, g, a.g.G, a.g.wps, a.g.partial, a.g.counters, a.g.nstrips, ep, sh, lane, rw);
  LAROSA_STAMP(6);
}

template <typename T, int RW, int NV>   // RW row-waves; NV 8-byte groups (4 elements each) per lane
// at most 128 vector registers per lane: two 8-wave workgroups (or one of 16 waves) stay resident per compute unit
__global__ __launch_bounds__(RW * 64) __attribute__((amdgpu_waves_per_eu(4, 4))) void fused_topk_gemv_kernel(FusedArgs a) {
  constexpr int E = NV * 4;
  constexpr int kFusedRW = RW;
  __shared__ TopkShared<RW> tk;
  __shared__ GemvShared<RW> sh;
  __shared__ int lst_idx[kFusedChunkMax];
  __shared__ float lst_val[kFusedChunkMax];

  LAROSA_STAMP(0);
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
  clear_words<RW * 64>(a, g);
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
    const uint2 v = i < d_in ? load_source4(a, b, i) : make_uint2(0u, 0u);
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
  LAROSA_STAMP(1);
  const auto st = block_select<kFusedRW, E>(raw, K, tk);
  LAROSA_STAMP(2);
  const Segment sg = segment_of(g, a.g.wps, a.g.chunk, K);
  const int n = sg.t1 - sg.t0;            // <= the list capacity by the plan
  int32_t* idx_out = (a.idx_out && g == 0) ? a.idx_out + static_cast<size_t>(b) * K : nullptr;
  // only lanes whose ranks meet this workgroup's rank range (a few percent) walk their elements
  const int p0 = static_cast<int>(st.first_rank()), p1 = static_cast<int>(st.end_rank());
  if (idx_out || (p0 < sg.t1 && p1 > sg.t0)) {
    for_each_kept<E>(st, [&](int q, unsigned upos, bool kept) {
      const int pos = static_cast<int>(upos);
      if (idx_out && kept) idx_out[pos] = base + q;          // idx_out is uniform over the workgroup
      const int e = pos - sg.t0;
      if (kept && static_cast<unsigned>(e) < static_cast<unsigned>(n)) {
        lst_idx[e] = base + q;
        lst_val[e] = T::to_f32(raw[q]);
      }
    });
  }
  LAROSA_STAMP(3);
  __syncthreads();
  LAROSA_STAMP(4);

  // ---- stream the kept rows of this workgroup's ranks
  const Epilogue ep{a.g.y, a.g.rms_src, a.g.rms_eps, a.g.residual, a.g.y_pre, d_in, a.g.d_out, a.pair_cols, a.pair_out,
                    a.hist_out, a.hist_col0, a.hist_col1, a.hist_weight};
  LdsRows rows;
  rows.idx = lst_idx;
  rows.val = lst_val;
  rows.base = sg.t0;
  bool col_valid;
  const int col = strip_lane_col(sg.s, lane, a.g.d_out, a.pair_cols, col_valid);
  float acc[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) acc[k] = 0.f;
  int ra, re;
  wave_run<kFusedRW>(sg.t0, sg.t1, rw, ra, re);
  stream_rows<T>(a.g.W + col, a.g.d_out, rows, ra, re, acc, col_valid);
  LAROSA_STAMP(5);
  reduce_and_finish<T, kFusedRW>(acc, sg.s, b, g, a.g.G, a.g.wps, a.g.partial, a.g.counters, a.g.nstrips, ep, sh, lane,
                                 rw);
  LAROSA_STAMP(6);
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
  LAROSA_FUSED_CASE(12)
  LAROSA_FUSED_CASE(16)
#undef LAROSA_FUSED_CASE
  return hipErrorInvalidValue;
}

template <typename T>
hipError_t launch_hinted(const FusedArgs& a, hipStream_t st) {
  if (a.side_G > 0 || a.src_mode == kSrcNorm || a.g.d_in > kHintMaxWidth) return hipErrorInvalidValue;
  dim3 grid(a.g.G, a.g.B), block(8 * 64);
  const int ns = (a.g.d_in + 2047) / 2048;
  if (ns <= 2) hipLaunchKernelGGL((fused_hinted_gemv_kernel<T, 2>), grid, block, 0, st, a);
  else if (ns <= 4) hipLaunchKernelGGL((fused_hinted_gemv_kernel<T, 4>), grid, block, 0, st, a);
  else if (ns <= 6) hipLaunchKernelGGL((fused_hinted_gemv_kernel<T, 6>), grid, block, 0, st, a);
  else if (ns <= 8) hipLaunchKernelGGL((fused_hinted_gemv_kernel<T, 8>), grid, block, 0, st, a);
  else if (ns <= 12) hipLaunchKernelGGL((fused_hinted_gemv_kernel<T, 12>), grid, block, 0, st, a);
  else if (ns <= 14) hipLaunchKernelGGL((fused_hinted_gemv_kernel<T, 14>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((fused_hinted_gemv_kernel<T, 16>), grid, block, 0, st, a);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_rw(const FusedArgs& a, hipStream_t st) {
  if (a.hist_in) return launch_hinted<T>(a, st);
  return launch_nv<T, 8>(a, st);
}

}  // namespace

GemvPlan plan_fused(int d_out, int K, int g_hint, int pair_cols) {
  // paired strips: ceil(d_ff / 256) strips of 512 columns (256 gate + 256 up); plan_gemv only needs the count
  const int cols = pair_cols > 0 ? (pair_cols + 255) / 256 * kStripCols : d_out;
  GemvPlan p = plan_gemv(cols, K, g_hint, kStripCols, kFusedChunkMax);
  // at most 28 workgroups on a strip: with 8 strips (4096 outputs) 224 selecting workgroups measured 0.4 - 0.6 us
  // per layer better than 256 on the 7B and 8B shapes (down projection); wider outputs never get that many
  constexpr int kMaxPerStrip = 28;
  if (g_hint == 0 && tuning().g_target == 0 && p.wps > kMaxPerStrip)
    p = plan_gemv(cols, K, p.nstrips * kMaxPerStrip, kStripCols, kFusedChunkMax);
  return p;
}

hipError_t launch_fused(const FusedArgs& a, bool bf16, hipStream_t s) {
  return bf16 ? launch_rw<BF16>(a, s) : launch_rw<F16>(a, s);
}

}  // namespace larosa
