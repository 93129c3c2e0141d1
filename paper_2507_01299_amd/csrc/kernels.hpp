// Host-side launch interface of the gfx950 kernels (internal to liblarosa).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace larosa {

// Row-streaming mat-vec  y[b,:] = epilogue( sum_t c[b,t] * W[row(b,t), :] ).
// row(b,t) = idx[b*K + t] (indexed: the column-sparse projection) or t (dense: rotation,
// adapter, dense baseline).  c = h[b,row] (* coef_scale[row]).
struct GemvArgs {
  const uint16_t* W;          // [d_in, d_out] input-channel-major
  const uint16_t* h;          // [B, d_in]
  const int32_t* idx;         // [B, K] or nullptr (dense: K == d_in)
  uint16_t* y;                // [B, d_out]
  int d_in, d_out, K, B;
  // work split: row-strips (strip s, kept row t) are numbered f = s*K + t; workgroup g takes
  // [g*chunk, (g+1)*chunk).  chunk <= K, so a workgroup touches at most two strips.
  int chunk, G, nstrips;
  float* partial;             // [B][G][2][strip_cols] fp32 partial sums
  unsigned* counters;         // [B][nstrips] arrival counters (kCounterStride apart), zero on entry and on exit
  // epilogue
  const uint16_t* coef_scale; // [d_in] or nullptr: multiplies the coefficient (pre-norm scale)
  const uint16_t* rms_src;    // [B, d_in] or nullptr: result is multiplied by 1/sqrt(mean(rms_src^2)+eps)
  float rms_eps;
  const uint16_t* residual;   // [B, d_out] or nullptr: y = R(residual + R(acc))
  uint16_t* y_pre;            // [B, d_out] or nullptr: receives R(acc) when a residual is added
};

constexpr int kCounterStride = 64;   // in 32-bit words: one arrival counter per 256 bytes

struct GemvPlan {
  int strip_cols, nstrips, chunk, G;
  size_t partial_floats;      // per token
};

struct Tuning {
  int g_target = 512;         // target workgroups per launch (two resident per CU)
  int min_rows = 8;           // minimum row-strips per workgroup
  int variant = 0;            // kernel shape variant
};
Tuning& tuning();

GemvPlan plan_gemv(int d_out, int K);
int gemv_strip_cols();
hipError_t launch_gemv(const GemvArgs& a, bool bf16, hipStream_t s);

// Top-K select over stored 16-bit magnitudes, one workgroup per token.
hipError_t launch_topk(const uint16_t* h, int B, int d, int K, int32_t* idx, uint16_t* vals, hipStream_t s);

// h2[b,i] = v-part of qkv for the GQA group of query head i/head_dim (context-length-1 attention).
hipError_t launch_gqa_expand(const uint16_t* qkv, uint16_t* h2, int B, int d_q, int d_kv, int head_dim,
                             hipStream_t s);
// h4 = R(SiLU(gate) * up) with gu = [gate | up]
hipError_t launch_silu_mul(const uint16_t* gu, uint16_t* h4, int B, int d_ff, bool bf16, hipStream_t s);
// y = R(x * rsqrt(mean(x^2)+eps) * scale)
hipError_t launch_rmsnorm(const uint16_t* x, const uint16_t* scale, uint16_t* y, int B, int d, float eps,
                          bool bf16, hipStream_t s);
hipError_t launch_fill_u32(unsigned* p, size_t n, unsigned v, hipStream_t s);
hipError_t launch_copy_u16(const uint16_t* src, uint16_t* dst, size_t n, hipStream_t s);

}  // namespace larosa
