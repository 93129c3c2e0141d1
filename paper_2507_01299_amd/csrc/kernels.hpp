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
  // work split: workgroup g takes strip g / wps and, with j = g mod wps, the ranks
  // [j*chunk, min(K, (j+1)*chunk)) of the kept list: one strip per workgroup, G = nstrips * wps.
  int chunk, G, nstrips, wps;
  float* partial;             // [B][G][strip_cols] fp32 partial sums
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
  int wps;                    // workgroups per strip (row-streaming kernels; the batched kernels split differently)
  size_t partial_floats;      // per token
};

struct Tuning {
  int g_target = 0;           // target workgroups per launch; 0 = automatic (256 or 512)
  int min_rows = 112;         // minimum kept rows per workgroup (14 per wave: fewer, fatter workgroups beat a full chip
                              // for the o projection: 2457 rows over 21 instead of 32 workgroups per strip, -0.5 us)
  int variant = 0;            // row-waves per workgroup: 0 -> 8, 1 -> 16, 2 -> 4
  int fused = 1;              // decoder layer: 1 = Top-K fused into the projections, 0 = separate kernels
  int side_main_g = 0;        // workgroups of a projection that shares its launch with a shortcut adapter; 0 = by size
  int w4_wide_min_cols = 32768;   // 4-bit kernel: narrowest output that uses the 2048-column geometry
  int fused_max_width = 16384;    // decoder layer: widest block input selected inside every projection workgroup
  int side_g = 0;             // workgroups of that adapter; 0 = by size (both jobs resident at once: at most 512 slots)
  int hinted = 1;             // decoder layer: 1 = the down projection takes its threshold from histograms that the gate|up launch builds
  int contraction_tiles = 0;  // offline contractions: 0 = workgroup tile by size, 1 = 256 x 128, 2 = 256 x 256
};
Tuning& tuning();

// g_hint > 0 asks for that many workgroups instead of the automatic choice
constexpr int kRowListMax = 2048;   // ranks of a workgroup whose (row, coefficient) pairs are staged in LDS
// max_ranks caps the ranks per workgroup (more workgroups per strip instead), so that its list fits in LDS
GemvPlan plan_gemv(int d_out, int K, int g_hint = 0, int strip_cols = 512, int max_ranks = kRowListMax);
hipError_t launch_gemv(const GemvArgs& a, bool bf16, hipStream_t s);

// The same mat-vec over 4-bit weights (w4.hip): g.W is unused; the row loop reads packed codes and
// per-row, per-128-column scales.
struct W4Args {
  GemvArgs g;
  const uint32_t* Wq;         // [d_in, d_out/8] dwords, nibble k of dword m = code of column 8m+k
  const uint16_t* scales;     // [d_in, ng] 16-bit, weight = (code - 8) * scale
  int ng;                     // ceil(d_out / 128)
};
hipError_t launch_gemv_w4(const W4Args& w, bool bf16, hipStream_t s);
// 4-bit kernel geometry for this output width: 2048-column strips with 16-byte loads (32 codes per
// lane and row) when rows are 16-byte aligned and wide enough, else the 512-column strips of the
// 16-bit kernel with dword loads.
int w4_strip_cols(int d_out);
// round-to-nearest codes and scales of a 16-bit weight [d_in, d_out]
hipError_t launch_quantize_w4(const uint16_t* W, int d_in, int d_out, uint32_t* Wq, uint16_t* scales, bool bf16,
                              hipStream_t s);

// Column-sparse projection with the Top-K select fused into its prologue: the kept list is
// built inside every workgroup from the block's input vector.
enum : int { kSrcPlain = 0, kSrcGqa = 1, kSrcSilu = 2, kSrcNorm = 3 };
constexpr int kFusedChunkMax = 2048;   // (strip, rank) pairs per workgroup that fit its LDS list
struct FusedArgs {
  GemvArgs g;                 // W, y, sizes, work split, workspace, epilogue; g.h and g.idx unused
  int src_mode;               // where the input vector of width g.d_in comes from:
  const uint16_t* src;        //   kSrcPlain: [B, d_in];  kSrcNorm: x [B, d_in] to be RMS-normed;
                              //   kSrcGqa: q|k|v [B, d_q+2d_kv]  (kSrcSilu is a Top-K kernel source only)
  int d_q, d_kv, head_dim, group;
  const uint16_t* norm_scale; // kSrcNorm: [d_in] or nullptr
  float norm_eps;
  uint16_t* h_out;            // nullable: receives the input vector [B, d_in]
  int32_t* idx_out;           // nullable: receives the kept indices [B, K], ascending
  // Optional dense mat-vec that shares the launch (a residual adapter on the block's shortcut: it
  // depends only on the block's input, so its rows stream while the projection's workgroups select).
  // Workgroups [0, side_G) of the grid run it; side.idx == nullptr, own counters and partials.
  GemvArgs side;
  int side_G;                 // 0: no side job
  // gate|up projection with paired strips: pair_cols = d_ff (g.d_out == 2 d_ff), the finishing
  // workgroups also store pair_out [B, d_ff] = R(SiLU(gate) * up).  The plan must use d_ff / 256 strips.
  int pair_cols;
  uint16_t* pair_out;
  // Histograms handed from the producer of a vector to the launch that selects on it (kHistWords words
  // per token, zero before the producer runs; see topk_core.hpp):
  const unsigned* hist_in;    // nullable: histograms of the keys of this launch's input vector, complete
  unsigned* hist_out;         // nullable: the finishing workgroups add the keys of pair_out (paired strips) or
  int hist_col0, hist_col1;   //   of the y columns [hist_col0, hist_col1), each counting hist_weight times
  unsigned hist_weight;
  unsigned* zero_ptr;         // nullable: zero_words words that this launch clears (histograms a later launch fills)
  int zero_words;
};
constexpr int kHistCoarse = 256;                   // histogram layout: [0, 256) top 8 key bits, [256 + key] every 15-bit key
constexpr int kHistWords = kHistCoarse + 32768;
constexpr int kHintMaxWidth = 32768;   // widest input vector of the launch form that takes hist_in
// pair_cols > 0: strips are 256 channels of gate and of up each (see FusedArgs)
GemvPlan plan_fused(int d_out, int K, int g_hint = 0, int pair_cols = 0);
hipError_t launch_fused(const FusedArgs& a, bool bf16, hipStream_t s);

// Batched variant: y[b,:] = epilogue( sum_j C[b,j] * W[j,:] ) over ALL rows j, where C holds each
// token's activations with dropped channels set to zero (or the plain input for a dense product).
struct BatchArgs {
  const uint16_t* W;          // [d_in, d_out] input-channel-major
  const uint16_t* C;          // [B, d_in] coefficients
  uint16_t* y;                // [B, d_out]
  int d_in, d_out, B;
  int chunk, G, nstrips, wps; // strip g / wps, rows [(g % wps) * chunk, + chunk) of all d_in
  float* partial;             // [groups][G][tokens per group][128] fp32
  unsigned* counters;         // [groups][nstrips] arrival counters
  const uint16_t* coef_scale; // as in GemvArgs
  const uint16_t* rms_src;
  float rms_eps;
  const uint16_t* residual;
  uint16_t* y_pre;
};
constexpr int kBatchChunkMax = 4096;   // rows per workgroup segment (LDS coefficient staging)
// g_hint > 0: number of workgroups to aim for (a product that shares its launch takes its share of the chip)
GemvPlan plan_batched(int d_in, int d_out, bool mfma, int g_hint = 0);
int batched_g_total();      // workgroups a whole batched launch aims for
bool batched_uses_mfma(int B, bool coef_scale);
int batched_tokens_per_group(int B, bool coef_scale);
hipError_t launch_batched(const BatchArgs& a, bool bf16, hipStream_t s);
// Two independent batched products in one launch of the matrix-core kernel (same token count, no
// fp32 coefficient scale): the first side_G workgroups of the grid run `side`.
struct BatchPair {
  BatchArgs main, side;
  int side_G;                 // 0: main only
};
hipError_t launch_batched_pair(const BatchPair& p, bool bf16, hipStream_t s);
// C[b,:] = 0 except C[b, idx[b,t]] = h[b, idx[b,t]]
hipError_t launch_batch_prep(const uint16_t* h, const int32_t* idx, uint16_t* C, int B, int d_in, int K, hipStream_t s);

// Top-K select over stored 16-bit magnitudes, one workgroup per token.  masked (nullable)
// receives h with the dropped channels set to zero.
hipError_t launch_topk(const uint16_t* h, int B, int d, int K, int32_t* idx, uint16_t* vals, uint16_t* masked,
                       hipStream_t s);
// The same select on a vector that is built on the fly (kSrcGqa from q|k|v, kSrcSilu from gate|up,
// kSrcNorm = RMS-normed src, kSrcPlain from src itself); h_out (nullable) receives the vector [B, d].
struct TopkSource {
  int mode;
  const uint16_t* src;
  int d_q, d_kv, head_dim, group;   // kSrcGqa
  const uint16_t* norm_scale;       // kSrcNorm: [d] or nullptr
  float norm_eps;
  uint16_t* h_out;
};
hipError_t launch_topk_from(const TopkSource& sc, int B, int d, int K, int32_t* idx, uint16_t* masked, bool bf16,
                            hipStream_t s);

// Magnitude-threshold sparsifier: idx[b, 0..count[b]) = ascending channels with |h[b,i]| > eps; idx rows are d apart.
hipError_t launch_threshold_select(const uint16_t* h, int B, int d, float eps, int32_t* idx, int32_t* count, bool bf16,
                                   hipStream_t s);

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

// ---- offline contractions on the matrix cores (offline.hip): C[m,n] = post_scale * sum over the listed
// term pairs and over k of A_term(k,m) * B_term(k,n), fp32 accumulate.
struct ContractionArgs {
  const uint16_t* A;        // a_kmajor: [terms][Kd][M], else [terms][M][Kd]
  const uint16_t* B;        // [terms][Kd][N]
  int M, N, Kd;
  long a_term_stride, b_term_stride;   // elements between the 16-bit terms of a split operand
  int npairs;
  int pa[8], pb[8];         // term indices of each product that is added up
  float* C32;               // [M][N] fp32, or null
  uint16_t* C16;            // [M][N] rounded to the storage type, or null
  float post_scale;
  int accumulate;           // C32 only: add to what is there
  int symmetric;            // A == B, M == N: compute tiles on or above the diagonal, store both halves
  int tiles_m, tiles_n, patches_m, patches_n;   // filled in by launch_contraction
  long a_elements, b_elements;                  // extent of each operand over all its terms (filled in as well)
};
hipError_t launch_contraction(ContractionArgs a, bool a_kmajor, bool bf16, hipStream_t s);
// number of 16-bit terms an fp32 operand is split into (2 for f16, 3 for bf16)
int contraction_terms(bool bf16);
// dst[t][i] for t < terms: src[i] * pre_scale = sum_t dst[t][i] up to the last term's rounding
hipError_t launch_split_terms(const float* src, uint16_t* dst, long n, float pre_scale, bool bf16, hipStream_t s);

}  // namespace larosa
