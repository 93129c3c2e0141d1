// C ABI of liblarosa: argument checks, workspace carving, launch sequencing.
// No arithmetic of the method lives here; every step runs in the kernels.
#include "../../include/larosa.h"

#include <hip/hip_runtime.h>

#include <mutex>

#include "kernels.hpp"

using namespace larosa;

// Scratch of the entry point that allocates nothing (larosa_sparse_gemv_static): arrival counters followed by
// partial strips, laid out like a caller's workspace.  One copy per GPU the library runs on, held until the
// process ends.  In host code this name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[LAROSA_STATIC_SCRATCH_BYTES];

namespace {

constexpr size_t kCounterSlots = 4096;                        // arrival counters at the head of a workspace
constexpr size_t kCounterWords = kCounterSlots * kCounterStride;
constexpr size_t kCounterBytes = kCounterWords * sizeof(unsigned);
constexpr int kMaxTopkD = 32768;
constexpr size_t kHistBytes = kHistWords * sizeof(unsigned);

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool dtype_ok(int t) { return t == LAROSA_F16 || t == LAROSA_BF16; }

size_t gemv_partial_bytes_bound(int B, int d_in_max, int d_out_max) {
  const int sc = 512;
  const long nstrips = (d_out_max + sc - 1) / sc;
  long G = tuning().g_target > 0 ? tuning().g_target : 512;
  if (G < nstrips) G = nstrips;
  // the 4-bit kernel's wide geometry: per-token launches, 2048-column strips (4x the partial per workgroup)
  const size_t wide = static_cast<size_t>(B) * static_cast<size_t>(G) * 2 * 2048 * sizeof(float);
  if (B > 1) {   // batched kernels: chunk is capped, so very large products use more workgroups
    const long by_rows = (nstrips * d_in_max + kBatchChunkMax - 1) / kBatchChunkMax;
    if (G < by_rows) G = by_rows;
    B = (B + 31) / 32 * 32;   // token groups are padded
  }
  const size_t narrow = static_cast<size_t>(B) * static_cast<size_t>(G) * 2 * sc * sizeof(float);
  return narrow > wide ? narrow : wide;
}

size_t batched_partial_bytes(const GemvPlan& p, int B, bool coef_scale) {
  const int tpg = batched_tokens_per_group(B, coef_scale);
  const size_t groups = (B + tpg - 1) / tpg;
  return groups * tpg * p.partial_floats * sizeof(float);
}

// One launch of the batched kernels (B > 1): C holds the tokens' coefficients over all rows.  An
// optional side product (side.W != nullptr: same token count, no coefficient scale) shares the launch.
int run_batched(BatchArgs a, bool bf16, void* ws, size_t ws_bytes, hipStream_t st, BatchArgs side = BatchArgs{}) {
  const bool cs = a.coef_scale != nullptr;
  const bool has_side = side.W != nullptr && batched_uses_mfma(a.B, cs);
  // two products in one launch share the chip in proportion to the bytes each has to read
  int g_main = 0, g_side = 0;
  if (has_side) {
    const double bm = static_cast<double>(a.d_in) * a.d_out, bs = static_cast<double>(side.d_in) * side.d_out;
    const int total = batched_g_total();
    g_side = static_cast<int>(total * bs / (bm + bs) + 0.5);
    if (g_side < 1) g_side = 1;
    g_main = total - g_side > 0 ? total - g_side : 1;
  }
  const GemvPlan p = plan_batched(a.d_in, a.d_out, batched_uses_mfma(a.B, cs), g_main);
  const int tpg = batched_tokens_per_group(a.B, cs);
  const size_t groups = (a.B + tpg - 1) / tpg;
  size_t slots = groups * p.nstrips;
  size_t pbytes = batched_partial_bytes(p, a.B, cs);
  unsigned* counters = static_cast<unsigned*>(ws);
  char* partial = static_cast<char*>(ws) + kCounterBytes;
  BatchPair pr{};
  if (has_side) {
    const GemvPlan ps = plan_batched(side.d_in, side.d_out, true, g_side);
    side.chunk = ps.chunk;
    side.G = ps.G;
    side.nstrips = ps.nstrips;
    side.wps = ps.wps;
    side.counters = counters + slots * kCounterStride;
    side.partial = reinterpret_cast<float*>(partial + pbytes);
    slots += groups * ps.nstrips;
    pbytes += batched_partial_bytes(ps, a.B, false);
    pr.side = side;
    pr.side_G = ps.G;
  }
  if (slots > kCounterSlots) return LAROSA_EUNSUPPORTED;
  if (!ws || !aligned(ws, 256) || ws_bytes < kCounterBytes + pbytes) return LAROSA_EWORKSPACE;
  a.chunk = p.chunk;
  a.G = p.G;
  a.nstrips = p.nstrips;
  a.wps = p.wps;
  a.counters = counters;
  a.partial = reinterpret_cast<float*>(partial);
  pr.main = a;
  if (launch_batched_pair(pr, bf16, st) != hipSuccess) return LAROSA_EHIP;
  if (side.W != nullptr && !has_side) return run_batched(side, bf16, ws, ws_bytes, st);   // FMA path: two launches
  return LAROSA_OK;
}

struct Carver {
  char* base;
  size_t off, cap;
  bool ok = true;
  void* take(size_t bytes) {
    off = round_up(off, 256);
    if (off + bytes > cap) { ok = false; return nullptr; }
    void* p = base + off;
    off += bytes;
    return p;
  }
};

// One launch of the row-streaming kernel with its plan and workspace checks.
int run_gemv(GemvArgs a, bool bf16, void* ws, size_t ws_bytes, hipStream_t st) {
  const GemvPlan p = plan_gemv(a.d_out, a.K);
  if (static_cast<size_t>(a.B) * p.nstrips > kCounterSlots) return LAROSA_EUNSUPPORTED;
  const size_t need = kCounterBytes + static_cast<size_t>(a.B) * p.partial_floats * sizeof(float);
  if (!ws || !aligned(ws, 256) || ws_bytes < need) return LAROSA_EWORKSPACE;
  a.chunk = p.chunk;
  a.wps = p.wps;
  a.G = p.G;
  a.nstrips = p.nstrips;
  a.counters = static_cast<unsigned*>(ws);
  a.partial = reinterpret_cast<float*>(static_cast<char*>(ws) + kCounterBytes);
  return launch_gemv(a, bf16, st) == hipSuccess ? LAROSA_OK : LAROSA_EHIP;
}

// Workgroups of a projection (main) and of the shortcut adapter that shares its launch, from the
// two jobs' sizes in strip-rows (512-column pieces of weight rows).  Measured on 7B-, 8B- and 70B-shaped
// layers: 256 + 192 is best while one workgroup's share stays small; an adapter at least as large as
// the projection takes half of the 512 resident slots; a projection several times the adapter whose
// workgroups would each stream more than 1 MiB takes seven eighths of them (70B gate|up: 130 us with
// 384 + 128, 125 with 448 + 128, 124 with 448 + 64, 137 with 224 + 128).
struct SideSplit { int main_g, side_g; };
SideSplit side_split(int d_out, int K, int side_d) {
  SideSplit r{256, 192};
  const long main_T = static_cast<long>((d_out + 511) / 512) * K;
  const long side_T = static_cast<long>((side_d + 511) / 512) * side_d;
  if (side_T >= main_T && side_T / 192 > 512) r = {256, 256};
  else if (main_T >= 4 * side_T && main_T / 256 > 1024) r = {448, 64};
  if (tuning().side_main_g > 0) r.main_g = tuning().side_main_g;
  if (tuning().side_g > 0) r.side_g = tuning().side_g;
  return r;
}

// One launch of the projection kernel with the Top-K prologue, optionally with a dense side job
// (a.side.W != nullptr: y_side = x_side * W_side over all rows) in the same grid.
int run_fused(FusedArgs a, bool bf16, void* ws, size_t ws_bytes, hipStream_t st) {
  const bool side = a.side.W != nullptr;
  const SideSplit split = side ? side_split(a.g.d_out, a.g.K, a.side.d_out) : SideSplit{0, 0};
  const GemvPlan p = plan_fused(a.g.d_out, a.g.K, split.main_g, a.pair_cols);
  size_t slots = static_cast<size_t>(a.g.B) * p.nstrips;
  size_t pfloats = static_cast<size_t>(a.g.B) * p.partial_floats;
  unsigned* counters = static_cast<unsigned*>(ws);
  float* partial = reinterpret_cast<float*>(static_cast<char*>(ws) + kCounterBytes);
  a.side_G = 0;
  if (side) {
    const GemvPlan ps = plan_gemv(a.side.d_out, a.side.K, split.side_g);
    a.side.chunk = ps.chunk;
    a.side.wps = ps.wps;
    a.side.G = ps.G;
    a.side.nstrips = ps.nstrips;
    a.side.counters = counters + slots * kCounterStride;
    a.side.partial = partial + pfloats;
    a.side_G = ps.G;
    slots += static_cast<size_t>(a.side.B) * ps.nstrips;
    pfloats += static_cast<size_t>(a.side.B) * ps.partial_floats;
  }
  if (slots > kCounterSlots) return LAROSA_EUNSUPPORTED;
  if (!ws || !aligned(ws, 256) || ws_bytes < kCounterBytes + pfloats * sizeof(float)) return LAROSA_EWORKSPACE;
  a.g.chunk = p.chunk;
  a.g.wps = p.wps;
  a.g.G = p.G;
  a.g.nstrips = p.nstrips;
  a.g.counters = counters;
  a.g.partial = partial;
  return launch_fused(a, bf16, st) == hipSuccess ? LAROSA_OK : LAROSA_EHIP;
}

int check_gemv_shapes(int B, int d_in, int d_out, int K) {
  if (B < 1 || d_in < 8 || d_out < 8 || K < 1 || K > d_in) return LAROSA_EINVAL;
  if (d_in % 8 || d_out % 8) return LAROSA_EINVAL;
  if (static_cast<long>((d_out + 511) / 512) * K >= (1L << 30)) return LAROSA_EUNSUPPORTED;
  if (B > 65535) return LAROSA_EUNSUPPORTED;
  return LAROSA_OK;
}

}  // namespace

extern "C" {

const char* larosa_status_string(int status) {
  switch (status) {
    case LAROSA_OK: return "ok";
    case LAROSA_EINVAL: return "invalid argument";
    case LAROSA_EUNSUPPORTED: return "unsupported size";
    case LAROSA_EWORKSPACE: return "workspace missing, misaligned or too small";
    case LAROSA_EHIP: return "HIP launch error";
    default: return "unknown status";
  }
}

int larosa_version(void) { return 100; }

size_t larosa_workspace_bytes(int B, int d_in_max, int d_out_max, int K_max) {
  if (B < 1 || d_in_max < 1 || d_out_max < 1 || K_max < 1) return 0;
  // counters | partial strips | (B > 1) masked coefficient matrix of larosa_sparse_gemv
  size_t n = round_up(kCounterBytes + gemv_partial_bytes_bound(B, d_in_max, d_out_max), 256);
  if (B > 1) n += round_up(static_cast<size_t>(B) * d_in_max * 2, 256);
  return n;
}

int larosa_workspace_init(void* ws, size_t ws_bytes, void* stream) {
  if (!ws || !aligned(ws, 256) || ws_bytes < kCounterBytes) return LAROSA_EWORKSPACE;
  return launch_fill_u32(static_cast<unsigned*>(ws), kCounterWords, 0u, static_cast<hipStream_t>(stream)) ==
                 hipSuccess
             ? LAROSA_OK
             : LAROSA_EHIP;
}

int larosa_dense_gemv(const void* Wp, const void* x, void* y, int B, int d_in, int d_out, larosa_dtype t,
                      void* ws, size_t ws_bytes, void* stream) {
  if (!Wp || !x || !y || !dtype_ok(t)) return LAROSA_EINVAL;
  if (!aligned(Wp, 16) || !aligned(x, 16) || !aligned(y, 16)) return LAROSA_EINVAL;
  if (int rc = check_gemv_shapes(B, d_in, d_out, d_in)) return rc;
  if (B > 1) {
    BatchArgs ba{};
    ba.W = static_cast<const uint16_t*>(Wp);
    ba.C = static_cast<const uint16_t*>(x);
    ba.y = static_cast<uint16_t*>(y);
    ba.d_in = d_in; ba.d_out = d_out; ba.B = B;
    return run_batched(ba, t == LAROSA_BF16, ws, ws_bytes, static_cast<hipStream_t>(stream));
  }
  GemvArgs a{};
  a.W = static_cast<const uint16_t*>(Wp);
  a.h = static_cast<const uint16_t*>(x);
  a.idx = nullptr;
  a.y = static_cast<uint16_t*>(y);
  a.d_in = d_in; a.d_out = d_out; a.K = d_in; a.B = B;
  return run_gemv(a, t == LAROSA_BF16, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

int larosa_rotate(const void* x, const void* Q, void* h, int B, int d, larosa_dtype t, void* ws,
                  size_t ws_bytes, void* stream) {
  return larosa_dense_gemv(Q, x, h, B, d, d, t, ws, ws_bytes, stream);
}

int larosa_topk(const void* h, int B, int d, int K, int32_t* idx, void* vals, larosa_dtype t, void* ws,
                size_t ws_bytes, void* stream) {
  (void)ws; (void)ws_bytes;
  if (!h || !idx || !dtype_ok(t)) return LAROSA_EINVAL;
  if (!aligned(h, 16) || !aligned(idx, 4) || (vals && !aligned(vals, 2))) return LAROSA_EINVAL;
  if (B < 1 || d < 8 || d % 8 || K < 1 || K > d) return LAROSA_EINVAL;
  if (d > kMaxTopkD || B > 65535) return LAROSA_EUNSUPPORTED;
  return launch_topk(static_cast<const uint16_t*>(h), B, d, K, idx, static_cast<uint16_t*>(vals), nullptr,
                     static_cast<hipStream_t>(stream)) == hipSuccess
             ? LAROSA_OK
             : LAROSA_EHIP;
}

int larosa_sparse_gemv(const void* Wp, const void* h, const int32_t* idx, void* y, int B, int d_in, int d_out,
                       int K, larosa_dtype t, void* ws, size_t ws_bytes, void* stream) {
  if (!Wp || !h || !idx || !y || !dtype_ok(t)) return LAROSA_EINVAL;
  if (!aligned(Wp, 16) || !aligned(h, 16) || !aligned(y, 16) || !aligned(idx, 4)) return LAROSA_EINVAL;
  if (int rc = check_gemv_shapes(B, d_in, d_out, K)) return rc;
  if (B > 1) {
    // masked coefficient matrix in the tail of the workspace, then one pass over the weight
    const GemvPlan p = plan_batched(d_in, d_out, batched_uses_mfma(B, false));
    const size_t head = round_up(kCounterBytes + batched_partial_bytes(p, B, false), 256);
    const size_t cbytes = static_cast<size_t>(B) * d_in * 2;
    if (!ws || !aligned(ws, 256) || ws_bytes < head + cbytes) return LAROSA_EWORKSPACE;
    uint16_t* C = reinterpret_cast<uint16_t*>(static_cast<char*>(ws) + head);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (launch_batch_prep(static_cast<const uint16_t*>(h), idx, C, B, d_in, K, st) != hipSuccess) return LAROSA_EHIP;
    BatchArgs ba{};
    ba.W = static_cast<const uint16_t*>(Wp);
    ba.C = C;
    ba.y = static_cast<uint16_t*>(y);
    ba.d_in = d_in; ba.d_out = d_out; ba.B = B;
    return run_batched(ba, t == LAROSA_BF16, ws, head, st);
  }
  GemvArgs a{};
  a.W = static_cast<const uint16_t*>(Wp);
  a.h = static_cast<const uint16_t*>(h);
  a.idx = idx;
  a.y = static_cast<uint16_t*>(y);
  a.d_in = d_in; a.d_out = d_out; a.K = K; a.B = B;
  return run_gemv(a, t == LAROSA_BF16, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

// ---------------------------------------------------------------------------------------------
// decoder layer
// ---------------------------------------------------------------------------------------------

static int check_layer(const larosa_layer* L, int B) {
  if (!L || B < 1 || B > 65535) return LAROSA_EINVAL;
  if (!dtype_ok(L->dtype)) return LAROSA_EINVAL;
  if (L->d < 8 || L->d_q < 8 || L->d_kv < 8 || L->d_ff < 8) return LAROSA_EINVAL;
  if (L->d % 8 || L->d_q % 8 || L->d_kv % 8 || L->d_ff % 8) return LAROSA_EINVAL;
  if (L->head_dim < 8 || L->head_dim % 8 || L->d_q % L->head_dim || L->d_kv % L->head_dim) return LAROSA_EINVAL;
  if ((L->d_q / L->head_dim) % (L->d_kv / L->head_dim)) return LAROSA_EINVAL;
  if (L->K1 < 1 || L->K1 > L->d || L->K2 < 1 || L->K2 > L->d_q || L->K3 < 1 || L->K3 > L->d || L->K4 < 1 ||
      L->K4 > L->d_ff)
    return LAROSA_EINVAL;
  if (!L->Wqkv || !L->Wo || !L->Wgu || !L->Wdown) return LAROSA_EINVAL;
  const void* ptrs[] = {L->Wqkv, L->Wo, L->Wgu, L->Wdown, L->Q_attn, L->Q_mlp, L->adapter, L->rms_attn, L->rms_mlp,
                        L->shortcut_attn, L->shortcut_mlp};
  for (const void* p : ptrs)
    if (p && !aligned(p, 16)) return LAROSA_EINVAL;
  if (L->attn_mode != 0) return LAROSA_EUNSUPPORTED;
  if (L->d > kMaxTopkD || L->d_q > kMaxTopkD || L->d_ff > kMaxTopkD) return LAROSA_EUNSUPPORTED;
  return LAROSA_OK;
}

static int max3(int a, int b, int c) { return a > b ? (a > c ? a : c) : (b > c ? b : c); }

static size_t layer_gemv_ws(const larosa_layer* L, int B) {
  size_t s = larosa_workspace_bytes(B, max3(L->d, L->d_q, L->d_ff), max3(L->d_q + 2 * L->d_kv, 2 * L->d_ff, L->d),
                                    max3(L->d, L->d_q, L->d_ff));
  const GemvPlan plans[] = {plan_fused(L->d_q + 2 * L->d_kv, L->K1), plan_fused(L->d, L->K2),
                            plan_fused(2 * L->d_ff, L->K3), plan_fused(L->d, L->K4)};
  for (const GemvPlan& p : plans) {
    const size_t need = round_up(kCounterBytes + static_cast<size_t>(B) * p.partial_floats * sizeof(float), 256);
    if (need > s) s = need;
  }
  if (L->shortcut_attn || L->shortcut_mlp) {   // a projection and its shortcut adapter in one launch
    const int douts[] = {L->d_q + 2 * L->d_kv, 2 * L->d_ff};
    const int Ks[] = {L->K1, L->K3};
    for (int i = 0; i < 2; ++i) {
      const SideSplit split = side_split(douts[i], Ks[i], L->d);
      const GemvPlan side = plan_gemv(L->d, L->d, split.side_g);
      for (int pair = 0; pair <= i; ++pair) {     // gate|up also in its paired-strip geometry
        const GemvPlan p = plan_fused(douts[i], Ks[i], split.main_g, pair ? L->d_ff : 0);
        const size_t need = round_up(
            kCounterBytes + static_cast<size_t>(B) * (p.partial_floats + side.partial_floats) * sizeof(float), 256);
        if (need > s) s = need;
      }
    }
  }
  if (B > 1) {
    const bool cs = L->rms_attn || L->rms_mlp;
    for (int mf = 0; mf < 2; ++mf) {
      const bool m = mf != 0;
      const GemvPlan bp[] = {plan_batched(L->d, L->d, m), plan_batched(L->d, L->d_q + 2 * L->d_kv, m),
                             plan_batched(L->d_q, L->d, m), plan_batched(L->d, 2 * L->d_ff, m),
                             plan_batched(L->d_ff, L->d, m)};
      const size_t side_bytes = (m && (L->shortcut_attn || L->shortcut_mlp)) ? batched_partial_bytes(bp[0], B, false) : 0;
      for (const GemvPlan& p : bp) {
        const size_t need = round_up(kCounterBytes + batched_partial_bytes(p, B, m ? false : cs) + side_bytes, 256);
        if (need > s) s = need;
      }
    }
  }
  return s;
}

size_t larosa_layer_workspace_bytes(const larosa_layer* L, int B) {
  if (check_layer(L, B) != LAROSA_OK) return 0;
  const size_t E = 2, Bz = static_cast<size_t>(B);
  size_t s = layer_gemv_ws(L, B);
  const size_t widths[] = {(size_t)L->d, (size_t)(L->d_q + 2 * L->d_kv), (size_t)L->d_q, (size_t)L->d,
                           (size_t)L->d, (size_t)L->d, (size_t)(2 * L->d_ff), (size_t)L->d_ff,
                           (size_t)L->d, (size_t)L->d, (size_t)L->d, (size_t)L->d};
  for (size_t w : widths) s += round_up(Bz * w * E, 256) + 256;
  const int Ks[] = {L->K1, L->K2, L->K3, L->K4};
  for (int k : Ks) s += round_up(Bz * k * sizeof(int32_t), 256) + 256;
  if (B > 1) s += round_up(Bz * max3(L->d, L->d_q, L->d_ff) * E, 256) + 256;   // masked activations
  s += round_up(kHistBytes, 256) + 256;                                       // key histograms of the MLP vector (batch 1)
  return s;
}

namespace {

enum LayerPart { kWholeLayer = 0, kUntilQkv = 1, kAfterAttention = 2 };

// The decoder layer, whole or split around a caller's attention core.  kUntilQkv: q|k|v goes to
// qkv_ext and the attention shortcut value (if the layer has that adapter) to s1_ext, then the call
// returns.  kAfterAttention: x_in is the residual of the attention block (the layer input, or that
// shortcut value) and attn_ext [B, d_q] the attention core's output, which takes the place of h2.
int layer_run(const larosa_layer* L, const void* x_in, void* x_out, int B, const larosa_trace* tr, void* ws,
              size_t ws_bytes, void* stream, LayerPart part, void* qkv_ext, void* s1_ext, const void* attn_ext) {
  if (int rc = check_layer(L, B)) return rc;
  if (!x_in || !aligned(x_in, 16)) return LAROSA_EINVAL;
  if (part == kUntilQkv) {
    if (!qkv_ext || !aligned(qkv_ext, 16)) return LAROSA_EINVAL;
    if (L->shortcut_attn && (!s1_ext || !aligned(s1_ext, 16))) return LAROSA_EINVAL;
  } else {
    if (!x_out || x_in == x_out || !aligned(x_out, 16)) return LAROSA_EINVAL;
    if (part == kAfterAttention && (!attn_ext || !aligned(attn_ext, 16))) return LAROSA_EINVAL;
  }
  if (!ws || !aligned(ws, 256) || ws_bytes < larosa_layer_workspace_bytes(L, B)) return LAROSA_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool bf = L->dtype == LAROSA_BF16;
  const size_t Bz = static_cast<size_t>(B);
  const int d = L->d, d_q = L->d_q, d_kv = L->d_kv, d_ff = L->d_ff;
  const int d_qkv = d_q + 2 * d_kv;
  const bool norm = L->rms_eps >= 0.f;

  const size_t gws = layer_gemv_ws(L, B);
  Carver cv{static_cast<char*>(ws), gws, ws_bytes};
  auto buf16 = [&](void* traced, size_t width) {
    return static_cast<uint16_t*>(traced ? traced : cv.take(Bz * width * 2));
  };
  auto bufidx = [&](int32_t* traced, int K) {
    return traced ? traced : static_cast<int32_t*>(cv.take(Bz * K * sizeof(int32_t)));
  };
  static const larosa_trace kNoTrace{};
  const larosa_trace& T = tr ? *tr : kNoTrace;
  uint16_t* h1 = buf16(T.h1, d);
  uint16_t* qkv = part == kUntilQkv ? static_cast<uint16_t*>(qkv_ext) : buf16(T.qkv, d_qkv);
  uint16_t* h2 = buf16(T.h2, d_q);
  uint16_t* o = buf16(T.o, d);
  uint16_t* x1 = buf16(T.x1, d);
  uint16_t* h3 = buf16(T.h3, d);
  uint16_t* gu = buf16(T.gu, 2 * d_ff);
  uint16_t* h4 = buf16(T.h4, d_ff);
  uint16_t* down = buf16(T.down, d);
  uint16_t* x2 = L->adapter ? buf16(T.x2, d) : static_cast<uint16_t*>(x_out);
  // after the attention core the shortcut value arrives as x_in, so there is none to compute
  uint16_t* s1 = !L->shortcut_attn || part == kAfterAttention ? nullptr
                 : part == kUntilQkv                         ? static_cast<uint16_t*>(s1_ext)
                                                             : buf16(T.s1, d);
  const uint16_t* attn = static_cast<const uint16_t*>(attn_ext);
  uint16_t* s2 = L->shortcut_mlp ? buf16(T.s2, d) : nullptr;
  int32_t* idx1 = bufidx(T.idx1, L->K1);
  int32_t* idx2 = bufidx(T.idx2, L->K2);
  int32_t* idx3 = bufidx(T.idx3, L->K3);
  int32_t* idx4 = bufidx(T.idx4, L->K4);
  uint16_t* masked = B > 1 ? static_cast<uint16_t*>(cv.take(Bz * max3(d, d_q, d_ff) * 2)) : nullptr;
  // batch 1: the gate|up launch's finishing workgroups build the key histograms of the MLP vector, the down
  // projection reads its threshold off them; the o projection's launch (always between two uses) clears them
  unsigned* hist4 = (B == 1 && tuning().fused && tuning().hinted) ? static_cast<unsigned*>(cv.take(kHistBytes)) : nullptr;
  if (!cv.ok) return LAROSA_EWORKSPACE;
  const uint16_t* x = static_cast<const uint16_t*>(x_in);

#define LAROSA_TRY(expr)                 \
  do {                                   \
    const int rc__ = (expr);             \
    if (rc__ != LAROSA_OK) return rc__;  \
  } while (0)
#define LAROSA_HIP(expr)                               \
  do {                                                 \
    if ((expr) != hipSuccess) return LAROSA_EHIP;      \
  } while (0)

  // block input: pre-norm, rotation, one rounding
  auto block_input = [&](const uint16_t* src, const void* Q, const void* scale, uint16_t* dst) -> int {
    if (Q && B > 1) {
      BatchArgs a{};
      a.W = static_cast<const uint16_t*>(Q);
      a.C = src; a.y = dst;
      a.d_in = d; a.d_out = d; a.B = B;
      if (norm) {
        a.rms_src = src;
        a.rms_eps = L->rms_eps;
        a.coef_scale = static_cast<const uint16_t*>(scale);
      }
      return run_batched(a, bf, ws, gws, st);
    }
    if (Q) {
      GemvArgs a{};
      a.W = static_cast<const uint16_t*>(Q);
      a.h = src; a.y = dst;
      a.d_in = d; a.d_out = d; a.K = d; a.B = B;
      if (norm) {
        a.rms_src = src;
        a.rms_eps = L->rms_eps;
        a.coef_scale = static_cast<const uint16_t*>(scale);
      }
      return run_gemv(a, bf, ws, gws, st);
    }
    if (norm)
      return launch_rmsnorm(src, static_cast<const uint16_t*>(scale), dst, B, d, L->rms_eps, bf, st) == hipSuccess
                 ? LAROSA_OK
                 : LAROSA_EHIP;
    return launch_copy_u16(src, dst, Bz * d, st) == hipSuccess ? LAROSA_OK : LAROSA_EHIP;
  };
  // residual adapter on a shortcut as a launch of its own: dst = R(src A)
  auto shortcut = [&](const uint16_t* src, const void* A, uint16_t* dst) -> int {
    if (B > 1) {
      BatchArgs a{};
      a.W = static_cast<const uint16_t*>(A);
      a.C = src; a.y = dst;
      a.d_in = d; a.d_out = d; a.B = B;
      return run_batched(a, bf, ws, gws, st);
    }
    GemvArgs a{};
    a.W = static_cast<const uint16_t*>(A);
    a.h = src; a.y = dst;
    a.d_in = d; a.d_out = d; a.K = d; a.B = B;
    return run_gemv(a, bf, ws, gws, st);
  };
  auto sparse = [&](const void* W, const uint16_t* h, const int32_t* idx, uint16_t* y, int d_in, int d_out, int K,
                    const uint16_t* residual, uint16_t* y_pre) -> int {
    GemvArgs a{};
    a.W = static_cast<const uint16_t*>(W);
    a.h = h; a.idx = idx; a.y = y;
    a.d_in = d_in; a.d_out = d_out; a.K = K; a.B = B;
    a.residual = residual; a.y_pre = y_pre;
    return run_gemv(a, bf, ws, gws, st);
  };

  auto mark = [&](int i) {
    if (T.stage_events[i]) (void)hipEventRecord(static_cast<hipEvent_t>(T.stage_events[i]), st);
  };
  mark(0);
  if (B > 1) {
    // Batched decode: per-token Top-K writes each token's activations with the dropped channels
    // zeroed (the index lists only when the caller traces them: the products do not read them), and one pass over all weight rows serves every token (the union of the index sets).
    // a projection over the masked activations; the shortcut adapter of the block (scA: dst = src scA)
    // shares its launch
    auto project = [&](const void* W, int d_in, int d_out, uint16_t* y, const uint16_t* residual, uint16_t* y_pre,
                       const void* scA = nullptr, const uint16_t* sc_src = nullptr, uint16_t* sc_dst = nullptr) -> int {
      BatchArgs a{};
      a.W = static_cast<const uint16_t*>(W);
      a.C = masked; a.y = y;
      a.d_in = d_in; a.d_out = d_out; a.B = B;
      a.residual = residual; a.y_pre = y_pre;
      BatchArgs side{};
      if (scA) {
        side.W = static_cast<const uint16_t*>(scA);
        side.C = sc_src; side.y = sc_dst;
        side.d_in = d; side.d_out = d; side.B = B;
      }
      return run_batched(a, bf, ws, gws, st, side);
    };
    // block input and its select: with an explicit rotation the matrix pass comes first; with the
    // rotation absorbed the pre-norm is formed inside the select kernel
    auto input_and_select = [&](const uint16_t* src, const void* Q, const void* scale, uint16_t* h, int K,
                                int32_t* idx, int stage) -> int {
      if (Q || !norm) {
        if (int rc = block_input(src, Q, scale, h)) return rc;
        mark(stage);
        return launch_topk(h, B, d, K, idx, nullptr, masked, st) == hipSuccess ? LAROSA_OK : LAROSA_EHIP;
      }
      mark(stage);
      TopkSource sc{};
      sc.mode = kSrcNorm; sc.src = src; sc.h_out = h;
      sc.norm_scale = static_cast<const uint16_t*>(scale); sc.norm_eps = L->rms_eps;
      return launch_topk_from(sc, B, d, K, idx, masked, bf, st) == hipSuccess ? LAROSA_OK : LAROSA_EHIP;
    };
    if (part != kAfterAttention) {
      LAROSA_TRY(input_and_select(x, L->Q_attn, L->rms_attn, h1, L->K1, T.idx1, 1));
      LAROSA_TRY(project(L->Wqkv, d, d_qkv, qkv, nullptr, nullptr, s1 ? L->shortcut_attn : nullptr, x, s1));
      mark(2);
      if (part == kUntilQkv) return LAROSA_OK;
    }
    {
      TopkSource sc{};
      sc.mode = attn ? kSrcPlain : kSrcGqa; sc.src = attn ? attn : qkv; sc.h_out = h2;
      sc.d_q = d_q; sc.d_kv = d_kv; sc.head_dim = L->head_dim;
      sc.group = (d_q / L->head_dim) / (d_kv / L->head_dim);
      LAROSA_HIP(launch_topk_from(sc, B, d_q, L->K2, T.idx2, masked, bf, st));
    }
    LAROSA_TRY(project(L->Wo, d_q, d, x1, s1 ? s1 : x, o));
    mark(3);
    LAROSA_TRY(input_and_select(x1, L->Q_mlp, L->rms_mlp, h3, L->K3, T.idx3, 4));
    LAROSA_TRY(project(L->Wgu, d, 2 * d_ff, gu, nullptr, nullptr, L->shortcut_mlp, x1, s2));
    mark(5);
    {
      TopkSource sc{};
      sc.mode = kSrcSilu; sc.src = gu; sc.h_out = h4;
      LAROSA_HIP(launch_topk_from(sc, B, d_ff, L->K4, T.idx4, masked, bf, st));
    }
    LAROSA_TRY(project(L->Wdown, d_ff, d, x2, s2 ? s2 : x1, down));
    mark(6);
  } else if (tuning().fused) {
    // Top-K fused into the projections: 4 projection kernels (+ one rotation each when Q is given)
    auto fused = [&](int mode, const uint16_t* src, const void* W, uint16_t* y, int d_in, int d_out, int K,
                     const uint16_t* residual, uint16_t* y_pre, uint16_t* h_out, int32_t* idx_out,
                     const void* nscale, const void* sideA = nullptr, const uint16_t* side_x = nullptr,
                     uint16_t* side_y = nullptr, int pair_cols = 0, uint16_t* pair_out = nullptr,
                     const unsigned* hist_in = nullptr, unsigned* hist_out = nullptr, unsigned* zero = nullptr) -> int {
      FusedArgs a{};
      a.pair_cols = pair_cols; a.pair_out = pair_out;
      a.hist_in = hist_in; a.hist_out = hist_out; a.hist_weight = 1;
      a.zero_ptr = zero; a.zero_words = zero ? static_cast<int>(kHistBytes / sizeof(unsigned)) : 0;
      if (sideA) {
        a.side.W = static_cast<const uint16_t*>(sideA);
        a.side.h = side_x; a.side.y = side_y;
        a.side.d_in = d; a.side.d_out = d; a.side.K = d; a.side.B = B;
      }
      a.g.W = static_cast<const uint16_t*>(W);
      a.g.y = y;
      a.g.d_in = d_in; a.g.d_out = d_out; a.g.K = K; a.g.B = B;
      a.g.residual = residual; a.g.y_pre = y_pre;
      a.src_mode = mode; a.src = src;
      a.d_q = d_q; a.d_kv = d_kv; a.head_dim = L->head_dim;
      a.group = (d_q / L->head_dim) / (d_kv / L->head_dim);
      a.norm_scale = static_cast<const uint16_t*>(nscale); a.norm_eps = L->rms_eps;
      a.h_out = h_out; a.idx_out = idx_out;
      return run_fused(a, bf, ws, gws, st);
    };
    // the block's first projection; its shortcut adapter (sc: A, dst) shares the launch
    auto first = [&](const uint16_t* src, const void* Q, const void* scale, uint16_t* h, void* h_traced, const void* W,
                     uint16_t* y, int d_out, int K, int32_t* idx_traced, const void* scA, uint16_t* sc_dst,
                     int pair_cols, uint16_t* pair_out, unsigned* hist_out) -> int {
      if (Q) {
        if (int rc = block_input(src, Q, scale, h)) return rc;
        mark(d_out == d_qkv && W == L->Wqkv ? 1 : 4);
        return fused(kSrcPlain, h, W, y, d, d_out, K, nullptr, nullptr, nullptr, idx_traced, nullptr, scA, src,
                     sc_dst, pair_cols, pair_out, nullptr, hist_out);
      }
      mark(d_out == d_qkv && W == L->Wqkv ? 1 : 4);
      return fused(norm ? kSrcNorm : kSrcPlain, src, W, y, d, d_out, K, nullptr, nullptr,
                   static_cast<uint16_t*>(h_traced), idx_traced, scale, scA, src, sc_dst, pair_cols, pair_out, nullptr,
                   hist_out);
    };
    if (part != kAfterAttention) {
      LAROSA_TRY(first(x, L->Q_attn, L->rms_attn, h1, T.h1, L->Wqkv, qkv, d_qkv, L->K1, T.idx1,
                       s1 ? L->shortcut_attn : nullptr, s1, 0, nullptr, nullptr));
      mark(2);
      if (part == kUntilQkv) return LAROSA_OK;
    }
    LAROSA_TRY(fused(attn ? kSrcPlain : kSrcGqa, attn ? attn : qkv, L->Wo, x1, d_q, d, L->K2, s1 ? s1 : x,
                     static_cast<uint16_t*>(T.o), static_cast<uint16_t*>(T.h2), T.idx2, nullptr, nullptr, nullptr, nullptr,
                     0, nullptr, nullptr, nullptr, hist4));
    mark(3);
    // gate|up with paired strips: the workgroups that finish it also store h4 = R(SiLU(gate) * up)
    LAROSA_TRY(first(x1, L->Q_mlp, L->rms_mlp, h3, T.h3, L->Wgu, gu, 2 * d_ff, L->K3, T.idx3, L->shortcut_mlp, s2, d_ff,
                     h4, hist4));
    mark(5);
    if (hist4) {
      LAROSA_TRY(fused(kSrcPlain, h4, L->Wdown, x2, d_ff, d, L->K4, s2 ? s2 : x1, static_cast<uint16_t*>(T.down),
                       nullptr, T.idx4, nullptr, nullptr, nullptr, nullptr, 0, nullptr, hist4));
    } else if (d_ff <= tuning().fused_max_width) {
      LAROSA_TRY(fused(kSrcPlain, h4, L->Wdown, x2, d_ff, d, L->K4, s2 ? s2 : x1, static_cast<uint16_t*>(T.down),
                       nullptr, T.idx4, nullptr));
    } else {
      // a wide intermediate vector makes the per-workgroup selection too long: select once instead
      LAROSA_HIP(launch_topk(h4, B, d_ff, L->K4, idx4, nullptr, nullptr, st));
      LAROSA_TRY(sparse(L->Wdown, h4, idx4, x2, d_ff, d, L->K4, s2 ? s2 : x1, down));
    }
    mark(6);
  } else {
  // attention block: h1 -> q|k|v -> (attention core) -> h2 -> o -> + residual
  if (part != kAfterAttention) {
    if (s1) LAROSA_TRY(shortcut(x, L->shortcut_attn, s1));
    LAROSA_TRY(block_input(x, L->Q_attn, L->rms_attn, h1));
    mark(1);
    LAROSA_HIP(launch_topk(h1, B, d, L->K1, idx1, nullptr, nullptr, st));
    LAROSA_TRY(sparse(L->Wqkv, h1, idx1, qkv, d, d_qkv, L->K1, nullptr, nullptr));
    mark(2);
    if (part == kUntilQkv) return LAROSA_OK;
    LAROSA_HIP(launch_gqa_expand(qkv, h2, B, d_q, d_kv, L->head_dim, st));
  } else {
    LAROSA_HIP(launch_copy_u16(attn, h2, Bz * d_q, st));
  }
  LAROSA_HIP(launch_topk(h2, B, d_q, L->K2, idx2, nullptr, nullptr, st));
  LAROSA_TRY(sparse(L->Wo, h2, idx2, x1, d_q, d, L->K2, s1 ? s1 : x, o));
  mark(3);
  // MLP block: h3 -> gate|up -> h4 -> down -> + residual
  if (s2) LAROSA_TRY(shortcut(x1, L->shortcut_mlp, s2));
  LAROSA_TRY(block_input(x1, L->Q_mlp, L->rms_mlp, h3));
  mark(4);
  LAROSA_HIP(launch_topk(h3, B, d, L->K3, idx3, nullptr, nullptr, st));
  LAROSA_TRY(sparse(L->Wgu, h3, idx3, gu, d, 2 * d_ff, L->K3, nullptr, nullptr));
  mark(5);
  LAROSA_HIP(launch_silu_mul(gu, h4, B, d_ff, bf, st));
  LAROSA_HIP(launch_topk(h4, B, d_ff, L->K4, idx4, nullptr, nullptr, st));
  LAROSA_TRY(sparse(L->Wdown, h4, idx4, x2, d_ff, d, L->K4, s2 ? s2 : x1, down));
  mark(6);
  }
  // residual adapter
  if (L->adapter && B > 1) {
    BatchArgs a{};
    a.W = static_cast<const uint16_t*>(L->adapter);
    a.C = x2; a.y = static_cast<uint16_t*>(x_out);
    a.d_in = d; a.d_out = d; a.B = B;
    LAROSA_TRY(run_batched(a, bf, ws, gws, st));
  } else if (L->adapter) {
    GemvArgs a{};
    a.W = static_cast<const uint16_t*>(L->adapter);
    a.h = x2; a.y = static_cast<uint16_t*>(x_out);
    a.d_in = d; a.d_out = d; a.K = d; a.B = B;
    LAROSA_TRY(run_gemv(a, bf, ws, gws, st));
  } else if (T.x2) {
    LAROSA_HIP(launch_copy_u16(x2, static_cast<uint16_t*>(T.x2), Bz * d, st));
  }
  mark(7);
#undef LAROSA_TRY
#undef LAROSA_HIP
  return LAROSA_OK;
}

}  // namespace

int larosa_layer_forward(const larosa_layer* L, const void* x_in, void* x_out, int B, const larosa_trace* tr,
                         void* ws, size_t ws_bytes, void* stream) {
  return layer_run(L, x_in, x_out, B, tr, ws, ws_bytes, stream, kWholeLayer, nullptr, nullptr, nullptr);
}

int larosa_layer_qkv(const larosa_layer* L, const void* x, void* qkv, void* s1, int B, const larosa_trace* tr,
                     void* ws, size_t ws_bytes, void* stream) {
  return layer_run(L, x, nullptr, B, tr, ws, ws_bytes, stream, kUntilQkv, qkv, s1, nullptr);
}

int larosa_layer_after_attention(const larosa_layer* L, const void* residual, const void* attn, void* x_out, int B,
                                 const larosa_trace* tr, void* ws, size_t ws_bytes, void* stream) {
  return layer_run(L, residual, x_out, B, tr, ws, ws_bytes, stream, kAfterAttention, nullptr, nullptr, attn);
}

// ---- offline contractions -------------------------------------------------------------------

namespace {

// f16 terms of a rotation are taken from 64 Q: entries of an orthogonal matrix are at most 1 in
// magnitude and mostly near 1/sqrt(d), whose second term would fall into the f16 subnormals.
inline float term_pre_scale(bool bf16) { return bf16 ? 1.0f : 64.0f; }

inline size_t terms_bytes(int d, bool bf16) {
  return round_up(static_cast<size_t>(contraction_terms(bf16)) * d * d * 2, 256);
}

int check_offline(const void* a, const void* b, const void* c, int d, larosa_dtype t) {
  if (!a || !b || !c || !dtype_ok(t)) return LAROSA_EINVAL;
  if (!aligned(a, 16) || !aligned(b, 16) || !aligned(c, 16)) return LAROSA_EINVAL;
  if (d < 8 || d % 8 || d > 32768) return LAROSA_EINVAL;
  return LAROSA_OK;
}

}  // namespace

size_t larosa_offline_workspace_bytes(int d, larosa_dtype t) {
  if (d < 8 || !dtype_ok(t)) return 0;
  return 2 * terms_bytes(d, t == LAROSA_BF16);
}

int larosa_second_moment(const void* X, int n_tokens, int d, larosa_dtype t, float* C, int accumulate,
                         void* stream) {
  if (int rc = check_offline(X, X, C, d, t)) return rc;
  if (n_tokens < 1) return LAROSA_EINVAL;
  ContractionArgs a{};
  a.A = a.B = static_cast<const uint16_t*>(X);
  a.M = a.N = d; a.Kd = n_tokens;
  a.npairs = 1;
  a.C32 = C;
  a.post_scale = 1.0f;
  a.accumulate = accumulate ? 1 : 0;
  a.symmetric = 1;
  return launch_contraction(a, true, t == LAROSA_BF16, static_cast<hipStream_t>(stream)) == hipSuccess ? LAROSA_OK
                                                                                                       : LAROSA_EHIP;
}

int larosa_fold_input(const float* Q, const void* W, int d, int d_out, larosa_dtype t, void* W_out, void* ws,
                      size_t ws_bytes, void* stream) {
  if (int rc = check_offline(Q, W, W_out, d, t)) return rc;
  if (d_out < 8 || d_out % 8 || W == W_out) return LAROSA_EINVAL;
  const bool bf16 = t == LAROSA_BF16;
  if (!ws || !aligned(ws, 256) || ws_bytes < terms_bytes(d, bf16)) return LAROSA_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  uint16_t* terms = static_cast<uint16_t*>(ws);
  const long n = static_cast<long>(d) * d;
  if (launch_split_terms(Q, terms, n, term_pre_scale(bf16), bf16, st) != hipSuccess) return LAROSA_EHIP;
  ContractionArgs a{};
  a.A = terms; a.B = static_cast<const uint16_t*>(W);
  a.M = d; a.N = d_out; a.Kd = d;
  a.a_term_stride = n;
  a.npairs = contraction_terms(bf16);
  for (int i = 0; i < a.npairs; ++i) { a.pa[i] = i; a.pb[i] = 0; }
  a.C16 = static_cast<uint16_t*>(W_out);
  a.post_scale = 1.0f / term_pre_scale(bf16);
  return launch_contraction(a, true, bf16, st) == hipSuccess ? LAROSA_OK : LAROSA_EHIP;
}

int larosa_fold_output(const void* W, const float* Q, int d_in, int d, larosa_dtype t, void* W_out, void* ws,
                       size_t ws_bytes, void* stream) {
  if (int rc = check_offline(Q, W, W_out, d, t)) return rc;
  if (d_in < 8 || d_in % 8 || W == W_out) return LAROSA_EINVAL;
  const bool bf16 = t == LAROSA_BF16;
  if (!ws || !aligned(ws, 256) || ws_bytes < terms_bytes(d, bf16)) return LAROSA_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  uint16_t* terms = static_cast<uint16_t*>(ws);
  const long n = static_cast<long>(d) * d;
  if (launch_split_terms(Q, terms, n, term_pre_scale(bf16), bf16, st) != hipSuccess) return LAROSA_EHIP;
  ContractionArgs a{};
  a.A = static_cast<const uint16_t*>(W); a.B = terms;
  a.M = d_in; a.N = d; a.Kd = d;
  a.b_term_stride = n;
  a.npairs = contraction_terms(bf16);
  for (int i = 0; i < a.npairs; ++i) { a.pa[i] = 0; a.pb[i] = i; }
  a.C16 = static_cast<uint16_t*>(W_out);
  a.post_scale = 1.0f / term_pre_scale(bf16);
  return launch_contraction(a, false, bf16, st) == hipSuccess ? LAROSA_OK : LAROSA_EHIP;
}

int larosa_residual_adapter(const float* Q_l, const float* Q_next, int d, larosa_dtype t, void* A_out, void* ws,
                            size_t ws_bytes, void* stream) {
  if (int rc = check_offline(Q_l, Q_next, A_out, d, t)) return rc;
  const bool bf16 = t == LAROSA_BF16;
  const size_t tb = terms_bytes(d, bf16);
  if (!ws || !aligned(ws, 256) || ws_bytes < 2 * tb) return LAROSA_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  uint16_t* ta = static_cast<uint16_t*>(ws);
  uint16_t* tb16 = reinterpret_cast<uint16_t*>(static_cast<char*>(ws) + tb);
  const long n = static_cast<long>(d) * d;
  const float pre = term_pre_scale(bf16);
  if (launch_split_terms(Q_l, ta, n, pre, bf16, st) != hipSuccess) return LAROSA_EHIP;
  if (launch_split_terms(Q_next, tb16, n, pre, bf16, st) != hipSuccess) return LAROSA_EHIP;
  ContractionArgs a{};
  a.A = ta; a.B = tb16;
  a.M = a.N = a.Kd = d;
  a.a_term_stride = a.b_term_stride = n;
  // every product of terms whose combined weight is above the fp32 rounding of the full product
  static const int f16_pairs[3][2] = {{0, 0}, {0, 1}, {1, 0}};
  static const int bf16_pairs[6][2] = {{0, 0}, {0, 1}, {1, 0}, {1, 1}, {0, 2}, {2, 0}};
  a.npairs = bf16 ? 6 : 3;
  for (int i = 0; i < a.npairs; ++i) {
    a.pa[i] = bf16 ? bf16_pairs[i][0] : f16_pairs[i][0];
    a.pb[i] = bf16 ? bf16_pairs[i][1] : f16_pairs[i][1];
  }
  a.C16 = static_cast<uint16_t*>(A_out);
  a.post_scale = 1.0f / (pre * pre);
  return launch_contraction(a, true, bf16, st) == hipSuccess ? LAROSA_OK : LAROSA_EHIP;
}

// ---- 4-bit weights and the threshold sparsifier ------------------------------------------------

int larosa_quantize_w4(const void* W, int d_in, int d_out, larosa_dtype t, void* Wq, void* scales, void* stream) {
  if (!W || !Wq || !scales || !dtype_ok(t)) return LAROSA_EINVAL;
  if (!aligned(W, 16) || !aligned(Wq, 16) || !aligned(scales, 2)) return LAROSA_EINVAL;
  if (d_in < 1 || d_in > 65535 || d_out < 8 || d_out % 8) return LAROSA_EINVAL;
  return launch_quantize_w4(static_cast<const uint16_t*>(W), d_in, d_out, static_cast<uint32_t*>(Wq),
                            static_cast<uint16_t*>(scales), t == LAROSA_BF16,
                            static_cast<hipStream_t>(stream)) == hipSuccess
             ? LAROSA_OK
             : LAROSA_EHIP;
}

int larosa_sparse_gemv_w4(const void* Wq, const void* scales, const void* h, const int32_t* idx, void* y, int B,
                          int d_in, int d_out, int K, larosa_dtype t, void* ws, size_t ws_bytes, void* stream) {
  if (!Wq || !scales || !h || !y || !dtype_ok(t)) return LAROSA_EINVAL;
  if (!aligned(Wq, 16) || !aligned(scales, 2) || !aligned(h, 16) || !aligned(y, 16) || (idx && !aligned(idx, 4)))
    return LAROSA_EINVAL;
  if (int rc = check_gemv_shapes(B, d_in, d_out, K)) return rc;
  if (!idx && K != d_in) return LAROSA_EINVAL;
  W4Args w{};
  GemvArgs& a = w.g;
  a.h = static_cast<const uint16_t*>(h);
  a.idx = idx;
  a.y = static_cast<uint16_t*>(y);
  a.d_in = d_in; a.d_out = d_out; a.K = K; a.B = B;
  w.Wq = static_cast<const uint32_t*>(Wq);
  w.scales = static_cast<const uint16_t*>(scales);
  w.ng = (d_out + 127) / 128;
  // the 2048-column geometry has a quarter of the strips: two workgroups per compute unit keep enough loads in
  // flight (70B gate|up: 47.1 us with 252 workgroups, 39.1 with 504)
  const int strip_cols = w4_strip_cols(d_out);
  const GemvPlan p = plan_gemv(d_out, K, strip_cols > 512 && tuning().g_target == 0 ? 512 : 0, strip_cols);
  if (static_cast<size_t>(B) * p.nstrips > kCounterSlots) return LAROSA_EUNSUPPORTED;
  const size_t need = kCounterBytes + static_cast<size_t>(B) * p.partial_floats * sizeof(float);
  if (!ws || !aligned(ws, 256) || ws_bytes < need) return LAROSA_EWORKSPACE;
  a.chunk = p.chunk; a.wps = p.wps; a.G = p.G; a.nstrips = p.nstrips;
  a.counters = static_cast<unsigned*>(ws);
  a.partial = reinterpret_cast<float*>(static_cast<char*>(ws) + kCounterBytes);
  return launch_gemv_w4(w, t == LAROSA_BF16, static_cast<hipStream_t>(stream)) == hipSuccess ? LAROSA_OK : LAROSA_EHIP;
}

int larosa_threshold_select(const void* h, int B, int d, float eps, larosa_dtype t, int32_t* idx, int32_t* count,
                            void* stream) {
  if (!h || !idx || !count || !dtype_ok(t)) return LAROSA_EINVAL;
  if (!aligned(h, 16) || !aligned(idx, 4) || !aligned(count, 4)) return LAROSA_EINVAL;
  if (B < 1 || d < 8 || d % 8 || !(eps >= 0.f)) return LAROSA_EINVAL;
  if (d > kMaxTopkD || B > 65535) return LAROSA_EUNSUPPORTED;
  return launch_threshold_select(static_cast<const uint16_t*>(h), B, d, eps, idx, count, t == LAROSA_BF16,
                                 static_cast<hipStream_t>(stream)) == hipSuccess
             ? LAROSA_OK
             : LAROSA_EHIP;
}

// ---- the entry point that allocates nothing ----------------------------------------------------

namespace {

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, looked up once per device

// Device address of this GPU's copy of the scratch array (the current device's), or nullptr.
void* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    scratch_ptr[dev] = p;
  }
  return scratch_ptr[dev];
}

}  // namespace

int larosa_sparse_gemv_static(const void* Wp, const void* h, const int32_t* idx, void* y, int B, int d_in,
                              int d_out, int K, larosa_dtype t, void* stream) {
  if (!Wp || !h || !idx || !y || !dtype_ok(t)) return LAROSA_EINVAL;
  if (int rc = check_gemv_shapes(B, d_in, d_out, K)) return rc;
  // the same scratch need as larosa_sparse_gemv's workspace, against the fixed size of the array
  size_t need;
  if (B > 1) {
    const GemvPlan p = plan_batched(d_in, d_out, batched_uses_mfma(B, false));
    need = round_up(kCounterBytes + batched_partial_bytes(p, B, false), 256) + static_cast<size_t>(B) * d_in * 2;
  } else {
    need = kCounterBytes + plan_gemv(d_out, K).partial_floats * sizeof(float);
  }
  if (need > LAROSA_STATIC_SCRATCH_BYTES) return LAROSA_EUNSUPPORTED;
  void* ws = static_scratch();
  if (!ws) return LAROSA_EHIP;
  // every call on a GPU shares the array: the counters must start at zero whatever the last call left
  if (launch_fill_u32(static_cast<unsigned*>(ws), kCounterWords, 0u, static_cast<hipStream_t>(stream)) != hipSuccess)
    return LAROSA_EHIP;
  const int rc = larosa_sparse_gemv(Wp, h, idx, y, B, d_in, d_out, K, t, ws, LAROSA_STATIC_SCRATCH_BYTES, stream);
  return rc == LAROSA_EWORKSPACE ? LAROSA_EUNSUPPORTED : rc;
}

int larosa_set_tuning(int key, int value) {
  switch (key) {
    case 0:
      if (value < 0 || value > 4096) return LAROSA_EINVAL;
      tuning().g_target = value;
      return LAROSA_OK;
    case 1:
      if (value < 1 || value > 1 << 20) return LAROSA_EINVAL;
      tuning().min_rows = value;
      return LAROSA_OK;
    case 2:
      if (value < 0 || value > 2) return LAROSA_EINVAL;
      tuning().variant = value;
      return LAROSA_OK;
    case 3:
      if (value < 0 || value > 1) return LAROSA_EINVAL;
      tuning().fused = value;
      return LAROSA_OK;
    case 5:
      if (value != 0 && (value < 8 || value > 2048)) return LAROSA_EINVAL;
      tuning().side_main_g = value;
      return LAROSA_OK;
    case 6:
      if (value != 0 && (value < 8 || value > 2048)) return LAROSA_EINVAL;
      tuning().side_g = value;
      return LAROSA_OK;
    case 7:
      if (value < 2048 || value > (1 << 30)) return LAROSA_EINVAL;
      tuning().w4_wide_min_cols = value;
      return LAROSA_OK;
    case 8:
      if (value < 8 || value > kMaxTopkD) return LAROSA_EINVAL;
      tuning().fused_max_width = value;
      return LAROSA_OK;
    case 9:
      if (value < 0 || value > 1) return LAROSA_EINVAL;
      tuning().hinted = value;
      return LAROSA_OK;
    case 10:
      if (value < 0 || value > 2) return LAROSA_EINVAL;
      tuning().contraction_tiles = value;
      return LAROSA_OK;
    default:
      return LAROSA_EINVAL;
  }
}

}  // extern "C"
