/*
 * liblarosa -- decode-time hot path of LaRoSA (layerwise rotated sparse activation,
 * arXiv 2507.01299) for one AMD MI355X (gfx950).
 *
 * Per token and per projection the method computes  y = S_k(x Q) (W Q)^T  (Sec. 4.3,
 * Eq. 9-10): rotate the block input with the layer's orthogonal matrix Q, keep the k
 * entries of largest magnitude (Eq. 8), and multiply by the folded weight, of which only
 * the k kept input channels are read (Sec. 4.4).
 *
 * Conventions common to every entry point
 *  - Every data pointer is a DEVICE pointer owned by the caller.  The library allocates
 *    nothing, frees nothing, and never synchronises: all work is enqueued on `stream`
 *    (a hipStream_t passed as void*; NULL = the default stream).
 *  - 16-bit tensors are IEEE binary16 (LAROSA_F16) or bfloat16 (LAROSA_BF16), row-major,
 *    with fp32 accumulation inside the kernels and one round-to-nearest-even at each store.
 *  - A folded weight W' is stored input-channel-major: row-major [d_in][d_out], so that
 *    input channel i owns one contiguous run of d_out values (Sec. 4.4, point 1: the
 *    "column-major" layout of the [d_out][d_in] linear-layer weight).
 *  - Data pointers must be 16-byte aligned; d_out and d must be multiples of 8.
 *  - Scratch memory comes from the caller's workspace `ws` (256-byte aligned) of at least
 *    the number of bytes the matching *_workspace_bytes() query returns.  A workspace must
 *    be passed once through larosa_workspace_init() after allocation (it zeroes the
 *    arrival counters at its head; the kernels leave them zero again on exit).
 *    One workspace serves one stream: two calls that use the same workspace must be ordered on
 *    one stream (calls that overlap on one workspace corrupt each other's partial sums and
 *    counters, silently).
 *  - Return value: LAROSA_OK (0) or a negative larosa_status.  Invalid arguments are
 *    rejected before anything is enqueued.  LAROSA_EHIP reports a failed launch
 *    (hipGetLastError() != hipSuccess after enqueueing).  After LAROSA_EHIP -- or after any
 *    launch that was aborted or faulted -- the arrival counters of the workspace may be left
 *    non-zero: pass it through larosa_workspace_init() again before the next call.
 *  - Index values (idx) are not range-checked: an index outside [0, d_in) reads outside Wp.
 */
#ifndef LAROSA_H
#define LAROSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { LAROSA_F16 = 0, LAROSA_BF16 = 1 } larosa_dtype;

typedef enum {
  LAROSA_OK = 0,
  LAROSA_EINVAL = -1,       /* null pointer, size out of range, misalignment, unknown dtype */
  LAROSA_EUNSUPPORTED = -2, /* valid request outside what the kernels cover (e.g. d > 32768 in Top-K) */
  LAROSA_EWORKSPACE = -3,   /* workspace missing, misaligned or too small */
  LAROSA_EHIP = -4          /* the HIP runtime reported an error at launch */
} larosa_status;

/* Static, NUL-terminated description of a status code.  Never NULL. */
const char* larosa_status_string(int status);

/* Library version: major*10000 + minor*100 + patch. */
int larosa_version(void);

/* Bytes of workspace that larosa_rotate / larosa_topk / larosa_sparse_gemv need for B tokens
 * with input width <= d_in_max, output width <= d_out_max and kept count <= K_max.
 * Pure host function (no device access).  Returns 0 for non-positive arguments. */
size_t larosa_workspace_bytes(int B, int d_in_max, int d_out_max, int K_max);

/* Zero the arrival counters at the head of a freshly allocated workspace (device pointer,
 * >= larosa_workspace_bytes(1,8,8,1) bytes).  Enqueued on `stream` as a fill kernel. */
int larosa_workspace_init(void* ws, size_t ws_bytes, void* stream);

/* Rotation (Sec. 4.3: the rotated activation x Q; App. A: h_i = sum_j x_j Q_ji).
 *   h[b,i] = sum_j x[b,j] * Q[j,i]
 * x [B,d], Q [d,d] row-major (row j = input channel j; column i = i-th principal direction),
 * h [B,d].  Also serves the residual adapter x (Q_l^T Q_{l+1}) (Sec. 4.2) and, being a dense
 * mat-vec over an input-channel-major matrix, the dense comparator (larosa_dense_gemv is the
 * same operation with a rectangular matrix). */
int larosa_rotate(const void* x, const void* Q, void* h, int B, int d, larosa_dtype t,
                  void* ws, size_t ws_bytes, void* stream);

/* Dense product over an input-channel-major matrix:  y[b,o] = sum_j x[b,j] * Wp[j,o].
 * x [B,d_in], Wp [d_in,d_out], y [B,d_out].  (Eq. 1 with the stored layout; the K = d_in
 * special case of the sparse projection, used as the dense baseline on the same GPU.) */
int larosa_dense_gemv(const void* Wp, const void* x, void* y, int B, int d_in, int d_out,
                      larosa_dtype t, void* ws, size_t ws_bytes, void* stream);

/* Top-K sparsifier S_k (Sec. 4.3, Eq. 8): for each token b, the K indices of largest |h[b,:]|.
 * Magnitudes are compared on the stored 16-bit values (sign bit cleared, bit pattern as an
 * unsigned integer); ties go to the larger magnitude, then to the lower index; exactly K
 * indices are produced, in ascending order.
 * h [B,d]; idx [B,K] int32 (output); vals [B,K] (output, nullable) receives h[b, idx[b,t]].
 * 1 <= K <= d <= 32768.  ws / ws_bytes are not used (the selection needs no scratch in device
 * memory; the arguments keep the signature uniform) and may be NULL / 0. */
int larosa_topk(const void* h, int B, int d, int K, int32_t* idx, void* vals,
                larosa_dtype t, void* ws, size_t ws_bytes, void* stream);

/* Column-sparse projection (Sec. 4.3, Eq. 10; Sec. 4.4 point 3):
 *   y[b,o] = sum_{t<K} h[b, idx[b,t]] * Wp[idx[b,t], o]
 * Only the rows of Wp named by idx are read.  Wp [d_in,d_out] input-channel-major,
 * h [B,d_in], idx [B,K] int32 with 0 <= idx < d_in (per-token index sets; need not be sorted,
 * must not repeat within a token), y [B,d_out] (output). */
int larosa_sparse_gemv(const void* Wp, const void* h, const int32_t* idx, void* y,
                       int B, int d_in, int d_out, int K, larosa_dtype t,
                       void* ws, size_t ws_bytes, void* stream);

/* larosa_sparse_gemv for callers that cannot allocate device memory or bring a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments
 * without `ws`, same kernels, same result bit for bit.  The arrival counters and partial strips
 * live in a device array of LAROSA_STATIC_SCRATCH_BYTES inside the library (one copy per GPU,
 * held until the process ends); the call allocates and frees nothing.  A request whose scratch
 * need exceeds that size returns LAROSA_EUNSUPPORTED and enqueues nothing (batch 1 always fits
 * for d_out <= 262144; for B > 1 the need is that of larosa_workspace_bytes(B, d_in, d_out, K)).
 * The array's address is looked up on the first call on each device (a host-side query, no
 * stream work).  The counters are zeroed by a fill kernel at the start of every call, so the
 * state a previous call left is irrelevant; every call on one GPU shares the one array, so two
 * calls that overlap on that GPU (different streams) race: order them on one stream. */
#define LAROSA_STATIC_SCRATCH_BYTES (8u << 20)
int larosa_sparse_gemv_static(const void* Wp, const void* h, const int32_t* idx, void* y,
                              int B, int d_in, int d_out, int K, larosa_dtype t, void* stream);

/* One decoder layer (Fig. 2; Sec. 3.1 for h1..h4; Sec. 4.2-4.3).  All pointers device, borrowed
 * for the duration of the call. */
typedef struct {
  int d, d_q, d_kv, d_ff;     /* hidden, q/o width, k/v width, intermediate */
  int head_dim;               /* d_q and d_kv are multiples of it; (d_q/head_dim) % (d_kv/head_dim) == 0 */
  int K1, K2, K3, K4;         /* kept counts for h1 (d), h2 (d_q), h3 (d), h4 (d_ff) */
  const void* Wqkv;           /* [d, d_q+2*d_kv]  q|k|v, folded with Q^T on the input side when h1 is rotated */
  const void* Wo;             /* [d_q, d]         meets the unrotated h2 (Q = I, Sec. 4.3) */
  const void* Wgu;            /* [d, 2*d_ff]      gate|up, folded like Wqkv */
  const void* Wdown;          /* [d_ff, d]        meets the unrotated h4 */
  const void* Q_attn;         /* [d,d] or NULL: NULL = x already arrives in the layer's basis (folded form) */
  const void* Q_mlp;          /* [d,d] or NULL */
  const void* adapter;        /* [d,d] Q_l^T Q_{l+1} applied to the layer output, or NULL */
  const void* rms_attn;       /* [d] pre-norm scale or NULL = 1 */
  const void* rms_mlp;        /* [d] or NULL */
  float rms_eps;              /* < 0 disables both pre-norms */
  int attn_mode;              /* 0: context-length-1 attention (softmax over one key = 1, so each query
                                    head outputs the value head of its group); must be 0.  A caller with an
                                    attention core of its own uses larosa_layer_qkv and
                                    larosa_layer_after_attention instead of larosa_layer_forward. */
  larosa_dtype dtype;
  /* Residual adapters on the two shortcuts (Sec. 4.2; with block-level rotations, Sec. 5.4, there is
   * one per block), each [d,d] or NULL = identity: the stream that skips the attention block is taken
   * through shortcut_attn (Q_attn^T Q_mlp when Wo was folded with Q_mlp on its output side), the one
   * that skips the MLP block through shortcut_mlp (Q_mlp^T Q_next with Wdown folded with Q_next).
   * They depend only on the block's input, so they run beside the block's first projection. */
  const void* shortcut_attn;
  const void* shortcut_mlp;
} larosa_layer;

/* Optional copies of every stage (device pointers, each nullable), for stage-by-stage checks:
 * h1 [B,d]; idx1 [B,K1]; qkv [B,d_q+2d_kv]; h2 [B,d_q]; idx2 [B,K2]; o [B,d]; x1 [B,d];
 * h3 [B,d]; idx3 [B,K3]; gu [B,2d_ff]; h4 [B,d_ff]; idx4 [B,K4]; down [B,d]; x2 [B,d];
 * s1, s2 [B,d]: the shortcut values (written only when the layer has that shortcut adapter). */
typedef struct {
  void *h1, *qkv, *h2, *o, *x1, *h3, *gu, *h4, *down, *x2;
  int32_t *idx1, *idx2, *idx3, *idx4;
  void *s1, *s2;
  /* Optional caller-created hipEvent_t handles (each nullable), recorded on `stream` at the stage
   * boundaries so a caller can time the stages of one call: [0] on entry, [1] after the h1 stage
   * (rotation / pre-norm), [2] after q|k|v, [3] after o, [4] after the h3 stage, [5] after gate|up,
   * [6] after down, [7] after the adapter.  Do not pass events while the stream is being captured. */
  void* stage_events[8];
} larosa_trace;

/* Workspace bytes larosa_layer_forward needs for this layer and B tokens (host only). */
size_t larosa_layer_workspace_bytes(const larosa_layer* L, int B);

/* x [B,d] -> x_out [B,d]:
 *   h1 = R(norm(x) Q_attn); qkv = R(S_K1(h1) Wqkv); h2 = attention core of qkv;
 *   o = R(S_K2(h2) Wo); x1 = R(s1 + o); h3 = R(norm(x1) Q_mlp); gu = R(S_K3(h3) Wgu);
 *   h4 = R(SiLU(gate) * up); down = R(S_K4(h4) Wdown); x2 = R(s2 + down);
 *   x_out = R(x2 adapter) or x2;  s1 = R(x shortcut_attn) or x;  s2 = R(x1 shortcut_mlp) or x1.
 *   R = one rounding to the layer dtype.
 * trace may be NULL.  x_out must not alias x. */
int larosa_layer_forward(const larosa_layer* L, const void* x, void* x_out, int B,
                         const larosa_trace* trace, void* ws, size_t ws_bytes, void* stream);

/* The same layer split around the caller's own attention core (KV cache, softmax: the method leaves it
 * unchanged and only sparsifies its output h2, Sec. 3.1).  Same workspace size, trace and errors as
 * larosa_layer_forward; each call writes only the trace fields of its own stages.
 *
 * larosa_layer_qkv: x [B,d] -> qkv [B, d_q+2*d_kv] = R(S_K1(h1) Wqkv), and, when the layer has
 * shortcut_attn, s1 [B,d] = R(x shortcut_attn) (required then; ignored and may be NULL otherwise).
 * trace->qkv and trace->s1 are not written (the caller has both).
 *
 * larosa_layer_after_attention: attn [B,d_q] is the attention core's output in the layer dtype and
 * takes the place of h2; residual [B,d] is what the attention block's output is added to: the layer
 * input x, or the s1 written by larosa_layer_qkv when the layer has shortcut_attn.  Runs
 * o = R(S_K2(attn) Wo); x1 = R(residual + o); then the MLP block and the adapter as above.
 * x_out must not alias residual. */
int larosa_layer_qkv(const larosa_layer* L, const void* x, void* qkv, void* s1, int B,
                     const larosa_trace* trace, void* ws, size_t ws_bytes, void* stream);
int larosa_layer_after_attention(const larosa_layer* L, const void* residual, const void* attn, void* x_out,
                                 int B, const larosa_trace* trace, void* ws, size_t ws_bytes, void* stream);

/* ---- Offline part on the GPU (Sec. 4.2: PCA rotation of each layer's input, rotation folded into the
 * neighbouring weights, residual adapter between consecutive layers).  The eigendecomposition itself
 * is left to the caller's solver: these calls produce its input and consume its output.
 * All pointers are device memory; matrices are dense row-major; d, d_in, d_out are multiples of 8;
 * 16-bit tensors are of type t; every call is asynchronous on `stream`.  Rotations are passed in fp32
 * and are NOT rounded to 16 bits before the products: they are split into 16-bit terms in `ws`
 * (borrowed for the duration of the call's kernels, 256-byte aligned).  Errors as for the calls above:
 * LAROSA_EINVAL for null/misaligned pointers or bad sizes, LAROSA_EWORKSPACE for a workspace that is
 * too small, LAROSA_EHIP when a launch fails. */

/* Bytes of workspace the three folding calls below need for d x d rotations of type t (host only). */
size_t larosa_offline_workspace_bytes(int d, larosa_dtype t);

/* Second-moment accumulation (Sec. 4.2): C (+)= X^T X for n_tokens calibration rows X [n_tokens, d]
 * (16-bit, type t), C [d, d] fp32, exactly symmetric.  accumulate = 0 overwrites C, 1 adds to it, so a
 * calibration set can be fed in batches; the caller divides by the token count if it wants the
 * average (the eigenvectors do not depend on it).  fp32 accumulation on the matrix cores. */
int larosa_second_moment(const void* X, int n_tokens, int d, larosa_dtype t, float* C, int accumulate,
                         void* stream);

/* Input-side fold (Sec. 4.2, Eq. 9-10): W_out = Q^T W for W [d, d_out] in the input-channel-major layout
 * the projections read, Q [d, d] fp32 with the principal directions as columns.  W_out [d, d_out] is
 * rounded once to type t.  W_out must not alias W. */
int larosa_fold_input(const float* Q, const void* W, int d, int d_out, larosa_dtype t, void* W_out, void* ws,
                      size_t ws_bytes, void* stream);

/* Output-side fold (Sec. 3.2): W_out = W Q for W [d_in, d]: the projection then emits its output in the
 * basis Q.  W_out [d_in, d], rounded once to type t, must not alias W. */
int larosa_fold_output(const void* W, const float* Q, int d_in, int d, larosa_dtype t, void* W_out, void* ws,
                       size_t ws_bytes, void* stream);

/* Residual adapter (Sec. 4.2): A = Q_l^T Q_next, [d, d], rounded once to type t: the dense mat-vec that
 * takes the residual stream from layer l's basis to the next layer's. */
int larosa_residual_adapter(const float* Q_l, const float* Q_next, int d, larosa_dtype t, void* A_out, void* ws,
                            size_t ws_bytes, void* stream);

/* ---- 4-bit weights (W4A16).  The paper reports that the method keeps its accuracy on round-to-nearest
 * and calibrated 4-bit weights (Sec. 5.4, Table 9) and names a kernel that does both as future work;
 * it fixes no storage format, so the one here is this library's own:
 *   Wq     [d_in, d_out/8] uint32: nibble k (bits 4k..4k+3) of dword m of row j = code q of column 8m+k
 *   scales [d_in, ceil(d_out/128)] 16-bit (type t): weight(j, o) = (q - 8) * scales[j, o/128]
 * i.e. symmetric codes with one scale per input-channel row and per group of 128 output columns, so
 * that a kept row is still one contiguous burst and its scales fold into the row's coefficient. */

/* Round-to-nearest quantisation of W [d_in, d_out] (16-bit, type t): scale = max|w| over the group / 7
 * rounded to type t, q = clip(rint(w / scale), -8, 7) + 8 (q = 8 where the scale is 0).
 * d_out % 8 == 0.  Device pointers, 16-byte aligned; asynchronous on `stream`. */
int larosa_quantize_w4(const void* W, int d_in, int d_out, larosa_dtype t, void* Wq, void* scales, void* stream);

/* Column-sparse projection (Sec. 4.3, Eq. 10) over the 4-bit weight:
 *   y[b,o] = sum_t h[b, idx[b,t]] * (q[idx[b,t], o] - 8) * scales[idx[b,t], o/128],  fp32 accumulate,
 * one rounding to type t.  idx as for larosa_sparse_gemv (ascending, distinct, per token), or NULL
 * with K == d_in for the dense product over all rows.  Workspace as for larosa_sparse_gemv. */
int larosa_sparse_gemv_w4(const void* Wq, const void* scales, const void* h, const int32_t* idx, void* y, int B,
                          int d_in, int d_out, int K, larosa_dtype t, void* ws, size_t ws_bytes, void* stream);

/* ---- Magnitude-threshold sparsifier S_eps (Eq. 4-5), the comparison method of Sec. 4.1 whose kept count
 * depends on the token: idx[b*d .. b*d + count[b]) = ascending channels with |h[b,i]| > eps (compared
 * exactly: 16-bit magnitudes widened to fp32 against the fp32 eps; NaN is dropped).
 * h [B, d] 16-bit, idx [B, d] int32 (capacity d per token), count [B] int32; device pointers;
 * d % 8 == 0, d <= 32768.  Feeding a token's idx and count[b] (read back by the caller) to
 * larosa_sparse_gemv gives the variable-K projection that the fixed-K Top-K path is compared with. */
int larosa_threshold_select(const void* h, int B, int d, float eps, larosa_dtype t, int32_t* idx, int32_t* count,
                            void* stream);

/* ---- NOT part of the stable interface: launch tuning for tests and experiments.
 * Process-wide host state read by every call (launch shapes AND workspace sizes depend on it): not
 * thread-safe; change it only while no call of this library is in flight, and before sizing a workspace.
 * Production callers never call it: the defaults are derived from the arguments of each call.
 * key 0 = target number of workgroups of the row-streaming kernels (0 = automatic),
 * key 1 = minimum kept rows per workgroup, key 2 = row-waves per workgroup of the stand-alone
 * row-streaming kernel (0: 8, 1: 16, 2: 4), key 3 = decoder layer with the Top-K fused into the
 * projection kernels (1, default) or as separate kernels (0),
 * key 5 / key 6 = workgroups of a projection / of the shortcut adapter that shares its launch
 * (0 = chosen from the two jobs' sizes, default),
 * key 7 = narrowest output width for which the 4-bit projection uses its 2048-column geometry,
 * key 8 = with key 9 = 0: widest MLP intermediate vector whose Top-K runs inside the down projection's
 * workgroups (wider ones are selected once by the Top-K kernel),
 * key 9 = batch-1 decoder layer: the down projection takes its Top-K threshold from key histograms
 * that the gate|up launch builds (1, default) or selects for itself (0),
 * key 10 = workgroup tile of the offline contractions: 0 = chosen by size (default), 1 = 256 x 128, 2 = 256 x 256.
 * Returns LAROSA_EINVAL for an unknown key or a value out of range. */
int larosa_set_tuning(int key, int value);

#ifdef __cplusplus
}
#endif
#endif /* LAROSA_H */
