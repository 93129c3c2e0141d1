// Offline part of the method on the matrix cores (Sec. 4.2): the uncentred second moment X^T X of the
// calibration tokens, the folded weights Q^T W and W Q, and the residual adapters Q_l^T Q_{l+1}.
// All four are dense contractions  C[m,n] = sum_k A(k,m) B(k,n)  and share one kernel.
//
//  * v_mfma_f32_32x32x16 (f16 / bf16 inputs, fp32 accumulate).  A workgroup of 4 waves owns a 128 x 128
//    tile of C, each wave a 64 x 64 quarter (2 x 2 instruction tiles, 64 accumulator registers).
//  * Operands are stored k-major ([k][m], the layout of X, Q and W), the instruction wants 8 values
//    along k per lane.  The transposition happens on the way into LDS: a lane loads 8 consecutive
//    columns of two neighbouring k rows, pairs them into dwords (k, k+1) and writes them to a tile
//    held as [column][k-pair] with an odd row stride (17 dwords), which makes both the transposing
//    writes and the operand reads bank-conflict free.  The k-contiguous operand of W Q is copied as is.
//  * A rotation comes from an eigen-solver in fp32 or better; rounding it to 16 bits before the
//    product would cost more than the 16-bit rounding of the folded weight itself.  It is therefore
//    split into 2 (f16) or 3 (bf16) 16-bit terms whose sum carries the fp32 value, and the kernel
//    adds the products of the listed term pairs into the same accumulators.
//  * 32 concurrent workgroups of an XCD (workgroup i runs on XCD i % 8) form a 4 x 8 patch of tiles,
//    so the operand panels they stream are shared through that XCD's L2.
//  * X^T X is symmetric: only tiles on or above the diagonal are computed and each is stored twice.
#include "kernels.hpp"
#include "numeric.hpp"

namespace larosa {

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bfloat8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kTile = 128;         // C tile edge per workgroup
constexpr int kKTile = 32;         // k rows per LDS stage
constexpr int kRowDwords = 17;     // 16 k-pairs + 1 pad: odd stride
constexpr int kTileDwords = kTile * kRowDwords;
constexpr int kPatchM = 4, kPatchN = 8;

template <typename T> struct Mfma;
template <> struct Mfma<F16> {
  static __device__ __forceinline__ float16v run(u32x4 a, u32x4 b, float16v c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
  }
};
template <> struct Mfma<BF16> {
  static __device__ __forceinline__ float16v run(u32x4 a, u32x4 b, float16v c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bfloat8, a), __builtin_bit_cast(bfloat8, b), c, 0, 0,
                                                   0);
  }
};

// Registers of one thread for one operand tile in flight.
struct Staged {
  uint4 r0, r1;
};

// k-major source P[k][ld]: rows k0 + 2 kp, k0 + 2 kp + 1, columns c0 + 8 g .. + 7.
__device__ __forceinline__ Staged load_kmajor(const uint16_t* __restrict__ P, long ld, int k0, int Kd, int c0, int cols,
                                              int g, int kp) {
  Staged s;
  s.r0 = make_uint4(0, 0, 0, 0);
  s.r1 = s.r0;
  const int c = c0 + 8 * g;
  const int k = k0 + 2 * kp;
  if (c < cols) {
    if (k < Kd) s.r0 = *reinterpret_cast<const uint4*>(P + static_cast<long>(k) * ld + c);
    if (k + 1 < Kd) s.r1 = *reinterpret_cast<const uint4*>(P + static_cast<long>(k + 1) * ld + c);
  }
  return s;
}

__device__ __forceinline__ void store_kmajor(uint32_t* tile, const Staged& s, int g, int kp) {
  const uint32_t a[4] = {s.r0.x, s.r0.y, s.r0.z, s.r0.w};
  const uint32_t b[4] = {s.r1.x, s.r1.y, s.r1.z, s.r1.w};
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    tile[(8 * g + 2 * q) * kRowDwords + kp] = (a[q] & 0xFFFFu) | (b[q] << 16);
    tile[(8 * g + 2 * q + 1) * kRowDwords + kp] = (a[q] >> 16) | (b[q] & 0xFFFF0000u);
  }
}

// k-contiguous source P[m][ld]: two 16-byte pieces per thread (items t and t + 256 of 128 rows x 4).
__device__ __forceinline__ Staged load_kcontig(const uint16_t* __restrict__ P, long ld, int k0, int Kd, int m0, int rows,
                                               int t) {
  Staged s;
  s.r0 = make_uint4(0, 0, 0, 0);
  s.r1 = s.r0;
  const int kq = t & 3;
  const int k = k0 + 8 * kq;
  const int ma = m0 + (t >> 2), mb = ma + 64;
  if (k < Kd) {
    if (ma < rows) s.r0 = *reinterpret_cast<const uint4*>(P + static_cast<long>(ma) * ld + k);
    if (mb < rows) s.r1 = *reinterpret_cast<const uint4*>(P + static_cast<long>(mb) * ld + k);
  }
  return s;
}

__device__ __forceinline__ void store_kcontig(uint32_t* tile, const Staged& s, int t) {
  const int kq = t & 3;
  uint32_t* pa = tile + (t >> 2) * kRowDwords + 4 * kq;
  uint32_t* pb = pa + 64 * kRowDwords;
  pa[0] = s.r0.x; pa[1] = s.r0.y; pa[2] = s.r0.z; pa[3] = s.r0.w;
  pb[0] = s.r1.x; pb[1] = s.r1.y; pb[2] = s.r1.z; pb[3] = s.r1.w;
}

__device__ __forceinline__ u32x4 read_operand(const uint32_t* tile, int row, int dword0) {
  const uint32_t* p = tile + row * kRowDwords + dword0;
  u32x4 v;
  v.x = p[0]; v.y = p[1]; v.z = p[2]; v.w = p[3];
  return v;
}

template <typename T, bool A_KMAJOR>
__global__ __launch_bounds__(256) void contraction_kernel(ContractionArgs a) {
  __shared__ uint32_t lds[2][2][kTileDwords];   // [buffer][A | B]

  // workgroup -> tile: 32 consecutive workgroups of one XCD take one 4 x 8 patch of tiles
  const int xcd = blockIdx.x & 7;
  const int local = blockIdx.x >> 3;
  const int patch = (local >> 5) * 8 + xcd;
  const int within = local & 31;
  if (patch >= a.patches_m * a.patches_n) return;
  const int tm = (patch / a.patches_n) * kPatchM + (within >> 3);
  const int tn = (patch % a.patches_n) * kPatchN + (within & 7);
  if (tm >= a.tiles_m || tn >= a.tiles_n) return;
  if (a.symmetric && tn < tm) return;
  const int m0 = tm * kTile, n0 = tn * kTile;

  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int g = (lane & 7) + 8 * (w & 1);
  const int kp = (lane >> 3) + 8 * (w >> 1);
  const int wm = w >> 1, wn = w & 1;

  float16v acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  const int ktiles = (a.Kd + kKTile - 1) / kKTile;
  const int iters = ktiles * a.npairs;

  auto fetch = [&](int it, Staged& sa, Staged& sb) {
    const int p = it / ktiles;
    const int k0 = (it - p * ktiles) * kKTile;
    const uint16_t* Ap = a.A + a.pa[p] * a.a_term_stride;
    const uint16_t* Bp = a.B + a.pb[p] * a.b_term_stride;
    if (A_KMAJOR)
      sa = load_kmajor(Ap, a.M, k0, a.Kd, m0, a.M, g, kp);
    else
      sa = load_kcontig(Ap, a.Kd, k0, a.Kd, m0, a.M, t);
    sb = load_kmajor(Bp, a.N, k0, a.Kd, n0, a.N, g, kp);
  };
  auto stash = [&](int buf, const Staged& sa, const Staged& sb) {
    if (A_KMAJOR)
      store_kmajor(lds[buf][0], sa, g, kp);
    else
      store_kcontig(lds[buf][0], sa, t);
    store_kmajor(lds[buf][1], sb, g, kp);
  };

  Staged sa, sb;
  fetch(0, sa, sb);
  stash(0, sa, sb);
  __syncthreads();
  for (int it = 0; it < iters; ++it) {
    const int buf = it & 1;
    const bool more = it + 1 < iters;
    if (more) fetch(it + 1, sa, sb);
    const uint32_t* At = lds[buf][0];
    const uint32_t* Bt = lds[buf][1];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int dw = s * 8 + (lane >> 5) * 4;
      u32x4 av[2], bv[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        av[i] = read_operand(At, wm * 64 + i * 32 + (lane & 31), dw);
        bv[i] = read_operand(Bt, wn * 64 + i * 32 + (lane & 31), dw);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = Mfma<T>::run(av[i], bv[j], acc[i][j]);
    }
    if (more) stash(buf ^ 1, sa, sb);
    __syncthreads();
  }

  // accumulator register r of lane l: row 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32
  const bool mirror = a.symmetric && tn != tm;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int n = n0 + wn * 64 + j * 32 + (lane & 31);
      if (n >= a.N) continue;
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int mb = m0 + wm * 64 + i * 32 + 8 * r4 + 4 * (lane >> 5);
        float v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = acc[i][j][r4 * 4 + q] * a.post_scale;
        if (a.C16) {
#pragma unroll
          for (int q = 0; q < 4; ++q)
            if (mb + q < a.M) a.C16[static_cast<long>(mb + q) * a.N + n] = T::from_f32(v[q]);
        } else {
#pragma unroll
          for (int q = 0; q < 4; ++q)
            if (mb + q < a.M) {
              float* c = a.C32 + static_cast<long>(mb + q) * a.N + n;
              const float o = a.accumulate ? *c + v[q] : v[q];
              *c = o;
              v[q] = o;
            }
          if (mirror && mb < a.M) {        // M % 4 == 0: the four rows are valid together
            float4 o4 = make_float4(v[0], v[1], v[2], v[3]);
            *reinterpret_cast<float4*>(a.C32 + static_cast<long>(n) * a.N + mb) = o4;
          }
        }
      }
    }
}

// fp32 -> NT 16-bit terms with x * pre_scale = t0 + t1 (+ t2) up to the last term's rounding.
template <typename T, int NT>
__global__ __launch_bounds__(256) void split_terms_kernel(const float* __restrict__ src, uint16_t* __restrict__ dst, long n,
                                                          float pre_scale) {
  const long i = static_cast<long>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= n) return;
  float r = src[i] * pre_scale;
#pragma unroll
  for (int s = 0; s < NT; ++s) {
    const uint16_t b = T::from_f32(r);
    dst[s * n + i] = b;
    r -= T::to_f32(b);
  }
}

}  // namespace

int contraction_terms(bool bf16) { return bf16 ? 3 : 2; }

hipError_t launch_split_terms(const float* src, uint16_t* dst, long n, float pre_scale, bool bf16, hipStream_t s) {
  const unsigned grid = static_cast<unsigned>((n + 255) / 256);
  if (bf16)
    hipLaunchKernelGGL((split_terms_kernel<BF16, 3>), dim3(grid), dim3(256), 0, s, src, dst, n, pre_scale);
  else
    hipLaunchKernelGGL((split_terms_kernel<F16, 2>), dim3(grid), dim3(256), 0, s, src, dst, n, pre_scale);
  return hipGetLastError();
}

hipError_t launch_contraction(ContractionArgs a, bool a_kmajor, bool bf16, hipStream_t s) {
  a.tiles_m = (a.M + kTile - 1) / kTile;
  a.tiles_n = (a.N + kTile - 1) / kTile;
  a.patches_m = (a.tiles_m + kPatchM - 1) / kPatchM;
  a.patches_n = (a.tiles_n + kPatchN - 1) / kPatchN;
  const long patches = static_cast<long>(a.patches_m) * a.patches_n;
  const long grid = (patches + 7) / 8 * 8 * 32;
  if (grid > 0x7FFFFFFFL) return hipErrorInvalidValue;
  dim3 gd(static_cast<unsigned>(grid)), bd(256);
  if (bf16) {
    if (a_kmajor)
      hipLaunchKernelGGL((contraction_kernel<BF16, true>), gd, bd, 0, s, a);
    else
      hipLaunchKernelGGL((contraction_kernel<BF16, false>), gd, bd, 0, s, a);
  } else {
    if (a_kmajor)
      hipLaunchKernelGGL((contraction_kernel<F16, true>), gd, bd, 0, s, a);
    else
      hipLaunchKernelGGL((contraction_kernel<F16, false>), gd, bd, 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace larosa
