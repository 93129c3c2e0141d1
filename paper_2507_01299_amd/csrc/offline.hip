// Offline part of the method on the matrix cores (Sec. 4.2): the uncentred second moment X^T X of the
// calibration tokens, the folded weights Q^T W and W Q, and the residual adapters Q_l^T Q_{l+1}.
// All four are dense contractions  C[m,n] = sum_k A(k,m) B(k,n)  and share one kernel.
//
//  * v_mfma_f32_32x32x16 (f16 / bf16 inputs, fp32 accumulate).  A workgroup of 4 waves owns a 256 x 128
//    tile of C, each wave a 128 x 64 quarter (4 x 2 instruction tiles, 128 accumulator registers): six
//    operand reads from LDS feed eight instructions.  The global loads of k-tile i + 2 are in flight
//    while tile i is multiplied and tile i + 1 moves from registers to the other LDS buffer.
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
//  * X^T X is symmetric: tiles that lie entirely below the diagonal are not computed; their elements are
//    stored by the tile that computes the mirrored position.
#include <type_traits>

#include "kernels.hpp"
#include "numeric.hpp"

namespace larosa {

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bfloat8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kTileM = 256;        // C tile of a workgroup: 256 rows (A columns) x TN columns, TN = 128 or 256
constexpr int kKTile = 32;         // k rows per LDS stage
constexpr int kRowDwords = 17;     // 16 k-pairs + 1 pad: odd stride
constexpr int kTileDwordsA = kTileM * kRowDwords;
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

// k-major source P[k][ld]: rows k0 + 2 kp, k0 + 2 kp + 1, columns c0 + 8 g .. + 7 -> r0, r1.
__device__ __forceinline__ void load_kmajor(const uint16_t* __restrict__ P, long ld, int k0, int Kd, int c0, int cols,
                                            int g, int kp, uint4& r0, uint4& r1) {
  r0 = make_uint4(0, 0, 0, 0);
  r1 = r0;
  const int c = c0 + 8 * g;
  const int k = k0 + 2 * kp;
  if (c < cols) {
    if (k < Kd) r0 = *reinterpret_cast<const uint4*>(P + static_cast<long>(k) * ld + c);
    if (k + 1 < Kd) r1 = *reinterpret_cast<const uint4*>(P + static_cast<long>(k + 1) * ld + c);
  }
}

__device__ __forceinline__ void store_kmajor(uint32_t* tile, const uint4& r0, const uint4& r1, int g, int kp) {
  const uint32_t a[4] = {r0.x, r0.y, r0.z, r0.w};
  const uint32_t b[4] = {r1.x, r1.y, r1.z, r1.w};
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    tile[(8 * g + 2 * q) * kRowDwords + kp] = (a[q] & 0xFFFFu) | (b[q] << 16);
    tile[(8 * g + 2 * q + 1) * kRowDwords + kp] = (a[q] >> 16) | (b[q] & 0xFFFF0000u);
  }
}

// k-contiguous source P[m][ld]: 16 bytes (8 k) of row m0 + row at k0 + 8 kq.
__device__ __forceinline__ uint4 load_kcontig(const uint16_t* __restrict__ P, long ld, int k0, int Kd, int m0, int rows,
                                              int row, int kq) {
  const int k = k0 + 8 * kq;
  const int m = m0 + row;
  if (k < Kd && m < rows) return *reinterpret_cast<const uint4*>(P + static_cast<long>(m) * ld + k);
  return make_uint4(0, 0, 0, 0);
}

__device__ __forceinline__ void store_kcontig(uint32_t* tile, const uint4& r, int row, int kq) {
  uint32_t* p = tile + row * kRowDwords + 4 * kq;
  p[0] = r.x; p[1] = r.y; p[2] = r.z; p[3] = r.w;
}

__device__ __forceinline__ u32x4 read_operand(const uint32_t* tile, int row, int dword0) {
  const uint32_t* p = tile + row * kRowDwords + dword0;
  u32x4 v;
  v.x = p[0]; v.y = p[1]; v.z = p[2]; v.w = p[3];
  return v;
}

// f(integral_constant<int, 0>), ..., f(integral_constant<int, N - 1>)
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (N > 0) {
    static_for<N - 1>(f);
    f(std::integral_constant<int, N - 1>{});
  }
}

// One k-tile of both operands in a thread's registers.
template <int TN>
struct Staged {
  uint4 a[4];
  uint4 b[TN / 64];
};

// Is the 256 x TN tile that holds element (row, col) left out of a symmetric product?
template <int TN>
__device__ __forceinline__ bool tile_skipped(int row, int col) {
  return TN * (col / TN + 1) <= kTileM * (row / kTileM);
}

// TN = 128 is the instantiated shape: 4 x 2 instruction tiles per wave, two workgroups per CU.
template <typename T, bool A_KMAJOR, int TN>
__global__ __launch_bounds__(256, TN == 128 ? 2 : 1) void contraction_kernel(ContractionArgs a) {
  constexpr int NJ = TN / 64;                    // instruction tiles of a wave along n
  constexpr int kTileN = TN;
  constexpr int kTileDwordsB = TN * kRowDwords;
  __shared__ uint32_t lds_a[2][kTileDwordsA];
  __shared__ uint32_t lds_b[2][kTileDwordsB];

  // workgroup -> tile: 32 consecutive workgroups of one XCD take one 4 x 8 patch of tiles
  const int xcd = blockIdx.x & 7;
  const int local = blockIdx.x >> 3;
  const int patch = (local >> 5) * 8 + xcd;
  const int within = local & 31;
  if (patch >= a.patches_m * a.patches_n) return;
  const int tm = (patch / a.patches_n) * kPatchM + (within >> 3);
  const int tn = (patch % a.patches_n) * kPatchN + (within & 7);
  if (tm >= a.tiles_m || tn >= a.tiles_n) return;
  const int m0 = tm * kTileM, n0 = tn * kTileN;
  if (a.symmetric && tile_skipped<TN>(m0, n0)) return;

  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int g = (lane & 7) + 8 * (w & 1);
  const int kp = (lane >> 3) + 8 * (w >> 1);
  const int wm = w >> 1, wn = w & 1;    // wave tile: rows wm * 128 .. + 127, columns wn * TN/2 .. + TN/2 - 1

  float16v acc[4][NJ];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  const int ktiles = (a.Kd + kKTile - 1) / kKTile;
  const int iters = ktiles * a.npairs;

  auto fetch = [&](int it, Staged<TN>& st) {
    const int p = it / ktiles;
    const int k0 = (it - p * ktiles) * kKTile;
    const uint16_t* Ap = a.A + a.pa[p] * a.a_term_stride;
    const uint16_t* Bp = a.B + a.pb[p] * a.b_term_stride;
    if (A_KMAJOR) {
      load_kmajor(Ap, a.M, k0, a.Kd, m0, a.M, g, kp, st.a[0], st.a[1]);
      load_kmajor(Ap, a.M, k0, a.Kd, m0, a.M, g + 16, kp, st.a[2], st.a[3]);
    } else {
#pragma unroll
      for (int r = 0; r < 4; ++r) st.a[r] = load_kcontig(Ap, a.Kd, k0, a.Kd, m0, a.M, (t >> 2) + 64 * r, t & 3);
    }
    load_kmajor(Bp, a.N, k0, a.Kd, n0, a.N, g, kp, st.b[0], st.b[1]);
    if (TN == 256) load_kmajor(Bp, a.N, k0, a.Kd, n0, a.N, g + 16, kp, st.b[NJ - 2], st.b[NJ - 1]);
  };
  auto stash = [&](int buf, const Staged<TN>& st) {
    if (A_KMAJOR) {
      store_kmajor(lds_a[buf], st.a[0], st.a[1], g, kp);
      store_kmajor(lds_a[buf], st.a[2], st.a[3], g + 16, kp);
    } else {
#pragma unroll
      for (int r = 0; r < 4; ++r) store_kcontig(lds_a[buf], st.a[r], (t >> 2) + 64 * r, t & 3);
    }
    store_kmajor(lds_b[buf], st.b[0], st.b[1], g, kp);
    if (TN == 256) store_kmajor(lds_b[buf], st.b[NJ - 2], st.b[NJ - 1], g + 16, kp);
  };
  auto compute = [&](int buf) {
    const uint32_t* At = lds_a[buf];
    const uint32_t* Bt = lds_b[buf];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int dw = s * 8 + (lane >> 5) * 4;
      u32x4 av[4], bv[NJ];
#pragma unroll
      for (int i = 0; i < 4; ++i) av[i] = read_operand(At, wm * 128 + i * 32 + (lane & 31), dw);
#pragma unroll
      for (int j = 0; j < NJ; ++j) bv[j] = read_operand(Bt, wn * (TN / 2) + j * 32 + (lane & 31), dw);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[i][j] = Mfma<T>::run(av[i], bv[j], acc[i][j]);
    }
  };

  // Tile it is computed from LDS buffer it & 1 while the loads of tile it + 2 are in flight and tile
  // it + 1 (loaded one step earlier) moves from registers to the other buffer: one barrier per tile.
  Staged<TN> s0, s1;
  fetch(0, s0);
  stash(0, s0);
  if (iters > 1) fetch(1, s1);
  __syncthreads();
  for (int it = 0; it < iters; it += 2) {
    if (it + 2 < iters) fetch(it + 2, s0);
    compute(0);
    if (it + 1 < iters) stash(1, s1);
    __syncthreads();
    if (it + 1 < iters) {
      if (it + 3 < iters) fetch(it + 3, s1);
      compute(1);
      if (it + 2 < iters) stash(0, s0);
      __syncthreads();
    }
  }

  // accumulator register r of lane l: row 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32.
  // The tile indices are compile-time constants (static_for): a run-time index into the accumulator
  // array would move all of it to scratch memory.
  static_for<4 * NJ>([&](auto ij) {
    constexpr int i = decltype(ij)::value / NJ;
    constexpr int j = decltype(ij)::value % NJ;
    const int n = n0 + wn * (TN / 2) + j * 32 + (lane & 31);
    if (n < a.N) {
      static_for<4>([&](auto r4c) {
        constexpr int r4 = decltype(r4c)::value;
        const int mb = m0 + wm * 128 + i * 32 + 8 * r4 + 4 * (lane >> 5);
        float v[4] = {acc[i][j][r4 * 4 + 0] * a.post_scale, acc[i][j][r4 * 4 + 1] * a.post_scale,
                      acc[i][j][r4 * 4 + 2] * a.post_scale, acc[i][j][r4 * 4 + 3] * a.post_scale};
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
          // element (n, mb .. mb + 3) of a symmetric product, when the tile it falls in is not computed
          // (M % 4 == 0 and mb % 4 == 0: the four are valid together and share a tile)
          if (a.symmetric && mb < a.M && tile_skipped<TN>(n, mb)) {
            float4 o4 = make_float4(v[0], v[1], v[2], v[3]);
            *reinterpret_cast<float4*>(a.C32 + static_cast<long>(n) * a.N + mb) = o4;
          }
        }
      });
    }
  });
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

namespace {

template <typename T, bool A_KMAJOR, int TN>
hipError_t launch_tiles(ContractionArgs a, hipStream_t s) {
  a.tiles_m = (a.M + kTileM - 1) / kTileM;
  a.tiles_n = (a.N + TN - 1) / TN;
  a.patches_m = (a.tiles_m + kPatchM - 1) / kPatchM;
  a.patches_n = (a.tiles_n + kPatchN - 1) / kPatchN;
  const long patches = static_cast<long>(a.patches_m) * a.patches_n;
  const long grid = (patches + 7) / 8 * 8 * 32;
  if (grid > 0x7FFFFFFFL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((contraction_kernel<T, A_KMAJOR, TN>), dim3(static_cast<unsigned>(grid)), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_contraction(ContractionArgs a, bool a_kmajor, bool bf16, hipStream_t s) {
  // (a 256 x 256 tile with 4 x 4 instruction tiles per wave needs more than the 512 registers of a
  // lane once two k-tiles of loads are in flight: measured 7x slower through scratch memory)
  if (bf16) return a_kmajor ? launch_tiles<BF16, true, 128>(a, s) : launch_tiles<BF16, false, 128>(a, s);
  return a_kmajor ? launch_tiles<F16, true, 128>(a, s) : launch_tiles<F16, false, 128>(a, s);
}

}  // namespace larosa
