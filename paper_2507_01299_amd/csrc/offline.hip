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

// Operand loads go through buffer resources that span the whole (multi-term) operand: a 16-byte load whose
// offset lies at or beyond the operand's size returns zeros, so rows past Kd need no test, and a lane whose
// columns lie outside the matrix carries the offset kOutside for good.  Per k-tile a load then costs one
// add (lane offset + the tile's scalar offset) and no branch.
constexpr uint32_t kOutside = 0x80000000u;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t operand_buffer(const uint16_t* p, long elements) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p), 0, static_cast<int>(elements * 2), 0x00027000);
}

__device__ __forceinline__ uint4 load16(__amdgpu_buffer_rsrc_t buf, uint32_t lane_off, uint32_t tile_off) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(buf, static_cast<int>(lane_off + tile_off), 0, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ void store_kmajor(uint32_t* tile, const uint4& r0, const uint4& r1, int g, int kp) {
  const uint32_t a[4] = {r0.x, r0.y, r0.z, r0.w};
  const uint32_t b[4] = {r1.x, r1.y, r1.z, r1.w};
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    tile[(8 * g + 2 * q) * kRowDwords + kp] = __builtin_amdgcn_perm(b[q], a[q], 0x05040100u);       // a.lo | b.lo << 16
    tile[(8 * g + 2 * q + 1) * kRowDwords + kp] = __builtin_amdgcn_perm(b[q], a[q], 0x07060302u);   // a.hi | b.hi << 16
  }
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

// One k-tile of both operands in a thread's registers: NA / NB 16-byte pieces of A / B.
template <int NA, int NB>
struct Staged {
  uint4 a[NA];
  uint4 b[NB];
};

// Is the 256 x TN tile that holds element (row, col) left out of a symmetric product?
template <int TN>
__device__ __forceinline__ bool tile_skipped(int row, int col) {
  return TN * (col / TN + 1) <= kTileM * (row / kTileM);
}

// A workgroup of NW waves owns a 256 x TN tile of C; every wave a 128 x 64 part (4 x 2 instruction tiles):
// NW = 4, TN = 128 (two workgroups per compute unit) or NW = 8, TN = 256 (one).  The larger tile moves a third
// fewer operand bytes from the L2 per flop, which is what bounds the product.
template <typename T, bool A_KMAJOR, int TN, int NW>
__global__ __launch_bounds__(NW * 64, NW == 4 ? 2 : 1) void contraction_kernel(ContractionArgs a) {
  constexpr int NT = NW * 64;
  constexpr int WN = NW / 2;                     // waves along n (two along m)
  constexpr int NJ = TN / (32 * WN);             // 32-column instruction tiles of a wave along n
  static_assert(NJ == 2, "a wave owns 128 x 64");
  constexpr int GA = 32 * 16 / NT;               // 8-column groups of A per thread (k-major: two rows each)
  constexpr int GB = (TN / 8) * 16 / NT;         // the same for B
  constexpr int NA = 2 * GA, NB = 2 * GB;
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
  constexpr int kGroupsPerPass = NT / 16;        // 8-column groups that the workgroup's threads cover at once
  const int g = (lane & 7) + 8 * (w % (NW / 2));
  const int kp = (lane >> 3) + 8 * (w / (NW / 2));
  const int wm = w / WN, wn = w % WN;   // wave tile: rows wm * 128 .. + 127, columns wn * 64 .. + 63

  float16v acc[4][NJ];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  const int ktiles = (a.Kd + kKTile - 1) / kKTile;
  const int iters = ktiles * a.npairs;

  // lane offsets (bytes) into the operands, fixed for the whole kernel
  const __amdgpu_buffer_rsrc_t bufA = operand_buffer(a.A, a.a_elements);
  const __amdgpu_buffer_rsrc_t bufB = operand_buffer(a.B, a.b_elements);
  uint32_t offA[NA], offB[NB];
  if (A_KMAJOR) {   // rows 2 kp, 2 kp + 1 of the k-tile, columns m0 + 8 (g + h * groups per pass) ..
#pragma unroll
    for (int h = 0; h < GA; ++h) {
      const int c = m0 + 8 * (g + kGroupsPerPass * h);
      offA[2 * h] = c < a.M ? static_cast<uint32_t>((2 * kp * a.M + c) * 2) : kOutside;
      offA[2 * h + 1] = c < a.M ? offA[2 * h] + static_cast<uint32_t>(a.M * 2) : kOutside;
    }
  } else {          // row m0 + t / 4 + (NT / 4) r, k values 8 (t % 4) .. + 7 of the k-tile
#pragma unroll
    for (int r = 0; r < NA; ++r) {
      const int m = m0 + (t >> 2) + (NT / 4) * r;
      offA[r] = m < a.M ? static_cast<uint32_t>((m * a.Kd + 8 * (t & 3)) * 2) : kOutside;
    }
  }
#pragma unroll
  for (int h = 0; h < GB; ++h) {
    const int c = n0 + 8 * (g + kGroupsPerPass * h);
    offB[2 * h] = c < a.N ? static_cast<uint32_t>((2 * kp * a.N + c) * 2) : kOutside;
    offB[2 * h + 1] = c < a.N ? offB[2 * h] + static_cast<uint32_t>(a.N * 2) : kOutside;
  }

  // iteration it = (term pair p, k-tile kt), kt fastest; the scalar offsets of its tile
  int f_p = 0, f_kt = 0;
  auto fetch = [&](Staged<NA, NB>& st) {
    const int k0 = f_kt * kKTile;
    const uint32_t ta = static_cast<uint32_t>((a.pa[f_p] * a.a_term_stride + (A_KMAJOR ? static_cast<long>(k0) * a.M : k0)) * 2);
    const uint32_t tb = static_cast<uint32_t>((a.pb[f_p] * a.b_term_stride + static_cast<long>(k0) * a.N) * 2);
    // rows of this k-tile at or past Kd are zero (with several terms the bytes behind a term are the next term's)
    const int kr = a.Kd - k0;
    const bool row0 = 2 * kp < kr, row1 = 2 * kp + 1 < kr;
    if (A_KMAJOR) {
#pragma unroll
      for (int r = 0; r < NA; ++r) st.a[r] = load16(bufA, ((r & 1) ? row1 : row0) ? offA[r] : kOutside, ta);
    } else {
      // a row's k values past Kd belong to the next row: those lanes read outside instead
      const bool in = k0 + 8 * (t & 3) < a.Kd;
#pragma unroll
      for (int r = 0; r < NA; ++r) st.a[r] = load16(bufA, in ? offA[r] : kOutside, ta);
    }
#pragma unroll
    for (int r = 0; r < NB; ++r) st.b[r] = load16(bufB, ((r & 1) ? row1 : row0) ? offB[r] : kOutside, tb);
    if (++f_kt == ktiles) { f_kt = 0; ++f_p; }
  };
  auto stash = [&](int buf, const Staged<NA, NB>& st) {
    if (A_KMAJOR) {
#pragma unroll
      for (int h = 0; h < GA; ++h) store_kmajor(lds_a[buf], st.a[2 * h], st.a[2 * h + 1], g + kGroupsPerPass * h, kp);
    } else {
#pragma unroll
      for (int r = 0; r < NA; ++r) store_kcontig(lds_a[buf], st.a[r], (t >> 2) + (NT / 4) * r, t & 3);
    }
#pragma unroll
    for (int h = 0; h < GB; ++h) store_kmajor(lds_b[buf], st.b[2 * h], st.b[2 * h + 1], g + kGroupsPerPass * h, kp);
  };
  // one 16-deep half (s = 0, 1) of the k-tile in LDS buffer buf
  auto compute_half = [&](int buf, int s) {
    const uint32_t* At = lds_a[buf];
    const uint32_t* Bt = lds_b[buf];
    const int dw = s * 8 + (lane >> 5) * 4;
    u32x4 av[4], bv[NJ];
#pragma unroll
    for (int i = 0; i < 4; ++i) av[i] = read_operand(At, wm * 128 + i * 32 + (lane & 31), dw);
#pragma unroll
    for (int j = 0; j < NJ; ++j) bv[j] = read_operand(Bt, wn * 64 + j * 32 + (lane & 31), dw);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j) acc[i][j] = Mfma<T>::run(av[i], bv[j], acc[i][j]);
  };

  // Tile it is computed from LDS buffer it & 1 while the loads of tile it + 2 are in flight and tile
  // it + 1 (loaded one step earlier) moves from registers to the other buffer: one barrier per tile.
  Staged<NA, NB> s0, s1;
  fetch(s0);
  stash(0, s0);
  if (iters > 1) fetch(s1);
  __syncthreads();
  for (int it = 0; it < iters; it += 2) {
    // (moving the stash between the two halves of the products, so that its writes complete behind matrix
    // instructions, measured no faster)
    if (it + 2 < iters) fetch(s0);
    compute_half(0, 0);
    compute_half(0, 1);
    if (it + 1 < iters) stash(1, s1);
    __syncthreads();
    if (it + 1 < iters) {
      if (it + 3 < iters) fetch(s1);
      compute_half(1, 0);
      compute_half(1, 1);
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
    const int n = n0 + wn * 64 + j * 32 + (lane & 31);
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

template <typename T, bool A_KMAJOR, int TN, int NW>
hipError_t launch_tiles(ContractionArgs a, hipStream_t s) {
  a.tiles_m = (a.M + kTileM - 1) / kTileM;
  a.tiles_n = (a.N + TN - 1) / TN;
  a.patches_m = (a.tiles_m + kPatchM - 1) / kPatchM;
  a.patches_n = (a.tiles_n + kPatchN - 1) / kPatchN;
  // the operands are addressed with 32-bit byte offsets from their first term
  int ta = 0, tb = 0;
  for (int i = 0; i < a.npairs; ++i) {
    ta = a.pa[i] > ta ? a.pa[i] : ta;
    tb = a.pb[i] > tb ? a.pb[i] : tb;
  }
  a.a_elements = ta * a.a_term_stride + static_cast<long>(a.Kd) * a.M;
  a.b_elements = tb * a.b_term_stride + static_cast<long>(a.Kd) * a.N;
  if (a.a_elements * 2 >= 0x7FFFFFF0L || a.b_elements * 2 >= 0x7FFFFFF0L) return hipErrorInvalidValue;
  const long patches = static_cast<long>(a.patches_m) * a.patches_n;
  const long grid = (patches + 7) / 8 * 8 * 32;
  if (grid > 0x7FFFFFFFL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((contraction_kernel<T, A_KMAJOR, TN, NW>), dim3(static_cast<unsigned>(grid)), dim3(NW * 64), 0, s, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_contraction(ContractionArgs a, bool a_kmajor, bool bf16, hipStream_t s) {
  // 256 x 256 tiles (8 waves) where the product has enough of them to fill the chip, else 256 x 128 (4 waves)
  long big_tiles = static_cast<long>((a.M + 255) / 256) * ((a.N + 255) / 256);
  if (a.symmetric) big_tiles /= 2;               // tiles below the diagonal are not computed
  const int forced = tuning().contraction_tiles; // 0: by size, 1: 256 x 128, 2: 256 x 256 (tests)
  const bool big = forced == 2 || (forced == 0 && big_tiles >= 256);
  if (big) {
    if (bf16) return a_kmajor ? launch_tiles<BF16, true, 256, 8>(a, s) : launch_tiles<BF16, false, 256, 8>(a, s);
    return a_kmajor ? launch_tiles<F16, true, 256, 8>(a, s) : launch_tiles<F16, false, 256, 8>(a, s);
  }
  if (bf16) return a_kmajor ? launch_tiles<BF16, true, 128, 4>(a, s) : launch_tiles<BF16, false, 128, 4>(a, s);
  return a_kmajor ? launch_tiles<F16, true, 128, 4>(a, s) : launch_tiles<F16, false, 128, 4>(a, s);
}

}  // namespace larosa
