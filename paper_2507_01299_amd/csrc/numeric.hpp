// 16-bit storage formats and small wave/block helpers shared by the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// The kernels rely on gfx950 behaviour that the HIP memory model does not promise (see the hand-off in
// gemv_core.hpp): accesses with the sc1 cache policy are coherent across the chip's eight L2 slices, a
// wave's s_waitcnt vmcnt(0) returns only after its stores were acknowledged there, and wave64 DPP /
// MFMA forms of this target.  Refuse to build the device code for anything else.
#if defined(__HIP_DEVICE_COMPILE__) && !defined(__gfx950__)
#error "liblarosa's device code is written for gfx950 (MI355X) only"
#endif

// Phase clocks of a diagnostic build (-DLAROSA_PHASE_CLOCK): lane 0 of a workgroup stores the
// 100 MHz wall clock to slot `n` of its row in a buffer whose address the host puts into
// larosa_phase_clock (null: off).  Product builds compile the stamps to nothing.
#ifdef LAROSA_PHASE_CLOCK
static __device__ unsigned long long* larosa_phase_clock = nullptr;
constexpr int kPhaseSlots = 16;
#define LAROSA_STAMP(n)                                                                         \
  do {                                                                                          \
    if (threadIdx.x == 0 && larosa_phase_clock)                                                 \
      larosa_phase_clock[(blockIdx.y * gridDim.x + blockIdx.x) * kPhaseSlots + (n)] = wall_clock64(); \
  } while (0)
#else
#define LAROSA_STAMP(n) do { } while (0)
#endif

namespace larosa {

constexpr int kWave = 64;

struct F16 {
  static __device__ __forceinline__ float to_f32(uint16_t b) {
    return static_cast<float>(__builtin_bit_cast(_Float16, b));
  }
  static __device__ __forceinline__ uint16_t from_f32(float f) {      // round to nearest even
    return __builtin_bit_cast(uint16_t, static_cast<_Float16>(f));
  }
  // two packed values in one dword -> two floats
  static __device__ __forceinline__ void unpack2(uint32_t w, float& lo, float& hi) {
    lo = to_f32(static_cast<uint16_t>(w & 0xFFFFu));
    hi = to_f32(static_cast<uint16_t>(w >> 16));
  }
};

struct BF16 {
  static __device__ __forceinline__ float to_f32(uint16_t b) {
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
  }
  static __device__ __forceinline__ uint16_t from_f32(float f) {      // round to nearest even
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return static_cast<uint16_t>((u >> 16) | 0x0040u);  // quiet NaN
    u += 0x7FFFu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
  }
  static __device__ __forceinline__ void unpack2(uint32_t w, float& lo, float& hi) {
    lo = __uint_as_float(w << 16);
    hi = __uint_as_float(w & 0xFFFF0000u);
  }
};

template <typename T>
__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) {
  T::unpack2(v.x, f[0], f[1]);
  T::unpack2(v.y, f[2], f[3]);
  T::unpack2(v.z, f[4], f[5]);
  T::unpack2(v.w, f[6], f[7]);
}

template <typename T>
__device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
  uint4 v;
  v.x = static_cast<uint32_t>(T::from_f32(f[0])) | (static_cast<uint32_t>(T::from_f32(f[1])) << 16);
  v.y = static_cast<uint32_t>(T::from_f32(f[2])) | (static_cast<uint32_t>(T::from_f32(f[3])) << 16);
  v.z = static_cast<uint32_t>(T::from_f32(f[4])) | (static_cast<uint32_t>(T::from_f32(f[5])) << 16);
  v.w = static_cast<uint32_t>(T::from_f32(f[6])) | (static_cast<uint32_t>(T::from_f32(f[7])) << 16);
  return v;
}

// value after one storage rounding
template <typename T>
__device__ __forceinline__ float round_store(float f) { return T::to_f32(T::from_f32(f)); }

// SiLU(g) = g / (1 + e^-g) with the hardware exp2 and reciprocal (about 1 ulp each in fp32, far
// below the 16-bit storage step the result is rounded to).
__device__ __forceinline__ float silu_f32(float g) {
  return g * __frcp_rn(1.0f + __expf(-g));
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// inclusive prefix sum across the 64 lanes of a wave, on the data-parallel-primitive path of the
// VALU (no LDS round trips): Hillis-Steele steps of 1, 2, 4, 8 lanes inside each row of 16, then
// the row totals are carried into the following rows by the two row-broadcast steps.
__device__ __forceinline__ unsigned wave_scan_inclusive(unsigned v, int /*lane*/) {
  // dpp_ctrl: row_shr:n = 0x110 + n, row_bcast:15 = 0x142, row_bcast:31 = 0x143.  old = 0 with
  // bound_ctrl off: lanes whose source lies outside the row (or outside row_mask) add zero.
  v += __builtin_amdgcn_update_dpp(0u, v, 0x111, 0xF, 0xF, false);
  v += __builtin_amdgcn_update_dpp(0u, v, 0x112, 0xF, 0xF, false);
  v += __builtin_amdgcn_update_dpp(0u, v, 0x114, 0xF, 0xF, false);
  v += __builtin_amdgcn_update_dpp(0u, v, 0x118, 0xF, 0xF, false);
  v += __builtin_amdgcn_update_dpp(0u, v, 0x142, 0xA, 0xF, false);   // lane 15 of rows 0, 2 -> rows 1, 3
  v += __builtin_amdgcn_update_dpp(0u, v, 0x143, 0xC, 0xF, false);   // lane 31 -> rows 2, 3
  return v;
}

}  // namespace larosa
