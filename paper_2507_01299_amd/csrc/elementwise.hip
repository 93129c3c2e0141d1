// Small elementwise kernels that glue the LaRoSA projections into a decoder layer
// (Fig. 2 of the paper: pre-norm, attention core stand-in, SwiGLU product).
#include "kernels.hpp"
#include "numeric.hpp"

namespace larosa {

namespace {

// Context-length-1 attention: softmax over one key is 1, so query head i outputs the value
// head of its group.  Pure 16-bit copy; 8 values (16 bytes) per lane.
__global__ void gqa_expand_kernel(const uint16_t* __restrict__ qkv, uint16_t* __restrict__ h2, int d_q, int d_kv,
                                  int head_dim, int group) {
  const int b = blockIdx.y;
  const int i = (blockIdx.x * blockDim.x + threadIdx.x) * 8;
  if (i >= d_q) return;
  const int head = i / head_dim;
  const int within = i - head * head_dim;
  const int src = (head / group) * head_dim + within;
  const size_t row = static_cast<size_t>(b) * (d_q + 2 * d_kv);
  const uint4 v = *reinterpret_cast<const uint4*>(qkv + row + d_q + d_kv + src);
  *reinterpret_cast<uint4*>(h2 + static_cast<size_t>(b) * d_q + i) = v;
}

template <typename T>
__global__ void silu_mul_kernel(const uint16_t* __restrict__ gu, uint16_t* __restrict__ h4, int d_ff) {
  const int b = blockIdx.y;
  const int i = (blockIdx.x * blockDim.x + threadIdx.x) * 8;
  if (i >= d_ff) return;
  const size_t row = static_cast<size_t>(b) * 2 * d_ff;
  float g[8], u[8], o[8];
  unpack8<T>(*reinterpret_cast<const uint4*>(gu + row + i), g);
  unpack8<T>(*reinterpret_cast<const uint4*>(gu + row + d_ff + i), u);
#pragma unroll
  for (int k = 0; k < 8; ++k) o[k] = silu_f32(g[k]) * u[k];
  *reinterpret_cast<uint4*>(h4 + static_cast<size_t>(b) * d_ff + i) = pack8<T>(o);
}

template <typename T>
__global__ __launch_bounds__(1024) void rmsnorm_kernel(const uint16_t* __restrict__ x,
                                                       const uint16_t* __restrict__ scale,
                                                       uint16_t* __restrict__ y, int d, float eps) {
  __shared__ float red[16];
  const int b = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint16_t* xb = x + static_cast<size_t>(b) * d;
  float ss = 0.f;
  for (int i = threadIdx.x * 8; i < d; i += 1024 * 8) {
    float w[8];
    unpack8<T>(*reinterpret_cast<const uint4*>(xb + i), w);
#pragma unroll
    for (int k = 0; k < 8; ++k) ss = fmaf(w[k], w[k], ss);
  }
  ss = wave_sum(ss);
  if (lane == 0) red[wave] = ss;
  __syncthreads();
  float tot = 0.f;
  for (int w2 = 0; w2 < 16; ++w2) tot += red[w2];
  const float rinv = 1.0f / sqrtf(tot / static_cast<float>(d) + eps);
  for (int i = threadIdx.x * 8; i < d; i += 1024 * 8) {
    float w[8];
    unpack8<T>(*reinterpret_cast<const uint4*>(xb + i), w);
    if (scale) {
      float g[8];
      unpack8<T>(*reinterpret_cast<const uint4*>(scale + i), g);
#pragma unroll
      for (int k = 0; k < 8; ++k) w[k] = w[k] * rinv * g[k];
    } else {
#pragma unroll
      for (int k = 0; k < 8; ++k) w[k] *= rinv;
    }
    *reinterpret_cast<uint4*>(y + static_cast<size_t>(b) * d + i) = pack8<T>(w);
  }
}

__global__ void fill_u32_kernel(unsigned* p, size_t n, unsigned v) {
  const size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

__global__ void copy_u16x8_kernel(const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, size_t n) {
  const size_t i = (static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x) * 8;
  if (i < n) *reinterpret_cast<uint4*>(dst + i) = *reinterpret_cast<const uint4*>(src + i);
}

}  // namespace

hipError_t launch_gqa_expand(const uint16_t* qkv, uint16_t* h2, int B, int d_q, int d_kv, int head_dim,
                             hipStream_t s) {
  const int group = (d_q / head_dim) / (d_kv / head_dim);
  dim3 block(256), grid((d_q / 8 + 255) / 256, B);
  hipLaunchKernelGGL(gqa_expand_kernel, grid, block, 0, s, qkv, h2, d_q, d_kv, head_dim, group);
  return hipGetLastError();
}

hipError_t launch_silu_mul(const uint16_t* gu, uint16_t* h4, int B, int d_ff, bool bf16, hipStream_t s) {
  dim3 block(256), grid((d_ff / 8 + 255) / 256, B);
  if (bf16)
    hipLaunchKernelGGL(silu_mul_kernel<BF16>, grid, block, 0, s, gu, h4, d_ff);
  else
    hipLaunchKernelGGL(silu_mul_kernel<F16>, grid, block, 0, s, gu, h4, d_ff);
  return hipGetLastError();
}

hipError_t launch_rmsnorm(const uint16_t* x, const uint16_t* scale, uint16_t* y, int B, int d, float eps,
                          bool bf16, hipStream_t s) {
  dim3 block(1024), grid(B);
  if (bf16)
    hipLaunchKernelGGL(rmsnorm_kernel<BF16>, grid, block, 0, s, x, scale, y, d, eps);
  else
    hipLaunchKernelGGL(rmsnorm_kernel<F16>, grid, block, 0, s, x, scale, y, d, eps);
  return hipGetLastError();
}

hipError_t launch_fill_u32(unsigned* p, size_t n, unsigned v, hipStream_t s) {
  dim3 block(256), grid(static_cast<unsigned>((n + 255) / 256));
  hipLaunchKernelGGL(fill_u32_kernel, grid, block, 0, s, p, n, v);
  return hipGetLastError();
}

hipError_t launch_copy_u16(const uint16_t* src, uint16_t* dst, size_t n, hipStream_t s) {
  dim3 block(256), grid(static_cast<unsigned>((n / 8 + 255) / 256));
  hipLaunchKernelGGL(copy_u16x8_kernel, grid, block, 0, s, src, dst, n);
  return hipGetLastError();
}

}  // namespace larosa
