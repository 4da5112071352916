// 4-bit NormalFloat block quantisation of frozen projection weights (quantised base + LoRA, paper
// Section 4.5 and Table 3; format of the public QLoRA description): blocks of 64 consecutive elements,
// one float absolute maximum per block, per element the index of the nearest of 16 fixed levels.
#include "common.h"

namespace {
// the 16 levels (quantiles of N(0,1) normalised to [-1, 1], with an exact zero)
__device__ __constant__ float kLevel[16] = {
    -1.0f, -0.6961928009986877f, -0.5250730514526367f, -0.39491748809814453f,
    -0.28444138169288635f, -0.18477343022823334f, -0.09105003625154495f, 0.0f,
    0.07958029955625534f, 0.16093020141124725f, 0.24611230194568634f, 0.33791524171829224f,
    0.44070982933044434f, 0.5626170039176941f, 0.7229568362236023f, 1.0f};

// one wave per 64-element block, lane i owns element i
template <typename T>
__global__ void nf4_quantize_kernel(const T* __restrict__ w, int64_t n_blocks, uint8_t* __restrict__ codes, float* __restrict__ absmax) {
  const int lane = threadIdx.x & 63;
  const int64_t blk = (int64_t)blockIdx.x * (blockDim.x / 64) + threadIdx.x / 64;
  if (blk >= n_blocks) return;
  const float v = to_f<T>(w[blk * 64 + lane]);
  float m = fabsf(v);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  const float x = v / (m > 0.f ? m : 1.f);
  int code = 0;
#pragma unroll
  for (int i = 0; i < 15; i++) code += (x >= (kLevel[i] + kLevel[i + 1]) * 0.5f) ? 1 : 0;   // a midpoint goes to the higher level
  const int hi = __shfl_down(code, 1, 64);
  if ((lane & 1) == 0) codes[blk * 32 + (lane >> 1)] = (uint8_t)(code | (hi << 4));
  if (lane == 0) absmax[blk] = m;
}

// one thread per 8 elements: four code bytes in, 8 values of type T out
template <typename T>
__global__ void nf4_dequantize_kernel(const uint8_t* __restrict__ codes, const float* __restrict__ absmax, int64_t n8, T* __restrict__ out) {
  __shared__ float lut[16];
  if (threadIdx.x < 16) lut[threadIdx.x] = kLevel[threadIdx.x];
  __syncthreads();
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n8) return;
  const uint32_t c = *reinterpret_cast<const uint32_t*>(codes + i * 4);
  const float a = absmax[i >> 3];
  T* o = out + i * 8;
#pragma unroll
  for (int e = 0; e < 8; e++) o[e] = from_f<T>(lut[(c >> (4 * e)) & 15] * a);
}
}  // namespace

int launch_nf4_quantize(as_ctx* ctx, int mode, const void* w, int64_t numel, uint8_t* codes, float* absmax, hipStream_t st) {
  if (numel <= 0) return AS_OK;
  if (numel % 64) return as_fail(ctx, AS_ERR_SHAPE, "nf4: the element count must be a multiple of 64");
  const int64_t nb = numel / 64;
  if (mode == AS_FP32) nf4_quantize_kernel<float><<<(unsigned)cdiv(nb, 4), 256, 0, st>>>((const float*)w, nb, codes, absmax);
  else nf4_quantize_kernel<bf16_t><<<(unsigned)cdiv(nb, 4), 256, 0, st>>>((const bf16_t*)w, nb, codes, absmax);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}

int launch_nf4_dequantize(as_ctx* ctx, int mode, const uint8_t* codes, const float* absmax, int64_t numel, void* out, hipStream_t st) {
  if (numel <= 0) return AS_OK;
  if (numel % 64) return as_fail(ctx, AS_ERR_SHAPE, "nf4: the element count must be a multiple of 64");
  if ((uintptr_t)codes % 4) return as_fail(ctx, AS_ERR_SHAPE, "nf4: the code array must be 4-byte aligned");
  const int64_t n8 = numel / 8;
  if (mode == AS_FP32) nf4_dequantize_kernel<float><<<(unsigned)cdiv(n8, 256), 256, 0, st>>>(codes, absmax, n8, (float*)out);
  else nf4_dequantize_kernel<bf16_t><<<(unsigned)cdiv(n8, 256), 256, 0, st>>>(codes, absmax, n8, (bf16_t*)out);
  AS_LAUNCH_CHECK(ctx);
  return AS_OK;
}
