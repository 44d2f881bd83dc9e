// Shared device/host helpers for the gfx950 kernels of libsama.  Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>

namespace sama {

typedef uint16_t bf16_t;  // raw bfloat16 bits

constexpr int WAVE = 64;

__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// two floats -> packed bf16 pair (a in the low half), round-to-nearest-even in hardware (v_cvt_pk_bf16_f32)
typedef __bf16 bf16x2_hw __attribute__((ext_vector_type(2)));
typedef float f32x2_hw __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  const f32x2_hw v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_hw));
}

// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)pack_bf16x2(f, 0.f); }

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}

// Sum over a block of up to 1024 threads in a fixed order: wave shuffles, then the wave leaders' values
// added serially from LDS.  Every thread gets the result.  `red` holds >= 16 floats.
__device__ __forceinline__ float block_sum(float x, float* red) {
  x = wave_sum(x);
  const int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = x;
  __syncthreads();
  float s = 0.f;
  for (int i = 0; i < nw; ++i) s += red[i];
  return s;
}

// A non-GEMM parameter as the current pass sees it: theta[k] + s * v[k], with s = +-eps read from the device
// (s_ptr == nullptr: the unperturbed parameter).
struct ParamView {
  const float* theta;
  const float* vdir;
  const float* eps_ptr;
  float sign;
  int flip_row;  // > 0: a kernel's rows >= flip_row see the opposite sign (the + and the - pass stacked in one launch)
  __device__ __forceinline__ float scale() const { return (eps_ptr != nullptr && sign != 0.f) ? sign * (*eps_ptr) : 0.f; }
  __device__ __forceinline__ float scale_row(int row) const {
    const float s = scale();
    return (flip_row > 0 && row >= flip_row) ? -s : s;
  }
  __device__ __forceinline__ float at(int64_t k, float s) const { return s != 0.f ? fmaf(s, vdir[k], theta[k]) : theta[k]; }
};

}  // namespace sama
