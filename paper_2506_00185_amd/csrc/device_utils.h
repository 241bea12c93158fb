// Device-side helpers shared by the decoding kernels (gfx950, 64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rb {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kMaxBeam = 16;
constexpr int kCtxMax = 8;          // tokens of history kept per hypothesis (LM order <= 9, stateless ctx <= 4)
constexpr uint64_t kHashBase = 1000003ull;
constexpr uint64_t kHashMod = 2147483647ull;  // 2^31 - 1

// One 32x32x2 fp32 matrix-core step: acc[i][j] += sum_{k<2} A[i][k] B[k][j].
// Lane l supplies A[i = l % 32][k = l / 32] and B[k = l / 32][j = l % 32]; it
// receives acc[i = 8 * (r / 4) + 4 * (l / 32) + r % 4][j = l % 32] in register r.
__device__ __forceinline__ floatx16 mfma32(float a, float b, floatx16 acc) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
}

// float32 -> bfloat16 (round to nearest even) -> float32
__device__ __forceinline__ float bf16_round(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7f800000u) == 0x7f800000u) return x;
  u += 0x7fffu + ((u >> 16) & 1u);
  u &= 0xffff0000u;
  return __uint_as_float(u);
}

__device__ __forceinline__ float4 bf16_round4(float4 v) {
  return make_float4(bf16_round(v.x), bf16_round(v.y), bf16_round(v.z), bf16_round(v.w));
}

__device__ __forceinline__ double logaddexp_d(double a, double b) {
  if (a == -INFINITY) return b;
  if (b == -INFINITY) return a;
  double m = a > b ? a : b;
  return m + log(exp(a - m) + exp(b - m));
}

template <typename T>
__device__ __forceinline__ T wave_max(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    T w = __shfl_xor(v, o);
    v = w > v ? w : v;
  }
  return v;
}

template <typename T>
__device__ __forceinline__ T wave_min(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    T w = __shfl_xor(v, o);
    v = w < v ? w : v;
  }
  return v;
}

template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// Candidate order used everywhere a "best" is chosen: larger value first, then
// smaller index.  Returns true if (v1, i1) comes before (v2, i2).
template <typename V, typename I>
__device__ __forceinline__ bool comes_before(V v1, I i1, V v2, I i2) {
  return v1 > v2 || (v1 == v2 && i1 < i2);
}

// Wave-wide best of (value, index) under comes_before; every lane gets the winner.
template <typename V, typename I>
__device__ __forceinline__ void wave_best(V &v, I &i) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    V v2 = __shfl_xor(v, o);
    I i2 = __shfl_xor(i, o);
    if (comes_before(v2, i2, v, i)) {
      v = v2;
      i = i2;
    }
  }
}

}  // namespace rb
