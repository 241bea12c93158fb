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

// ---- bfloat16 operands of the bf16 matrix instructions
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));
typedef uint32_t uintx4_t __attribute__((ext_vector_type(4)));
typedef uint32_t uintx2_t __attribute__((ext_vector_type(2)));

// two float32 -> two bfloat16 in one word (low half first), round to nearest even: one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi) {
  const floatx2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// One 32x32x16 bf16 matrix-core step fed from float32 registers: the lane's 8 k-values are the 4 + 4 floats it holds
// for two consecutive 8-k rounds of the float32 scheme (see mfma32), rounded to bf16 here.  Both operands use the
// same lane -> k assignment, so every k of the 16 meets its partner exactly once.
__device__ __forceinline__ floatx16 mfma32_bf16_from_f32(float4 a0, float4 a1, float4 b0, float4 b1, floatx16 acc) {
  const uintx4_t pa = {pack_bf16_rne(a0.x, a0.y), pack_bf16_rne(a0.z, a0.w), pack_bf16_rne(a1.x, a1.y),
                       pack_bf16_rne(a1.z, a1.w)};
  const uintx4_t pb = {pack_bf16_rne(b0.x, b0.y), pack_bf16_rne(b0.z, b0.w), pack_bf16_rne(b1.x, b1.y),
                       pack_bf16_rne(b1.z, b1.w)};
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, pa), __builtin_bit_cast(bf16x8_t, pb), acc, 0,
                                                 0, 0);
}

__device__ __forceinline__ double logaddexp_d(double a, double b) {
  if (a == -INFINITY) return b;
  if (b == -INFINITY) return a;
  double m = a > b ? a : b;
  return m + log(exp(a - m) + exp(b - m));
}

// Stores and loads that are coherent across the whole device on their own (they bypass the caches
// that are private to a group of compute units), for the few words that one block hands to another
// inside a kernel.  A device-wide release / acquire fence would write back and invalidate the whole
// L2 instead, which costs microseconds.
template <typename T>
__device__ __forceinline__ void store_agent(T *p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ T load_agent(const T *p) {
  return __hip_atomic_load(const_cast<T *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Blocks the calling wave until every global load and store it has issued has completed; a write-through
// store completes when the memory side has acknowledged it.  (gfx9 counts stores in vmcnt.)
__device__ __forceinline__ void wait_stores_acknowledged() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Results that only a LATER launch reads.  A plain store leaves its line dirty in the XCD's L2, and the end of
// every kernel waits until all dirty lines have been written back (the L2s of the XCDs are not coherent with each
// other, so that is how one launch's output becomes visible to the next).  Writing through at once takes that
// wait off the chain of dependent launches: 20.0 -> 19.5 ms per decode at 2 061 launches.
template <typename T>
__device__ __forceinline__ void store_through(T *p, T v) {
  store_agent(p, v);
}

// 16 bytes written through (one instruction; the atomic store above exists for 4 and 8 bytes only)
__device__ __forceinline__ void store16_through(float *p, floatx4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}

// Candidate order used everywhere a "best" is chosen: larger value first, then
// smaller index.  Returns true if (v1, i1) comes before (v2, i2).
template <typename V, typename I>
__device__ __forceinline__ bool comes_before(V v1, I i1, V v2, I i2) {
  return v1 > v2 || (v1 == v2 && i1 < i2);
}
// the same without short circuits, for unrolled runs of comparisons (the compiler turns the form above into a branch
// per comparison when the values are doubles, which costs more than the compares themselves)
template <typename V, typename I>
__device__ __forceinline__ int comes_before_count(V v1, I i1, V v2, I i2) {
  return (int)(v1 > v2) | ((int)(v1 == v2) & (int)(i1 < i2));
}

// ---- cross-lane exchange without the LDS crossbar --------------------------
// __shfl_* compiles to ds_bpermute (LDS latency, ~100+ cycles per exchange); a
// data-parallel-primitive move costs one VALU instruction.  The four patterns
// below are butterflies inside a row of 16 lanes: lane ^ 1, lane ^ 2, then the
// mirror of each half row (pairs quads) and the mirror of the row (pairs halves).
constexpr int kDppXor1 = 0xB1;        // quad_perm [1, 0, 3, 2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2, 3, 0, 1]
constexpr int kDppHalfMirror = 0x141; // row_half_mirror
constexpr int kDppMirror = 0x140;     // row_mirror

template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) {
  return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __int_as_float(dpp_i<CTRL>(__float_as_int(v)));
}
template <int CTRL>
__device__ __forceinline__ double dpp_d(double v) {
  const long long b = __double_as_longlong(v);
  const int lo = dpp_i<CTRL>((int)(b & 0xffffffffll)), hi = dpp_i<CTRL>((int)(b >> 32));
  return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
__device__ __forceinline__ float readlane_f(float v, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ double readlane_d(double v, int lane) {
  const long long b = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_readlane((int)(b & 0xffffffffll), lane);
  const int hi = __builtin_amdgcn_readlane((int)(b >> 32), lane);
  return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

// all-reduce over aligned groups of LANES (4, 8 or 16) lanes
template <int LANES>
__device__ __forceinline__ float group_max(float v) {
  v = fmaxf(v, dpp_f<kDppXor1>(v));
  v = fmaxf(v, dpp_f<kDppXor2>(v));
  if constexpr (LANES >= 8) v = fmaxf(v, dpp_f<kDppHalfMirror>(v));
  if constexpr (LANES >= 16) v = fmaxf(v, dpp_f<kDppMirror>(v));
  return v;
}
template <int LANES>
__device__ __forceinline__ float group_sum(float v) {
  v += dpp_f<kDppXor1>(v);
  v += dpp_f<kDppXor2>(v);
  if constexpr (LANES >= 8) v += dpp_f<kDppHalfMirror>(v);
  if constexpr (LANES >= 16) v += dpp_f<kDppMirror>(v);
  return v;
}
template <int CTRL, typename V>
__device__ __forceinline__ void best_step(V &v, int &i) {
  V v2;
  if constexpr (sizeof(V) == 8) v2 = dpp_d<CTRL>(v); else v2 = dpp_f<CTRL>(v);
  const int i2 = dpp_i<CTRL>(i);
  if (comes_before(v2, i2, v, i)) {
    v = v2;
    i = i2;
  }
}
// best (value, index) pair of an aligned group of LANES lanes, in every lane of the group
template <int LANES, typename V>
__device__ __forceinline__ void group_best(V &v, int &i) {
  best_step<kDppXor1>(v, i);
  best_step<kDppXor2>(v, i);
  if constexpr (LANES >= 8) best_step<kDppHalfMirror>(v, i);
  if constexpr (LANES >= 16) best_step<kDppMirror>(v, i);
}

// ---- candidates packed into one sortable word ---------------------------------
// (key, index) -> 64 bits whose unsigned order is the candidate order: larger key first, then
// smaller index.  One compare instead of three, and a pair moves as two DPP words.
__device__ __forceinline__ uint32_t orderable(float f) {
  const uint32_t u = __float_as_uint(f);
  return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
}
__device__ __forceinline__ float from_orderable(uint32_t u) {
  return __uint_as_float(u ^ (((u >> 31) - 1u) | 0x80000000u));
}
__device__ __forceinline__ uint64_t pack_cand(float key, int idx) {
  return ((uint64_t)orderable(key) << 32) | (uint32_t)(0x7fffffff - idx);
}
__device__ __forceinline__ float cand_key(uint64_t c) { return from_orderable((uint32_t)(c >> 32)); }
__device__ __forceinline__ int cand_idx(uint64_t c) { return 0x7fffffff - (int)(uint32_t)c; }
// "no candidate": key -inf, index 0x7fffffff; every real candidate is larger
__device__ __forceinline__ uint64_t no_cand() { return pack_cand(-INFINITY, 0x7fffffff); }

template <int CTRL>
__device__ __forceinline__ uint64_t dpp_u64(uint64_t v) {
  const int lo = dpp_i<CTRL>((int)(uint32_t)v), hi = dpp_i<CTRL>((int)(uint32_t)(v >> 32));
  return ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo;
}
template <int CTRL>
__device__ __forceinline__ uint64_t max_step(uint64_t v) {
  const uint64_t w = dpp_u64<CTRL>(v);
  return w > v ? w : v;
}
// largest packed candidate of an aligned group of LANES lanes, in every lane of the group
template <int LANES>
__device__ __forceinline__ uint64_t group_max_u64(uint64_t v) {
  v = max_step<kDppXor1>(v);
  v = max_step<kDppXor2>(v);
  if constexpr (LANES >= 8) v = max_step<kDppHalfMirror>(v);
  if constexpr (LANES >= 16) v = max_step<kDppMirror>(v);
  return v;
}
// wave-wide max of packed candidates, in every lane
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
  v = group_max_u64<16>(v);
  uint64_t best = 0;
#pragma unroll
  for (int r = 0; r < 64; r += 16) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, r);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), r);
    const uint64_t w = ((uint64_t)hi << 32) | lo;
    best = w > best ? w : best;
  }
  return best;
}

template <int LANES>
__device__ __forceinline__ int group_min_i(int v) {
  v = min(v, dpp_i<kDppXor1>(v));
  v = min(v, dpp_i<kDppXor2>(v));
  if constexpr (LANES >= 8) v = min(v, dpp_i<kDppHalfMirror>(v));
  if constexpr (LANES >= 16) v = min(v, dpp_i<kDppMirror>(v));
  return v;
}

// wave-wide versions: reduce inside the four rows, then combine the rows through scalar reads
__device__ __forceinline__ float wave_max(float v) {
  v = group_max<16>(v);
  return fmaxf(fmaxf(readlane_f(v, 0), readlane_f(v, 16)), fmaxf(readlane_f(v, 32), readlane_f(v, 48)));
}
__device__ __forceinline__ float wave_sum(float v) {
  v = group_sum<16>(v);
  return (readlane_f(v, 0) + readlane_f(v, 16)) + (readlane_f(v, 32) + readlane_f(v, 48));
}
__device__ __forceinline__ int wave_sum_i(int v) {
  v += dpp_i<kDppXor1>(v);
  v += dpp_i<kDppXor2>(v);
  v += dpp_i<kDppHalfMirror>(v);
  v += dpp_i<kDppMirror>(v);
  return (__builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16)) +
         (__builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48));
}
__device__ __forceinline__ void wave_best(float &v, int &i) {
  group_best<16>(v, i);
  float bv = readlane_f(v, 0);
  int bi = __builtin_amdgcn_readlane(i, 0);
#pragma unroll
  for (int r = 16; r < 64; r += 16) {
    const float v2 = readlane_f(v, r);
    const int i2 = __builtin_amdgcn_readlane(i, r);
    if (comes_before(v2, i2, bv, bi)) {
      bv = v2;
      bi = i2;
    }
  }
  v = bv;
  i = bi;
}
__device__ __forceinline__ void wave_best(double &v, int &i) {
  group_best<16>(v, i);
  double bv = readlane_d(v, 0);
  int bi = __builtin_amdgcn_readlane(i, 0);
#pragma unroll
  for (int r = 16; r < 64; r += 16) {
    const double v2 = readlane_d(v, r);
    const int i2 = __builtin_amdgcn_readlane(i, r);
    if (comes_before(v2, i2, bv, bi)) {
      bv = v2;
      bi = i2;
    }
  }
  v = bv;
  i = bi;
}

}  // namespace rb
