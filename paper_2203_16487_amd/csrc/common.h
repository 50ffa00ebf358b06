// Shared device helpers for the gfx950 kernels (wave size 64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sd {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kHeadDim = 64;   // d_model = 64 * n_heads for every model in the paper's setups
constexpr int kTopN = 8;       // depth of the per-row top lists (SPECDEC_BETA_MAX)
constexpr float kNegInf = -__builtin_inff();

// Value caches are stored in blocks of 8 keys: element (key, e) of one (sequence, head) lies at
//   ((key / 8) * 64 + e) * 8 + key % 8
// so the 8 consecutive keys that one lane feeds to the P.V product are one 16-byte load, and
// the 64 dims of one key block are 1 KB contiguous.
__host__ __device__ __forceinline__ long vt_off(int key, int e) {
  return ((long)(key >> 3) * kHeadDim + e) * 8 + (key & 7);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ int wave_max_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o, 64));
  return v;
}

// Insert v into a descending list t[0..N) (keeps the N largest, duplicates kept).
template <int N>
__device__ __forceinline__ void top_insert(float (&t)[N], float v) {
  if (v > t[N - 1]) {
    t[N - 1] = v;
#pragma unroll
    for (int i = N - 1; i > 0; --i) {
      float hi = fmaxf(t[i - 1], t[i]);
      float lo = fminf(t[i - 1], t[i]);
      t[i - 1] = hi;
      t[i] = lo;
    }
  }
}

}  // namespace sd
