// Shared device helpers for the gfx950 kernels (wave size 64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// operands of __builtin_amdgcn_global_load_lds (global memory -> LDS without a register stop)
#define SD_LDS_PTR(p) ((void __attribute__((address_space(3)))*)(p))
#define SD_GLB_PTR(p) ((const void __attribute__((address_space(1)))*)(p))

namespace sd {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kHeadDim = 64;   // d_model = 64 * n_heads for every model in the paper's setups
constexpr float kNegInf = -__builtin_inff();

// Value caches are stored in blocks of 8 keys: element (key, e) of one (sequence, head) lies at
//   ((key / 8) * 64 + e) * 8 + key % 8
// so the 8 consecutive keys that one lane feeds to the P.V product are one 16-byte load, and
// the 64 dims of one key block are 1 KB contiguous.
__host__ __device__ __forceinline__ long vt_off(int key, int e) {
  return ((long)(key >> 3) * kHeadDim + e) * 8 + (key & 7);
}

// Wave-wide reductions; every lane receives the result.  The four steps inside a row of 16 lanes
// are DPP moves (swap neighbours, swap pairs, mirror halves of 8, mirror the row), which cost an
// ordinary vector instruction each and leave the row's result in all its lanes; the four row
// results are then read as scalars (v_readlane of lanes 0, 16, 32, 48) and combined in a fixed
// order, r0 + r1 + r2 + r3 from the left.  No step goes through LDS (ds_bpermute costs a round
// trip of its own, and a LayerNorm is two dependent reductions).
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
constexpr int kDppSwap1 = 0xB1, kDppSwap2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;

__device__ __forceinline__ float row_lane_f(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f<kDppSwap1>(v);
  v += dpp_f<kDppSwap2>(v);
  v += dpp_f<kDppHalfMirror>(v);
  v += dpp_f<kDppMirror>(v);
  return ((row_lane_f(v, 0) + row_lane_f(v, 16)) + row_lane_f(v, 32)) + row_lane_f(v, 48);
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_f<kDppSwap1>(v));
  v = fmaxf(v, dpp_f<kDppSwap2>(v));
  v = fmaxf(v, dpp_f<kDppHalfMirror>(v));
  v = fmaxf(v, dpp_f<kDppMirror>(v));
  return fmaxf(fmaxf(row_lane_f(v, 0), row_lane_f(v, 16)), fmaxf(row_lane_f(v, 32), row_lane_f(v, 48)));
}
__device__ __forceinline__ int wave_max_i(int v) {
  v = max(v, dpp_i<kDppSwap1>(v));
  v = max(v, dpp_i<kDppSwap2>(v));
  v = max(v, dpp_i<kDppHalfMirror>(v));
  v = max(v, dpp_i<kDppMirror>(v));
  return max(max(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
             max(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}

// 1 / sqrt(x) for a LayerNorm on a kernel's critical path: the hardware's reciprocal square root
// (1 ulp) with one Newton step, instead of the correctly rounded square root and division (several
// dozen instructions).
__device__ __forceinline__ float fast_rsqrt(float x) {
  const float r = __builtin_amdgcn_rsqf(x);
  return r * __builtin_fmaf(-0.5f * x * r, r, 1.5f);
}

// Workgroup barrier that orders LDS traffic only: __syncthreads() also waits for every global
// load in flight (vmcnt(0)), which serialises requests a kernel issued early on purpose.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Wait states between the last MFMA of a chain and ordinary vector instructions that read its
// result.  Seen on this toolchain: when a branch separates the two, the required wait states
// are not always inserted and the last result registers are read before they are written
// (wrong sums in columns 4g+2, 4g+3 of a 16x16 tile).  The asm statements below consume the
// accumulators, so they cannot move above the MFMAs, and hold 32 idle issue slots (the longest
// MFMA needs 19); whatever reads the accumulators afterwards reads settled registers.
__device__ __forceinline__ void mfma_settle(f32x4& a) { asm volatile("s_nop 15\n\ts_nop 15" : "+v"(a)); }
__device__ __forceinline__ void mfma_settle(f32x4& a, f32x4& b) {
  asm volatile("s_nop 15\n\ts_nop 15" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ void mfma_settle(f32x4 (&a)[4]) {
  asm volatile("s_nop 15\n\ts_nop 15" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]));
}
__device__ __forceinline__ void mfma_settle(f32x16& a) { asm volatile("s_nop 15\n\ts_nop 15" : "+v"(a)); }

// Accesses that are coherent among all workgroups of a running kernel: relaxed atomics at
// device scope go to the coherence point instead of the issuing CU's L1 / XCD's L2, so a
// value stored this way and acknowledged (s_waitcnt vmcnt(0)) is what a later load of this
// kind returns, on whichever XCD the two workgroups run.
__device__ __forceinline__ float ld_coh(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int ld_coh(const int* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ bf16x8 ld_coh16(const bf16* p) {   // 16 bytes, 8-byte aligned halves
  const unsigned long long* q = reinterpret_cast<const unsigned long long*>(p);
  unsigned long long u[2];
  u[0] = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  u[1] = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  bf16x8 v;
  __builtin_memcpy(&v, u, 16);
  return v;
}
__device__ __forceinline__ void st_coh(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_coh(bf16* p, bf16 v) {
  unsigned short bits;
  __builtin_memcpy(&bits, &v, 2);
  __hip_atomic_store(reinterpret_cast<unsigned short*>(p), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// FP8 E4M3 codes (OCP 8-bit float: 1-4-3, bias 7, largest value 448, no infinities) as stored
// weights / keys / values: eight codes are one operand fragment's worth.
typedef unsigned char fp8;
typedef unsigned int fp8x8 __attribute__((ext_vector_type(2)));
// Eight codes -> the bf16 operand of an MFMA: the hardware's E4M3 -> fp32 conversion, one code (byte
// select 0..3) per instruction; an E4M3 value has 3 mantissa bits, so the upper half of its fp32
// pattern IS its bf16 pattern, and v_perm packs two upper halves.
__device__ __forceinline__ bf16x8 e4m3x8_to_bf16(const fp8x8& f) {
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  u32x4 o;
#pragma unroll
  for (int w = 0; w < 2; ++w) {
    const unsigned c0 = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_f32_fp8((int)f[w], 0));
    const unsigned c1 = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_f32_fp8((int)f[w], 1));
    const unsigned c2 = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_f32_fp8((int)f[w], 2));
    const unsigned c3 = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_f32_fp8((int)f[w], 3));
    o[2 * w] = __builtin_amdgcn_perm(c1, c0, 0x07060302u);
    o[2 * w + 1] = __builtin_amdgcn_perm(c3, c2, 0x07060302u);
  }
  return __builtin_bit_cast(bf16x8, o);
}

template <bool COH>
__device__ __forceinline__ bf16x8 ld16(const bf16* p) {
  if (COH) return ld_coh16(p);
  return *reinterpret_cast<const bf16x8*>(p);
}

}  // namespace sd
