// Scaled dot-product attention for few queries against a streamed key/value set.
//
// One block = one (sequence, head, group of up to 64 queries).  Keys and values are streamed
// once per block in chunks of 64 rows through LDS and shared by all its queries; every query
// keeps an online softmax (running max, running sum, 64-wide accumulator with one output
// dimension per lane).  A query sees keys [0, limit): this covers the causal verify pass
// (limit grows by one per row), the drafter's mask slots (limit = whole block) and padded
// cross-attention / encoder attention (limit = source length).
#include "common.h"
#include "kernels.h"

namespace sd {

constexpr int kAttnThreads = 256;
constexpr int kQPerBlock = 64;
constexpr int kQPerWave = kQPerBlock / 4;
constexpr int kKPitch = 65;   // fp32 row pitch of the key tile: lane = key reads hit 64 banks

__global__ __launch_bounds__(kAttnThreads) void attn_kernel(AttnArgs a) {
  __shared__ float Qs[kQPerBlock][kHeadDim];
  __shared__ float Ks[64][kKPitch];
  __shared__ float Vs[64][kHeadDim];
  __shared__ int Lim[kQPerBlock];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.z, h = blockIdx.y, q0 = blockIdx.x * kQPerBlock;
  const int nq_seq = a.q_count ? a.q_count[b] : a.T;
  const int nq = min(nq_seq - q0, kQPerBlock);
  if (nq <= 0) return;

  if (tid < kQPerBlock) {
    int lim = 0;
    if (tid < nq) lim = a.lim_row ? a.lim_row[b * a.T + q0 + tid] : a.lim_seq[b];
    Lim[tid] = lim;
  }
  // queries -> LDS as fp32, pre-scaled by 1/sqrt(64)
  for (int idx = tid; idx < kQPerBlock * 8; idx += kAttnThreads) {
    int qi = idx >> 3, ch = idx & 7;
    float f[8];
    if (qi < nq) {
      bf16x8 v = *reinterpret_cast<const bf16x8*>(a.q + b * a.q_b + (long)(q0 + qi) * a.q_row + h * kHeadDim + ch * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] = (float)v[e] * 0.125f;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] = 0.f;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) Qs[qi][ch * 8 + e] = f[e];
  }
  __syncthreads();
  int kmax = 0;
  {
    int l = lane < kQPerBlock ? Lim[lane] : 0;
    kmax = wave_max_i(l);
  }

  float mrun[kQPerWave], lrun[kQPerWave], acc[kQPerWave];
#pragma unroll
  for (int j = 0; j < kQPerWave; ++j) { mrun[j] = kNegInf; lrun[j] = 0.f; acc[j] = 0.f; }

  const bf16* kbase = a.k + b * a.kv_b + h * a.kv_h;
  const bf16* vbase = a.v + b * a.kv_b + h * a.kv_h;

  for (int c0 = 0; c0 < kmax; c0 += 64) {
    // stage 64 keys and 64 values (rows beyond kmax are zero: they may hold anything)
    for (int idx = tid; idx < 64 * 8; idx += kAttnThreads) {
      int key = idx >> 3, ch = idx & 7;
      float fk[8], fv[8];
      if (c0 + key < kmax) {
        bf16x8 kk = *reinterpret_cast<const bf16x8*>(kbase + (long)(c0 + key) * a.kv_row + ch * 8);
        bf16x8 vv = *reinterpret_cast<const bf16x8*>(vbase + (long)(c0 + key) * a.kv_row + ch * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) { fk[e] = (float)kk[e]; fv[e] = (float)vv[e]; }
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) { fk[e] = 0.f; fv[e] = 0.f; }
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) { Ks[key][ch * 8 + e] = fk[e]; Vs[key][ch * 8 + e] = fv[e]; }
    }
    __syncthreads();

#pragma unroll
    for (int j = 0; j < kQPerWave; ++j) {
      const int qi = wave + 4 * j;          // wave-uniform
      if (qi < nq) {
        const int lim = Lim[qi];
        if (c0 < lim) {
          // lane = key: score
          float s = 0.f;
#pragma unroll 16
          for (int e = 0; e < kHeadDim; ++e) s += Qs[qi][e] * Ks[lane][e];
          const bool valid = (c0 + lane) < lim;
          s = valid ? s : kNegInf;
          float cm = wave_max(s);           // finite: key c0 is visible
          float mnew = fmaxf(mrun[j], cm);
          float p = valid ? __expf(s - mnew) : 0.f;
          float alpha = __expf(mrun[j] - mnew);   // exp(-inf) = 0 on the first chunk
          lrun[j] = lrun[j] * alpha + wave_sum(p);
          mrun[j] = mnew;
          // lane = output dimension: acc += sum_key p[key] * V[key][lane]
          float o = acc[j] * alpha;
#pragma unroll
          for (int key = 0; key < 64; ++key) o += __shfl(p, key, 64) * Vs[key][lane];
          acc[j] = o;
        }
      }
    }
    __syncthreads();
  }

#pragma unroll
  for (int j = 0; j < kQPerWave; ++j) {
    const int qi = wave + 4 * j;
    if (qi < nq) {
      float o = lrun[j] > 0.f ? acc[j] / lrun[j] : 0.f;
      a.o[b * a.o_b + (long)(q0 + qi) * a.o_row + h * kHeadDim + lane] = (bf16)o;
    }
  }
}

hipError_t attention(hipStream_t st, const AttnArgs& a) {
  if (a.B <= 0 || a.T <= 0) return hipSuccess;
  dim3 grid((a.T + kQPerBlock - 1) / kQPerBlock, a.H, a.B);
  hipLaunchKernelGGL(attn_kernel, grid, dim3(kAttnThreads), 0, st, a);
  return hipGetLastError();
}

}  // namespace sd
