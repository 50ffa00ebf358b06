// Passes of at most 32 rows with half as many dependent kernels: a sub-layer is owned by head
// (attention) or by slice of the FFN width instead of by output column, so that a kernel ends only
// where a reduction over full rows cannot be avoided.
//
//   head kernel, self  : [sum of the previous sub-layer's slices, LayerNorm] -> this head's Q, K, V
//                        (K/V appended to the cache) -> attention of the head -> the head's 64-wide
//                        slice of the O-projection as a partial result [R][d]
//   head kernel, cross : the same with the cross-attention Q projection and the precomputed K/V
//   ffn kernel         : [sum, LayerNorm] -> a slice of W1 (+ReLU) -> the matching k slice of W2 as a
//                        partial result [R][d]
//
// The partial results of a kernel are summed, in a fixed order, by the prologue of the next one
// (sk_hidden_sum), which also adds bias and residual and applies the LayerNorm: results do not
// depend on scheduling.  Three kernels per decoder layer instead of six.
#include "skinny_core.h"

namespace sd {

constexpr int kHeadWaves = 12;     // one 16-column tile of the head's Q | K | V per wave
constexpr int kFfnWaves = 8;
constexpr int kAttPitch = 64 + 8;  // bf16 per row of the attention output tile in LDS

template <int PER>
struct Sk2Lds {   // hb [32][d+8] bf16 | hown (unused slices) | vs [waves][32][kVtPitch] | att [32][72]
  static constexpr int d = 64 * PER, kPitch = d + kSkPad;
  static constexpr size_t kHb = (size_t)kSkRows * kPitch * 2;
  static constexpr size_t kOwn = (size_t)2 * kSkRows * 16 * 4;
  static constexpr size_t kVs = (size_t)kHeadWaves * 32 * kVtPitch * 2;
  static constexpr size_t kAtt = (size_t)kSkRows * kAttPitch * 2;
  static constexpr size_t kBytes = kHb + kOwn + kVs + kAtt;
};

// SELF: Q | K | V of head blockIdx.x from W [3d][d] (rows part*d + h*64 + c), K/V appended, causal
// attention over the cache; else Q from W [d][d] and attention over the precomputed cross K/V.
// Wo [d][d]: the head's k range [64 h, 64 h + 64) -> part_out[h] [R][d] (no bias, no residual).
template <int PER, bool SELF, bool TWO>
__global__ __launch_bounds__(64 * kHeadWaves) void sk2_head_kernel(SkSrc src, int R, AttnArgs a,
                                                                   const bf16* __restrict__ W,
                                                                   const bf16* __restrict__ bias,
                                                                   bf16* __restrict__ q, bf16* __restrict__ kc,
                                                                   bf16* __restrict__ vc,
                                                                   const int* __restrict__ row_b,
                                                                   const int* __restrict__ row_pos, int Lcap,
                                                                   const bf16* __restrict__ Wo,
                                                                   float* __restrict__ part_out) {
  extern __shared__ __attribute__((aligned(16))) char sk_smem[];
  typedef Sk2Lds<PER> L;
  constexpr int d = L::d, pitch = L::kPitch, STEPS = d / 32;
  bf16* hb = reinterpret_cast<bf16*>(sk_smem);
  float* hown = reinterpret_cast<float*>(sk_smem + L::kHb);
  bf16(*vs)[32][kVtPitch] = reinterpret_cast<bf16(*)[32][kVtPitch]>(sk_smem + L::kHb + L::kOwn);
  bf16* att = reinterpret_cast<bf16*>(sk_smem + L::kHb + L::kOwn + L::kVs);
  const int h = blockIdx.x, H = a.H;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lq = lane & 15, g = lane >> 4;
  constexpr int NQKV = SELF ? 12 : 4;                 // projection column tiles of the head
  const bool pwave = wave < NQKV;
  const int prt = wave >> 2, cw = wave & 3;          // 0 q, 1 k, 2 v; 16-column tile inside the head
  const int nrow0 = prt * d + h * kHeadDim + cw * 16;   // first weight row of this wave's tile
  bf16x8 wf[STEPS];
  if (pwave) sk_wload<STEPS>(W, d, nrow0, SELF ? 3 * d : d, 0, wf);
  float bia[4];
  int rb[2] = {-1, -1}, rp[2] = {0, 0};
  if (pwave) {
#pragma unroll
    for (int r = 0; r < 4; ++r) bia[r] = (float)bias[nrow0 + 4 * g + r];
    if (SELF) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const int m = min(t * 16 + lq, R - 1);
        rb[t] = row_b[m]; rp[t] = row_pos[m];
      }
    }
  }
  if (src.np > 0) sk_hidden_sum<PER, kHeadWaves, 64>(src, R, TWO ? 32 : 16, hb, hown, -64, true, -64);
  else if (wave < 4) sk_hidden<PER>(src, R, TWO ? 32 : 16, hb, hown, -64, true);
  __syncthreads();
  if (pwave) {
    f32x4 acc[2];
    sk_zero(acc);
    sk_mma<STEPS, TWO>(wf, 0, [&](int t, int k) { return *reinterpret_cast<const bf16x8*>(hb + (t * 16 + lq) * pitch + k); }, acc);
    // this lane: activation row m = t*16 + lq, the tile's columns 4g .. 4g+3
#pragma unroll
    for (int t = 0; t < (TWO ? 2 : 1); ++t) {
      const int m = t * 16 + lq;
      if (m >= R) continue;
      const float v[4] = {acc[t][0] + bia[0], acc[t][1] + bia[1], acc[t][2] + bia[2], acc[t][3] + bia[3]};
      const int c = h * kHeadDim + cw * 16 + 4 * g;
      if (prt == 0) {
        st_coh4(q + (size_t)m * d + c, v);
      } else if (rb[t] >= 0) {
        bf16* cache = prt == 1 ? kc : vc;
        st_coh4(cache + (((size_t)rb[t] * H + h) * Lcap + rp[t]) * kHeadDim + cw * 16 + 4 * g, v);
      }
    }
  }
  // the head's slice of the output projection travels while the attention runs
  constexpr int OT = d / 16;                          // output column tiles
  constexpr int OPW = (OT + kHeadWaves - 1) / kHeadWaves;
  bf16x8 wo[OPW][2];
#pragma unroll
  for (int u = 0; u < OPW; ++u) {
    const int ct = min(wave + u * kHeadWaves, OT - 1);
    bf16x8 t2[2];
    sk_wload<2>(Wo, d, ct * 16, d, h * kHeadDim, t2);
    wo[u][0] = t2[0]; wo[u][1] = t2[1];
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // (also: this wave's Q / K / V stores are acknowledged)
  __syncthreads();
  // one (sequence, head) pair per wave
  for (int b = wave; b < a.B; b += kHeadWaves) {
    constexpr int NQT = TWO ? 2 : 1;
    int nq = min(a.q_count ? a.q_count[b] : a.T, 16 * NQT);
    float mrun[NQT], lrun[NQT];
    f32x4 oacc[NQT][4];
    attn_wave<NQT, !SELF, true, SELF>(a, b, h, 0, nq, 0, 1, vs[wave], mrun, lrun, oacc);
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
      const int qi = qt * 16 + lq;
      if (qi < nq) {
        const float inv = lrun[qt] > 0.f ? 1.f / lrun[qt] : 0.f;
        bf16* op = att + (b * a.T + qi) * kAttPitch;
#pragma unroll
        for (int et = 0; et < 4; ++et)
#pragma unroll
          for (int r = 0; r < 4; ++r) op[et * 16 + 4 * g + r] = (bf16)(oacc[qt][et][r] * inv);
      }
    }
  }
  __syncthreads();
  float* po = part_out + (size_t)h * kSkRows * d;
#pragma unroll
  for (int u = 0; u < OPW; ++u) {
    const int ct = wave + u * kHeadWaves;
    if (ct >= OT) break;
    f32x4 acc[2];
    sk_zero(acc);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const int k = ks * 32 + 8 * g;
      acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wo[u][ks], *reinterpret_cast<const bf16x8*>(att + lq * kAttPitch + k), acc[0], 0, 0, 0);
      if (TWO) acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wo[u][ks], *reinterpret_cast<const bf16x8*>(att + (16 + lq) * kAttPitch + k), acc[1], 0, 0, 0);
    }
    mfma_settle(acc[0], acc[1]);
#pragma unroll
    for (int t = 0; t < (TWO ? 2 : 1); ++t) {
      const int m = t * 16 + lq;
      if (m < R) *reinterpret_cast<f32x4*>(po + (size_t)m * d + ct * 16 + 4 * g) = acc[t];
    }
  }
}

// Slice s = blockIdx.x of the FFN width, FSL columns: hid = ReLU(hidden W1[s]^T + b1[s]) stays in LDS,
// part_out[s] = hid W2[:, s]^T  [R][d].
template <int PER, int FSL, bool TWO>
__global__ __launch_bounds__(64 * kFfnWaves) void sk2_ffn_kernel(SkSrc src, int R, const bf16* __restrict__ W1,
                                                                 const bf16* __restrict__ b1, int F,
                                                                 const bf16* __restrict__ W2,
                                                                 float* __restrict__ part_out) {
  extern __shared__ __attribute__((aligned(16))) char sk_smem[];
  constexpr int d = 64 * PER, pitch = d + kSkPad, STEPS = d / 32, HP = FSL + 8;
  bf16* hb = reinterpret_cast<bf16*>(sk_smem);
  float* hown = reinterpret_cast<float*>(sk_smem + (size_t)kSkRows * pitch * 2);
  bf16* hid = reinterpret_cast<bf16*>(sk_smem + (size_t)kSkRows * pitch * 2 + (size_t)2 * kSkRows * 16 * 4);   // [32][HP]
  const int f0 = blockIdx.x * FSL;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lq = lane & 15, g = lane >> 4;
  constexpr int HT = FSL / 16;                        // column tiles of the hidden slice
  bf16x8 wf[STEPS];
  const bool w1wave = wave < HT;
  if (w1wave) sk_wload<STEPS>(W1, d, f0 + wave * 16, F, 0, wf);
  if (src.np > 0) sk_hidden_sum<PER, kFfnWaves>(src, R, TWO ? 32 : 16, hb, hown, -64, true, -64);
  else if (wave < 4) sk_hidden<PER>(src, R, TWO ? 32 : 16, hb, hown, -64, true);
  __syncthreads();
  auto getH = [&](int t, int k) { return *reinterpret_cast<const bf16x8*>(hb + (t * 16 + lq) * pitch + k); };
  for (int ct = wave; ct < HT; ct += kFfnWaves) {
    if (ct != wave) sk_wload<STEPS>(W1, d, f0 + ct * 16, F, 0, wf);
    float bia[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) bia[r] = (float)b1[f0 + ct * 16 + 4 * g + r];
    f32x4 acc[2];
    sk_zero(acc);
    sk_mma<STEPS, TWO>(wf, 0, getH, acc);
#pragma unroll
    for (int t = 0; t < (TWO ? 2 : 1); ++t) {
      bf16x4 o;
#pragma unroll
      for (int r = 0; r < 4; ++r) o[r] = (bf16)fmaxf(acc[t][r] + bia[r], 0.f);
      *reinterpret_cast<bf16x4*>(hid + (t * 16 + lq) * HP + ct * 16 + 4 * g) = o;   // (rows >= R: unused)
    }
  }
  __syncthreads();
  constexpr int OT = d / 16, KS = FSL / 32;
  float* po = part_out + (size_t)blockIdx.x * kSkRows * d;
  for (int ct = wave; ct < OT; ct += kFfnWaves) {
    bf16x8 w2[KS];
    sk_wload<KS>(W2, F, ct * 16, d, f0, w2);
    f32x4 acc[2];
    sk_zero(acc);
    sk_mma<KS, TWO>(w2, 0, [&](int t, int k) { return *reinterpret_cast<const bf16x8*>(hid + (t * 16 + lq) * HP + k); }, acc);
#pragma unroll
    for (int t = 0; t < (TWO ? 2 : 1); ++t) {
      const int m = t * 16 + lq;
      if (m < R) *reinterpret_cast<f32x4*>(po + (size_t)m * d + ct * 16 + 4 * g) = acc[t];
    }
  }
}

// ------------------------------------------------------------------------------------ launchers
int sk2_ffn_slice(int F) { return F >= 4096 ? 256 : (F >= 2048 ? 128 : 32); }
int sk2_ffn_slices(int F) { return F / sk2_ffn_slice(F); }
bool sk2_supported(int d, int F) {
  return (d == 128 || d == 512 || d == 1024) && (F == 256 || F == 2048 || F == 4096);
}

#define SK2_DISPATCH(d, CALL)                     \
  switch ((d) / 64) {                             \
    case 2: { constexpr int PER = 2; CALL; } break;   \
    case 8: { constexpr int PER = 8; CALL; } break;   \
    case 16: { constexpr int PER = 16; CALL; } break; \
    default: return hipErrorInvalidValue;         \
  }
#define SK2_ROWS(R, CALL)                                       \
  if ((R) > 16) { constexpr bool TWO = true; CALL; }            \
  else { constexpr bool TWO = false; CALL; }

template <int PER, bool SELF, bool TWO>
static hipError_t sk2_head_launch(hipStream_t st, const SkSrc& src, int R, const AttnArgs& a, const bf16* W,
                                  const bf16* bias, bf16* q, bf16* kc, bf16* vc, const int* row_b, const int* row_pos,
                                  int Lcap, const bf16* Wo, float* part_out) {
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(sk2_head_kernel<PER, SELF, TWO>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)Sk2Lds<PER>::kBytes);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL((sk2_head_kernel<PER, SELF, TWO>), dim3(a.H), dim3(64 * kHeadWaves), Sk2Lds<PER>::kBytes, st, src, R, a,
                     W, bias, q, kc, vc, row_b, row_pos, Lcap, Wo, part_out);
  return hipGetLastError();
}
hipError_t skinny2_head(hipStream_t st, const SkSrc& src, int R, int d, const AttnArgs& a, bool self, const bf16* W,
                        const bf16* bias, bf16* q, bf16* kc, bf16* vc, const int* row_b, const int* row_pos, int Lcap,
                        const bf16* Wo, float* part_out) {
  if (self) {
    SK2_DISPATCH(d, SK2_ROWS(R, return (sk2_head_launch<PER, true, TWO>(st, src, R, a, W, bias, q, kc, vc, row_b, row_pos, Lcap, Wo, part_out))));
  } else {
    SK2_DISPATCH(d, SK2_ROWS(R, return (sk2_head_launch<PER, false, TWO>(st, src, R, a, W, bias, q, kc, vc, row_b, row_pos, Lcap, Wo, part_out))));
  }
  return hipErrorInvalidValue;
}

template <int PER, int FSL, bool TWO>
static hipError_t sk2_ffn_launch(hipStream_t st, const SkSrc& src, int R, const bf16* W1, const bf16* b1, int F,
                                 const bf16* W2, float* part_out) {
  constexpr int d = 64 * PER;
  constexpr size_t bytes = (size_t)kSkRows * (d + kSkPad) * 2 + (size_t)2 * kSkRows * 16 * 4 + (size_t)kSkRows * (FSL + 8) * 2;
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(sk2_ffn_kernel<PER, FSL, TWO>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL((sk2_ffn_kernel<PER, FSL, TWO>), dim3(F / FSL), dim3(64 * kFfnWaves), bytes, st, src, R, W1, b1, F, W2,
                     part_out);
  return hipGetLastError();
}
hipError_t skinny2_ffn(hipStream_t st, const SkSrc& src, int R, int d, const bf16* W1, const bf16* b1, int F,
                       const bf16* W2, float* part_out) {
  switch (sk2_ffn_slice(F)) {
    case 32: SK2_DISPATCH(d, SK2_ROWS(R, return (sk2_ffn_launch<PER, 32, TWO>(st, src, R, W1, b1, F, W2, part_out)))); break;
    case 128: SK2_DISPATCH(d, SK2_ROWS(R, return (sk2_ffn_launch<PER, 128, TWO>(st, src, R, W1, b1, F, W2, part_out)))); break;
    case 256: SK2_DISPATCH(d, SK2_ROWS(R, return (sk2_ffn_launch<PER, 256, TWO>(st, src, R, W1, b1, F, W2, part_out)))); break;
  }
  return hipErrorInvalidValue;
}

}  // namespace sd
