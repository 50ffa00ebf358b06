// Scaled dot-product attention for few queries against a streamed key/value set, on MFMA.
//
// A wave owns one (sequence, head) pair and a group of up to 16*NQT queries; it walks the keys
// in chunks of 32 with an online softmax.  Query, key and blocked-value operands are 16-byte
// global loads in exactly the register layout the instruction wants.
//
//   S^T[key][q]  = sum_e K[key][e] Q[q][e]        mfma 16x16x32: A = key rows, B = query rows
//   O^T[e][q]   += sum_key V^T[e][key] P^T[key][q] mfma 16x16x32: A = V^T rows, B = P (registers)
//
// Row i of key tile t stands for key c0 + 8*(i/4) + 4*t + i%4, so that the eight scores a lane
// holds after the two S^T tiles (q = lane%16, keys c0 + 8*(lane/16) .. +7) are already the B
// operand of the second product, and its V^T operand is one contiguous 16-byte load.  This is
// what the key-blocked value layout (vt_off) of the cross-attention values is for; values in
// row layout (the self-attention cache, appended row by row) are turned around through a
// wave-private LDS tile instead.  Both results keep q = lane%16, so the running max / sum of
// a query live in the lanes that hold its accumulators.
//
// A query sees keys [0, limit): causal verify rows (limit grows by one per row), the
// drafter's mask slots (limit = whole block), padded cross / encoder attention (limit = source
// length).  With key_split the 4 waves of a block share one pair and take every 4th chunk;
// their partial (max, sum, O) are merged through LDS.
#include "attn_core.h"

namespace sd {

constexpr int kAttnThreads = 256;

template <int NQT, bool VBLK, bool KV8>
__global__ __launch_bounds__(kAttnThreads) void attn_kernel(AttnArgs a) {
  __shared__ float Om[4][NQT * 16][kHeadDim + 1];
  __shared__ float Ms[4][NQT * 16], Ls[4][NQT * 16];
  __shared__ __attribute__((aligned(16))) bf16 Vs[VBLK ? 1 : 4][VBLK ? 1 : 32][kVtPitch];

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lq = lane & 15, g = lane >> 4;
  const int qgroups = (a.T + NQT * 16 - 1) / (NQT * 16);
  int pair, q0, kw, kstep;
  if (a.key_split) {
    pair = blockIdx.x / qgroups; q0 = (blockIdx.x % qgroups) * NQT * 16; kw = wave; kstep = 4;
  } else {
    const int u = blockIdx.x * 4 + wave;
    pair = u / qgroups; q0 = (u % qgroups) * NQT * 16; kw = 0; kstep = 1;
  }
  const bool active_pair = pair < a.B * a.H;
  const int b = active_pair ? pair / a.H : 0, h = active_pair ? pair % a.H : 0;
  float mrun[NQT], lrun[NQT];
  f32x4 oacc[NQT][4];
  int nq = active_pair ? -1 : 0;   // -1: the pair's query count is read inside, after the first requests
  attn_wave<NQT, VBLK, false, false, KV8>(a, b, h, q0, nq, kw, kstep, Vs[VBLK ? 0 : wave], mrun, lrun, oacc);
  bf16* obase = a.q_off ? a.o + (long)(active_pair ? a.q_off[b] : 0) * a.o_row : a.o + b * a.o_b;

  // oacc[qt][et][r] = O^T[e = et*16 + 4g + r][q = qt*16 + lq]
  if (!a.key_split) {
    if (!active_pair) return;
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
      const int qi = qt * 16 + lq;
      if (qi < nq) {
        const float inv = lrun[qt] > 0.f ? 1.f / lrun[qt] : 0.f;
        bf16* op = obase + (long)(q0 + qi) * a.o_row + h * kHeadDim;
#pragma unroll
        for (int et = 0; et < 4; ++et) {
          bf16x4 w;
#pragma unroll
          for (int r = 0; r < 4; ++r) w[r] = (bf16)(oacc[qt][et][r] * inv);
          *reinterpret_cast<bf16x4*>(op + et * 16 + 4 * g) = w;
        }
      }
    }
    return;
  }
  // merge the four key splits
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    const int qi = qt * 16 + lq;
    if (g == 0) { Ms[wave][qi] = mrun[qt]; Ls[wave][qi] = lrun[qt]; }
#pragma unroll
    for (int et = 0; et < 4; ++et)
#pragma unroll
      for (int r = 0; r < 4; ++r) Om[wave][qi][et * 16 + 4 * g + r] = oacc[qt][et][r];
  }
  __syncthreads();
  for (int idx = tid; idx < NQT * 16 * kHeadDim; idx += kAttnThreads) {
    const int qi = idx >> 6, e = idx & 63;
    if (qi < nq) {
      float M = kNegInf;
#pragma unroll
      for (int w = 0; w < 4; ++w) M = fmaxf(M, Ms[w][qi]);
      float L = 0.f, O = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float mw = Ms[w][qi];
        const float f = (mw > kNegInf) ? __expf(mw - M) : 0.f;
        L += Ls[w][qi] * f;
        O += Om[w][qi][e] * f;
      }
      obase[(long)(q0 + qi) * a.o_row + h * kHeadDim + e] = (bf16)(L > 0.f ? O / L : 0.f);
    }
  }
}

template <bool VBLK, bool KV8>
static hipError_t attention_launch(hipStream_t st, const AttnArgs& a) {
  const int nqt = a.T <= 16 ? 1 : (a.T <= 32 ? 2 : 4);
  const int qgroups = (a.T + nqt * 16 - 1) / (nqt * 16);
  const long units = (long)a.B * a.H * qgroups;
  const unsigned blocks = (unsigned)(a.key_split ? units : (units + 3) / 4);
  if (nqt == 1) SD_LAUNCH_TIMED((attn_kernel<1, VBLK, KV8>), dim3(blocks), dim3(kAttnThreads), 0, st, a);
  else if (nqt == 2) SD_LAUNCH_TIMED((attn_kernel<2, VBLK, KV8>), dim3(blocks), dim3(kAttnThreads), 0, st, a);
  else SD_LAUNCH_TIMED((attn_kernel<4, VBLK, KV8>), dim3(blocks), dim3(kAttnThreads), 0, st, a);
  return hipGetLastError();
}

hipError_t attention(hipStream_t st, const AttnArgs& a) {
  if (a.B <= 0 || a.T <= 0) return hipSuccess;
  if (a.cap < 32 || a.cap % 32 != 0) return hipErrorInvalidValue;   // whole chunks are read
  if (a.k_scale || a.v_scale) {   // FP8 keys and values
    if (!a.k_scale || !a.v_scale || !a.v_blocked) return hipErrorInvalidValue;
    return attention_launch<true, true>(st, a);
  }
  return a.v_blocked ? attention_launch<true, false>(st, a) : attention_launch<false, false>(st, a);
}

}  // namespace sd
