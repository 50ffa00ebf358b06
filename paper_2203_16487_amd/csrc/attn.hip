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
#include "common.h"
#include "kernels.h"

namespace sd {

constexpr int kAttnThreads = 256;

__device__ __forceinline__ bf16x8 zero_tail(bf16x8 v, int nvalid) {
  // keep elements [0, nvalid), zero the rest (values beyond a sequence's keys may be anything)
  bf16x8 o;
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = (i < nvalid) ? v[i] : (bf16)0.f;
  return o;
}

constexpr int kVtPitch = 68;   // bf16 per staged value row: 34 banks, so the transposed 2-byte
                               // reads of the four lane groups (8 rows apart) hit disjoint banks

template <int NQT, bool VBLK>
__global__ __launch_bounds__(kAttnThreads) void attn_kernel(AttnArgs a) {
  __shared__ float Om[4][NQT * 16][kHeadDim + 1];
  __shared__ float Ms[4][NQT * 16], Ls[4][NQT * 16];
  __shared__ __attribute__((aligned(16))) bf16 Vs[VBLK ? 1 : 4][VBLK ? 1 : 32][kVtPitch];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
  const int nq_seq = a.q_count ? a.q_count[b] : a.T;
  const int nq = active_pair ? min(nq_seq - q0, NQT * 16) : 0;

  // this lane's queries: q0 + qt*16 + lq; limits and Q operands (pre-scaled by 1/sqrt(64))
  int lim[NQT];
  bf16x8 qf[NQT][2];
  int kmax = 0;
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    const int qi = qt * 16 + lq;
    const bool ok = qi < nq;
    lim[qt] = ok ? (a.lim_row ? a.lim_row[b * a.T + q0 + qi] : a.lim_seq[b]) : 0;
    kmax = max(kmax, lim[qt]);
    const bf16* qp = a.q + b * a.q_b + (long)(q0 + (ok ? qi : 0)) * a.q_row + h * kHeadDim + g * 8;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      bf16x8 v = *reinterpret_cast<const bf16x8*>(qp + ks * 32);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = (bf16)((float)v[e] * 0.125f);   // exact: power of two
      qf[qt][ks] = v;
    }
  }
  kmax = wave_max_i(kmax);

  float mrun[NQT], lrun[NQT];
  f32x4 oacc[NQT][4];
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    mrun[qt] = kNegInf; lrun[qt] = 0.f;
#pragma unroll
    for (int et = 0; et < 4; ++et) oacc[qt][et] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  const bf16* kbase = a.k + b * a.k_b + h * a.k_h;
  const bf16* vbase = a.v + b * a.v_b + h * a.v_h;
  const int kclamp = max(kmax - 1, 0);

  // operands of one 32-key chunk (8 x 16 B per lane); the next chunk is fetched while the
  // current one is multiplied, so a wave pays the memory latency once, not once per chunk
  auto load_chunk = [&](int c0, bf16x8 (&kf)[2][2], bf16x8 (&vf)[4]) {
    // K operands: tile t, row lq  <->  key c0 + 8*(lq/4) + 4*t + lq%4
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int key = min(c0 + 8 * (lq >> 2) + 4 * t + (lq & 3), kclamp);
      const bf16* kp = kbase + (long)key * a.k_row + g * 8;
      kf[t][0] = *reinterpret_cast<const bf16x8*>(kp);
      kf[t][1] = *reinterpret_cast<const bf16x8*>(kp + 32);
    }
    if (VBLK) {
      // V operands: dim e = et*16 + lq, keys c0 + 8g .. +7 = one block of the key-blocked layout
#pragma unroll
      for (int et = 0; et < 4; ++et)
        vf[et] = *reinterpret_cast<const bf16x8*>(vbase + vt_off(c0 + 8 * g, et * 16 + lq));
    } else {
      // row layout: fetch 32 whole rows (lane -> row 8*i + lane/8, dims 8*(lane%8) .. +7); they
      // are turned into operands through LDS when the chunk is used
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int key = min(c0 + 8 * i + (lane >> 3), kclamp);
        vf[i] = *reinterpret_cast<const bf16x8*>(vbase + (long)key * a.v_row + (lane & 7) * 8);
      }
    }
  };
  bf16x8 kf[2][2], vf[4], kn[2][2], vn[4];
  const int cfirst = kw * 32, cstep = kstep * 32;
  if (cfirst < kmax) load_chunk(cfirst, kf, vf);

  for (int c0 = cfirst; c0 < kmax; c0 += cstep) {
    const bool more = c0 + cstep < kmax;
    if (more) load_chunk(c0 + cstep, kn, vn);
    if (!VBLK) {
      // wave-private transposition: rows -> LDS -> (dim, 8 consecutive keys) operands
      // (LDS operations of one wave execute in order, so no barrier is needed; memcpy keeps
      // the 16-byte store and the 2-byte loads in one alias class for the compiler)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        __builtin_memcpy(&Vs[wave][8 * i + (lane >> 3)][(lane & 7) * 8], &vf[i], 16);
#pragma unroll
      for (int et = 0; et < 4; ++et)
#pragma unroll
        for (int i = 0; i < 8; ++i) vf[et][i] = Vs[wave][8 * g + i][et * 16 + lq];
    }
    if (c0 + 32 > kmax) {
      const int nvalid = kmax - (c0 + 8 * g);
#pragma unroll
      for (int et = 0; et < 4; ++et) vf[et] = zero_tail(vf[et], nvalid);
    }
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
      f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[0][0], qf[qt][0], s0, 0, 0, 0);
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[0][1], qf[qt][1], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[1][0], qf[qt][0], s1, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[1][1], qf[qt][1], s1, 0, 0, 0);
      // this lane: query lq of tile qt, keys kb .. kb+7 = {s0[0..3], s1[0..3]}
      const int kb = c0 + 8 * g;
      float s[8];
      float cm = kNegInf;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        s[r] = (kb + r < lim[qt]) ? s0[r] : kNegInf;
        s[4 + r] = (kb + 4 + r < lim[qt]) ? s1[r] : kNegInf;
      }
#pragma unroll
      for (int r = 0; r < 8; ++r) cm = fmaxf(cm, s[r]);
      cm = fmaxf(cm, __shfl_xor(cm, 16, 64));
      cm = fmaxf(cm, __shfl_xor(cm, 32, 64));
      const float mnew = fmaxf(mrun[qt], cm);
      const bool any = mnew > kNegInf;
      const float alpha = any ? __expf(mrun[qt] - mnew) : 1.f;   // exp(-inf) = 0 on first use
      float ps = 0.f;
      bf16x8 pf;
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        float p = (any && s[r] > kNegInf) ? __expf(s[r] - mnew) : 0.f;
        ps += p;
        pf[r] = (bf16)p;
      }
      ps += __shfl_xor(ps, 16, 64);
      ps += __shfl_xor(ps, 32, 64);
      lrun[qt] = lrun[qt] * alpha + ps;
      mrun[qt] = mnew;
#pragma unroll
      for (int et = 0; et < 4; ++et) {
#pragma unroll
        for (int r = 0; r < 4; ++r) oacc[qt][et][r] *= alpha;
        oacc[qt][et] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[et], pf, oacc[qt][et], 0, 0, 0);
      }
    }
    if (more) {
#pragma unroll
      for (int t = 0; t < 2; ++t) { kf[t][0] = kn[t][0]; kf[t][1] = kn[t][1]; }
#pragma unroll
      for (int et = 0; et < 4; ++et) vf[et] = vn[et];
    }
  }

  // oacc[qt][et][r] = O^T[e = et*16 + 4g + r][q = qt*16 + lq]
  if (!a.key_split) {
    if (!active_pair) return;
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
      const int qi = qt * 16 + lq;
      if (qi < nq) {
        const float inv = lrun[qt] > 0.f ? 1.f / lrun[qt] : 0.f;
        bf16* op = a.o + b * a.o_b + (long)(q0 + qi) * a.o_row + h * kHeadDim;
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
      a.o[b * a.o_b + (long)(q0 + qi) * a.o_row + h * kHeadDim + e] = (bf16)(L > 0.f ? O / L : 0.f);
    }
  }
}

template <bool VBLK>
static hipError_t attention_launch(hipStream_t st, const AttnArgs& a) {
  const int nqt = a.T <= 16 ? 1 : (a.T <= 32 ? 2 : 4);
  const int qgroups = (a.T + nqt * 16 - 1) / (nqt * 16);
  const long units = (long)a.B * a.H * qgroups;
  const unsigned blocks = (unsigned)(a.key_split ? units : (units + 3) / 4);
  if (nqt == 1) hipLaunchKernelGGL((attn_kernel<1, VBLK>), dim3(blocks), dim3(kAttnThreads), 0, st, a);
  else if (nqt == 2) hipLaunchKernelGGL((attn_kernel<2, VBLK>), dim3(blocks), dim3(kAttnThreads), 0, st, a);
  else hipLaunchKernelGGL((attn_kernel<4, VBLK>), dim3(blocks), dim3(kAttnThreads), 0, st, a);
  return hipGetLastError();
}

hipError_t attention(hipStream_t st, const AttnArgs& a) {
  if (a.B <= 0 || a.T <= 0) return hipSuccess;
  return a.v_blocked ? attention_launch<true>(st, a) : attention_launch<false>(st, a);
}

}  // namespace sd
