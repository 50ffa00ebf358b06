// Wave-level attention core shared by the attention kernel and the fused small-batch kernels.
#pragma once
#include "common.h"
#include "kernels.h"

namespace sd {

__device__ __forceinline__ bf16x8 zero_tail(bf16x8 v, int nvalid) {
  // keep elements [0, nvalid), zero the rest (values beyond a sequence's keys may be anything)
  bf16x8 o;
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = (i < nvalid) ? v[i] : (bf16)0.f;
  return o;
}

constexpr int kVtPitch = 68;   // bf16 per staged value row: 34 banks, so the transposed 2-byte
                               // reads of the four lane groups (8 rows apart) hit disjoint banks

// One wave, one (sequence b, head h) pair, queries q0 .. q0 + nq - 1 (nq <= 16*NQT) against the
// key chunks kw, kw + kstep, ... of 32 keys.  Results: running max / sum per query (lane%16
// of tile qt) and the unnormalised O^T accumulators oacc[qt][et][r] = O^T[e = et*16 + 4*(lane/16)
// + r][q = qt*16 + lane%16].  Vs: wave-private LDS tile [32][kVtPitch] (row-layout values only).
// COHQ / COHKV: queries / keys and row-layout values may have been written by other workgroups
// of the running kernel (coherent loads, see ld16).
template <int NQT, bool VBLK, bool COHQ = false, bool COHKV = false>
__device__ __forceinline__ void attn_wave(const AttnArgs& a, int b, int h, int q0, int nq, int kw, int kstep,
                                          bf16 (*Vs)[kVtPitch], float (&mrun)[NQT], float (&lrun)[NQT],
                                          f32x4 (&oacc)[NQT][4]) {
  const int lane = threadIdx.x & 63;
  const int lq = lane & 15, g = lane >> 4;
  const bf16* kbase = a.k + b * a.k_b + h * a.k_h;
  const bf16* vbase = a.v + b * a.v_b + h * a.v_h;

  // operands of one 32-key chunk (8 x 16 B per lane), key rows clamped to `last`; the next
  // chunk is fetched while the current one is multiplied
  auto load_chunk = [&](int c0, int last, bf16x8 (&kf)[2][2], bf16x8 (&vf)[4]) {
    // K operands: tile t, row lq  <->  key c0 + 8*(lq/4) + 4*t + lq%4
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int key = min(c0 + 8 * (lq >> 2) + 4 * t + (lq & 3), last);
      const bf16* kp = kbase + (long)key * a.k_row + g * 8;
      kf[t][0] = ld16<COHKV>(kp);
      kf[t][1] = ld16<COHKV>(kp + 32);
    }
    if (VBLK) {
      // V operands: dim e = et*16 + lq, keys kb .. kb+7 = one block of the key-blocked layout
      const int kb = min(c0 + 8 * g, a.cap - 8);
#pragma unroll
      for (int et = 0; et < 4; ++et)
        vf[et] = *reinterpret_cast<const bf16x8*>(vbase + vt_off(kb, et * 16 + lq));
    } else {
      // row layout: fetch 32 whole rows (lane -> row 8*i + lane/8, dims 8*(lane%8) .. +7); they
      // are turned into operands through LDS when the chunk is used
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int key = min(c0 + 8 * i + (lane >> 3), last);
        vf[i] = ld16<COHKV>(vbase + (long)key * a.v_row + (lane & 7) * 8);
      }
    }
  };
  // The first chunk is requested before the limits are known (its addresses depend on no
  // loaded value: rows are clamped to the arena, whose every row may be read; keys past a
  // query's limit are masked by selection and their values zeroed), so limits, queries, keys
  // and values of a short context arrive in one memory round trip.
  bf16x8 kf[2][2], vf[4], kn[2][2], vn[4];
  const int cfirst = kw * 32, cstep = kstep * 32;
  load_chunk(cfirst, a.cap - 1, kf, vf);

  // this lane's queries: q0 + qt*16 + lq; limits and Q operands (pre-scaled by 1/sqrt(64))
  int lim[NQT];
  bf16x8 qf[NQT][2];
  int kmax = 0;
  const bf16* qbase = a.q_off ? a.q + (long)a.q_off[b] * a.q_row : a.q + b * a.q_b;
  const int lbase = a.q_off ? a.q_off[b] : b * a.T;
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    const int qi = qt * 16 + lq;
    const bool ok = qi < nq;
    lim[qt] = ok ? (a.lim_row ? a.lim_row[lbase + q0 + qi] : a.lim_seq[b]) : 0;
    kmax = max(kmax, lim[qt]);
    const bf16* qp = qbase + (long)(q0 + (ok ? qi : 0)) * a.q_row + h * kHeadDim + g * 8;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      bf16x8 v = ld16<COHQ>(qp + ks * 32);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = (bf16)((float)v[e] * 0.125f);   // exact: power of two
      qf[qt][ks] = v;
    }
  }
  kmax = wave_max_i(kmax);

#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    mrun[qt] = kNegInf; lrun[qt] = 0.f;
#pragma unroll
    for (int et = 0; et < 4; ++et) oacc[qt][et] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  const int kclamp = max(kmax - 1, 0);

  for (int c0 = cfirst; c0 < kmax; c0 += cstep) {
    const bool more = c0 + cstep < kmax;
    if (more) load_chunk(c0 + cstep, kclamp, kn, vn);
    if (!VBLK) {
      // wave-private transposition: rows -> LDS -> (dim, 8 consecutive keys) operands
      // (LDS operations of one wave execute in order, so no barrier is needed; memcpy keeps
      // the 16-byte store and the 2-byte loads in one alias class for the compiler)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        __builtin_memcpy(&Vs[8 * i + (lane >> 3)][(lane & 7) * 8], &vf[i], 16);
#pragma unroll
      for (int et = 0; et < 4; ++et)
#pragma unroll
        for (int i = 0; i < 8; ++i) vf[et][i] = Vs[8 * g + i][et * 16 + lq];
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
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) mfma_settle(oacc[qt]);
}

}  // namespace sd
