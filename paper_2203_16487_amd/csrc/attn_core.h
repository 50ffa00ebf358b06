// Wave-level attention core shared by the attention kernel and the fused small-batch kernels.
#pragma once
#include <type_traits>
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

// One wave, one (sequence b, head h) pair, queries q0 .. q0 + nq - 1 (nq <= 16*NQT; nq < 0 on entry: what
// a.q_count leaves of the group, read here so that no request waits for it, and returned) against the
// key chunks kw, kw + kstep, ... of 32 keys.  Results: running max / sum per query (lane%16
// of tile qt) and the unnormalised O^T accumulators oacc[qt][et][r] = O^T[e = et*16 + 4*(lane/16)
// + r][q = qt*16 + lane%16].  Vs: wave-private LDS tile [32][kVtPitch] (row-layout values only).
// COHQ / COHKV: queries / keys and row-layout values may have been written by other workgroups
// of the running kernel (coherent loads, see ld16).
// QOFF = false: the caller never sets a.q_off (rows b*T .. of sequence b): no request depends on a loaded value.
// KV8 (key-blocked values only): keys and values are E4M3 codes with one fp32 scale per key and head;
// fragments are half as wide, become bf16 operands in registers, and the scales go where they
// factor out: score[key] = k_scale[key] * (codes . q), O += (p[key] * v_scale[key]) * codes.
template <bool KV8> struct AttnFrag { typedef bf16x8 type; };
template <> struct AttnFrag<true> { typedef fp8x8 type; };
__device__ __forceinline__ bf16x8 attn_operand(const bf16x8& f) { return f; }
__device__ __forceinline__ bf16x8 attn_operand(const fp8x8& f) { return e4m3x8_to_bf16(f); }

template <int NQT, bool VBLK, bool COHQ = false, bool COHKV = false, bool KV8 = false, bool QOFF = true>
__device__ __forceinline__ void attn_wave(const AttnArgs& a, int b, int h, int q0, int& nq, int kw, int kstep,
                                          bf16 (*Vs)[kVtPitch], float (&mrun)[NQT], float (&lrun)[NQT],
                                          f32x4 (&oacc)[NQT][4]) {
  const int lane = threadIdx.x & 63;
  const int lq = lane & 15, g = lane >> 4;
  // the pair and its query group are the same for the whole wave: say so, and per-sequence values are
  // read with scalar loads (no vector-memory wait stands between them and the requests that follow)
  b = __builtin_amdgcn_readfirstlane(b);
  h = __builtin_amdgcn_readfirstlane(h);
  q0 = __builtin_amdgcn_readfirstlane(q0);
  static_assert(!KV8 || (VBLK && !COHKV), "FP8 keys / values: cross-attention arenas only");
  typedef typename AttnFrag<KV8>::type Frag;
  typedef typename std::conditional<KV8, fp8, bf16>::type Elem;
  const Elem* kbase = reinterpret_cast<const Elem*>(a.k) + b * a.k_b + h * a.k_h;
  const Elem* vbase = reinterpret_cast<const Elem*>(a.v) + b * a.v_b + h * a.v_h;
  const float* ksc = KV8 ? a.k_scale + (b * a.k_b + h * a.k_h) / kHeadDim : nullptr;
  const float* vsc = KV8 ? a.v_scale + (b * a.v_b + h * a.v_h) / kHeadDim : nullptr;
  typedef float f32x4s __attribute__((ext_vector_type(4)));
  struct Scales { f32x4s k[2], v[2]; };   // of keys c0 + 8*(lane/16) .. + 7 (this lane's eight scores)

  // operands of one 32-key chunk (8 x 16 B per lane), key rows clamped to `last`; the next
  // chunk is fetched while the current one is multiplied
  auto load_chunk = [&](int c0, int last, Frag (&kf)[2][2], Frag (&vf)[4], Scales& sc) {
    // K operands: tile t, row lq  <->  key c0 + 8*(lq/4) + 4*t + lq%4
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int key = min(c0 + 8 * (lq >> 2) + 4 * t + (lq & 3), last);
      const Elem* kp = kbase + (long)key * a.k_row + g * 8;
      if constexpr (KV8) {
        kf[t][0] = *reinterpret_cast<const fp8x8*>(kp);
        kf[t][1] = *reinterpret_cast<const fp8x8*>(kp + 32);
      } else {
        kf[t][0] = ld16<COHKV>(kp);
        kf[t][1] = ld16<COHKV>(kp + 32);
      }
    }
    if constexpr (KV8) {
      const int kb = min(c0 + 8 * g, a.cap - 8);
#pragma unroll
      for (int et = 0; et < 4; ++et)
        vf[et] = *reinterpret_cast<const fp8x8*>(vbase + vt_off(kb, et * 16 + lq));
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        sc.k[i] = *reinterpret_cast<const f32x4s*>(ksc + kb + 4 * i);
        sc.v[i] = *reinterpret_cast<const f32x4s*>(vsc + kb + 4 * i);
      }
    } else if constexpr (VBLK) {
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
        if constexpr (!KV8) vf[i] = ld16<COHKV>(vbase + (long)key * a.v_row + (lane & 7) * 8);
      }
    }
  };
  // The first chunk is requested before the limits are known (its addresses depend on no
  // loaded value: rows are clamped to the arena, whose every row may be read; keys past a
  // query's limit are masked by selection and their values zeroed), so limits, queries, keys
  // and values of a short context arrive in one memory round trip.
  Frag kf[2][2], vf[4], kn[2][2], vn[4];
  Scales sc, scn;
  const int cfirst = kw * 32, cstep = kstep * 32;
  load_chunk(cfirst, a.cap - 1, kf, vf, sc);

  // this lane's queries: q0 + qt*16 + lq; limits and Q operands (pre-scaled by 1/sqrt(64)).
  // Nothing here waits for a loaded value before the last request is out: what is per sequence (first
  // row, source length) is read with scalar loads, and a lane without a query reads the row and the limit
  // of the clamped index min(q0 + qi, T - 1) -- rows below T exist for every sequence -- and discards
  // them, so that addresses never depend on the query count.  (Coherent queries keep the older form:
  // their row is the first one when the lane has no query.)
  int lim[NQT];
  bf16x8 qf[NQT][2];
  int kmax = 0;
  // the three per-sequence values first (one round trip together), then their uses; the query count is not
  // needed before every request is out (it only decides which lanes' results count)
  const int qcount = (nq < 0 && a.q_count) ? a.q_count[b] : a.T;
  const int qo = (QOFF && a.q_off) ? a.q_off[b] : 0;
  const int lseq = a.lim_row ? 0 : a.lim_seq[b];
  if constexpr (COHQ) {
    if (nq < 0) nq = min(qcount - q0, NQT * 16);
    nq = __builtin_amdgcn_readfirstlane(nq);
  }
  auto request = [&](const bf16* qbase, int lbase) {
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
      const int qi = qt * 16 + lq;
      int row;
      if constexpr (COHQ) {
        const bool ok = qi < nq;
        row = q0 + (ok ? qi : 0);
        lim[qt] = ok ? (a.lim_row ? a.lim_row[lbase + q0 + qi] : lseq) : 0;
      } else {
        row = min(q0 + qi, a.T - 1);
        lim[qt] = a.lim_row ? a.lim_row[lbase + row] : lseq;
      }
      const bf16* qp = qbase + (long)row * a.q_row + h * kHeadDim + g * 8;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) qf[qt][ks] = ld16<COHQ>(qp + ks * 32);
    }
  };
  // two copies of the requests, so that only the packed one (rows found through q_off) waits for a loaded value
  if (QOFF && a.q_off) request(a.q + (long)qo * a.q_row, qo);
  else request(a.q + b * a.q_b, b * a.T);
  if constexpr (!COHQ) {
    if (nq < 0) nq = min(qcount - q0, NQT * 16);
    nq = __builtin_amdgcn_readfirstlane(nq);
  }
  // The queries are needed where the limits are (same round trip): this use keeps their requests here,
  // ahead of the first wait, instead of letting them sink behind the branch around the key loop.
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) asm volatile("" : : "v"(qf[qt][0]), "v"(qf[qt][1]), "v"(lim[qt]));
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    if constexpr (!COHQ) lim[qt] = (qt * 16 + lq < nq) ? lim[qt] : 0;
    kmax = max(kmax, lim[qt]);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int e = 0; e < 8; ++e) qf[qt][ks][e] = (bf16)((float)qf[qt][ks][e] * 0.125f);   // exact: power of two
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
    if (more) load_chunk(c0 + cstep, kclamp, kn, vn, scn);
    // value operands of this chunk: the fetched registers themselves unless they hold codes
    bf16x8 vo8[KV8 ? 4 : 1];
    bf16x8(&vo)[4] = [&]() -> bf16x8(&)[4] {
      if constexpr (KV8) return vo8;
      else return vf;
    }();
    if constexpr (!VBLK) {
      // wave-private transposition: rows -> LDS -> (dim, 8 consecutive keys) operands
      // (LDS operations of one wave execute in order, so no barrier is needed; memcpy keeps
      // the 16-byte store and the 2-byte loads in one alias class for the compiler)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        __builtin_memcpy(&Vs[8 * i + (lane >> 3)][(lane & 7) * 8], &vf[i], 16);
#pragma unroll
      for (int et = 0; et < 4; ++et)
#pragma unroll
        for (int i = 0; i < 8; ++i) vo[et][i] = Vs[8 * g + i][et * 16 + lq];
    } else if constexpr (KV8) {
#pragma unroll
      for (int et = 0; et < 4; ++et) vo[et] = attn_operand(vf[et]);
    }
    if (c0 + 32 > kmax) {
      const int nvalid = kmax - (c0 + 8 * g);
#pragma unroll
      for (int et = 0; et < 4; ++et) vo[et] = zero_tail(vo[et], nvalid);
    }
    const bf16x8 ko00 = attn_operand(kf[0][0]), ko01 = attn_operand(kf[0][1]);
    const bf16x8 ko10 = attn_operand(kf[1][0]), ko11 = attn_operand(kf[1][1]);
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
      f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ko00, qf[qt][0], s0, 0, 0, 0);
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ko01, qf[qt][1], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ko10, qf[qt][0], s1, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ko11, qf[qt][1], s1, 0, 0, 0);
      if constexpr (KV8) {
#pragma unroll
        for (int r = 0; r < 4; ++r) { s0[r] *= sc.k[0][r]; s1[r] *= sc.k[1][r]; }
      }
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
        const bool on = any && s[r] > kNegInf;
        float p = on ? __expf(s[r] - mnew) : 0.f;
        ps += p;
        // (a masked key's scale may be anything, NaN included: it must not meet the 0)
        if constexpr (KV8) pf[r] = (bf16)(on ? p * sc.v[r >> 2][r & 3] : 0.f);
        else pf[r] = (bf16)p;
      }
      ps += __shfl_xor(ps, 16, 64);
      ps += __shfl_xor(ps, 32, 64);
      lrun[qt] = lrun[qt] * alpha + ps;
      mrun[qt] = mnew;
#pragma unroll
      for (int et = 0; et < 4; ++et) {
#pragma unroll
        for (int r = 0; r < 4; ++r) oacc[qt][et][r] *= alpha;
        oacc[qt][et] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vo[et], pf, oacc[qt][et], 0, 0, 0);
      }
    }
    if (more) {
#pragma unroll
      for (int t = 0; t < 2; ++t) { kf[t][0] = kn[t][0]; kf[t][1] = kn[t][1]; }
#pragma unroll
      for (int et = 0; et < 4; ++et) vf[et] = vn[et];
      sc = scn;
    }
  }
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) mfma_settle(oacc[qt]);
}

}  // namespace sd
